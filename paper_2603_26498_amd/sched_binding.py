"""ctypes binding of the scheduling front-end in libtcmv.so: same names as
include/tcms.h, argument marshalling only (numpy arrays in, numbers out)."""
from __future__ import annotations

import ctypes as C

import numpy as np

from . import binding as _B

TCMS_MOTORCYCLE, TCMS_CAR, TCMS_TRUCK = 0, 1, 2
TCMS_FCFS, TCMS_STATIC, TCMS_REGULATED = 0, 1, 2
TCMS_OK, TCMS_E_INVALID_ARG, TCMS_E_EMPTY, TCMS_E_DEGENERATE = 0, -1, -2, -3

_D = C.POINTER(C.c_double)


class tcms_cluster_model(C.Structure):
    _fields_ = [("mean", C.c_double * 2), ("scale", C.c_double * 2), ("centroid", (C.c_double * 2) * 3)]


class tcms_regulator(C.Structure):
    _fields_ = [("static_priority", C.c_double * 3), ("k", C.c_double * 3), ("p", C.c_double * 3)]


class TcmsError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__(f"{where}: error {code}")


# name -> (restype, argtypes); the list of symbols include/tcms.h declares
SIGNATURES = {
    "tcms_fit_linear": (C.c_int, [_D, _D, C.c_int64, _D, _D]),
    "tcms_pinball_loss": (C.c_double, [_D, _D, C.c_int64, C.c_double, C.c_double, C.c_double]),
    "tcms_fit_quantile": (C.c_int, [_D, _D, C.c_int64, C.c_double, _D, _D, _D]),
    "tcms_fit_linear2": (C.c_int, [_D, _D, _D, C.c_int64, _D]),
    "tcms_pinball_loss2": (C.c_double, [_D, _D, _D, C.c_int64, C.c_double, _D]),
    "tcms_fit_quantile2": (C.c_int, [_D, _D, _D, C.c_int64, C.c_double, _D, _D]),
    "tcms_classify_naive": (C.c_int, [C.c_int]),
    "tcms_cluster_fit": (C.c_int, [_D, C.c_int64, C.c_int, C.POINTER(tcms_cluster_model)]),
    "tcms_cluster_assign": (C.c_int, [C.POINTER(tcms_cluster_model), C.c_double, C.c_double]),
    "tcms_regulator_default": (None, [C.POINTER(tcms_regulator)]),
    "tcms_priority": (C.c_double, [C.POINTER(tcms_regulator), C.c_int, C.c_double]),
    "tcms_score": (C.c_double, [C.POINTER(tcms_regulator), C.c_int, C.c_double]),
    "tcms_queues_create": (C.c_void_p, [C.POINTER(tcms_regulator), C.c_int]),
    "tcms_queues_destroy": (None, [C.c_void_p]),
    "tcms_queues_push": (C.c_int, [C.c_void_p, C.c_int64, C.c_int, C.c_double]),
    "tcms_queues_pop": (C.c_int, [C.c_void_p, C.c_double, C.POINTER(C.c_int64), C.POINTER(C.c_int), _D]),
    "tcms_queues_stats": (C.c_int, [C.c_void_p, C.c_double, C.POINTER(C.c_int64), _D]),
    "tcms_simulate": (C.c_int, [C.POINTER(tcms_regulator), C.c_int, C.c_int64, _D, _D, C.POINTER(C.c_int32), _D]),
}

_ready = False


def lib():
    global _ready
    l = _B.lib()
    if not _ready:
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(l, name)
            fn.restype = res
            fn.argtypes = args
        _ready = True
    return l


def _arr(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(_D)


def _check(rc, where):
    if rc != TCMS_OK:
        raise TcmsError(rc, where)


def tcms_fit_linear(x, y):
    x, px = _arr(x)
    y, py = _arr(y)
    s, i = C.c_double(), C.c_double()
    _check(lib().tcms_fit_linear(px, py, len(x), C.byref(s), C.byref(i)), "tcms_fit_linear")
    return s.value, i.value


def tcms_pinball_loss(x, y, q, slope, intercept):
    x, px = _arr(x)
    y, py = _arr(y)
    return lib().tcms_pinball_loss(px, py, len(x), q, slope, intercept)


def tcms_fit_quantile(x, y, q):
    x, px = _arr(x)
    y, py = _arr(y)
    s, i, l = C.c_double(), C.c_double(), C.c_double()
    _check(lib().tcms_fit_quantile(px, py, len(x), q, C.byref(s), C.byref(i), C.byref(l)), "tcms_fit_quantile")
    return s.value, i.value, l.value


def tcms_fit_linear2(x1, x2, y):
    x1, p1 = _arr(x1)
    x2, p2 = _arr(x2)
    y, py = _arr(y)
    coef = (C.c_double * 3)()
    _check(lib().tcms_fit_linear2(p1, p2, py, len(y), coef), "tcms_fit_linear2")
    return tuple(coef)


def tcms_pinball_loss2(x1, x2, y, q, coef):
    x1, p1 = _arr(x1)
    x2, p2 = _arr(x2)
    y, py = _arr(y)
    return lib().tcms_pinball_loss2(p1, p2, py, len(y), q, (C.c_double * 3)(*coef))


def tcms_fit_quantile2(x1, x2, y, q):
    x1, p1 = _arr(x1)
    x2, p2 = _arr(x2)
    y, py = _arr(y)
    coef = (C.c_double * 3)()
    l = C.c_double()
    _check(lib().tcms_fit_quantile2(p1, p2, py, len(y), q, coef, C.byref(l)), "tcms_fit_quantile2")
    return tuple(coef), l.value


def tcms_classify_naive(modality):
    r = lib().tcms_classify_naive(int(modality))
    if r < 0:
        raise TcmsError(r, "tcms_classify_naive")
    return r


def tcms_cluster_fit(features, max_iter=100):
    f, pf = _arr(features)
    m = tcms_cluster_model()
    _check(lib().tcms_cluster_fit(pf, f.shape[0], max_iter, C.byref(m)), "tcms_cluster_fit")
    return m


def tcms_cluster_assign(model, time, tokens):
    r = lib().tcms_cluster_assign(C.byref(model), float(time), float(tokens))
    if r < 0:
        raise TcmsError(r, "tcms_cluster_assign")
    return r


def tcms_regulator_default():
    r = tcms_regulator()
    lib().tcms_regulator_default(C.byref(r))
    return r


def make_regulator(static, k, p):
    r = tcms_regulator()
    for c in range(3):
        r.static_priority[c], r.k[c], r.p[c] = static[c], k[c], p[c]
    return r


def tcms_priority(reg, cls, wait):
    return lib().tcms_priority(C.byref(reg), int(cls), float(wait))


def tcms_score(reg, cls, wait):
    return lib().tcms_score(C.byref(reg), int(cls), float(wait))


def tcms_queues_create(reg, policy):
    q = lib().tcms_queues_create(C.byref(reg), int(policy))
    if not q:
        raise TcmsError(TCMS_E_INVALID_ARG, "tcms_queues_create")
    return q


def tcms_queues_destroy(q):
    lib().tcms_queues_destroy(q)


def tcms_queues_push(q, rid, cls, arrival):
    _check(lib().tcms_queues_push(q, int(rid), int(cls), float(arrival)), "tcms_queues_push")


def tcms_queues_pop(q, now):
    """(id, class, arrival) of the request to serve next, or None when nothing waits."""
    rid, cls, arr = C.c_int64(), C.c_int(), C.c_double()
    rc = lib().tcms_queues_pop(q, float(now), C.byref(rid), C.byref(cls), C.byref(arr))
    if rc == TCMS_E_EMPTY:
        return None
    _check(rc, "tcms_queues_pop")
    return rid.value, cls.value, arr.value


def tcms_queues_stats(q, now):
    ln = (C.c_int64 * 3)()
    mw = (C.c_double * 3)()
    _check(lib().tcms_queues_stats(q, float(now), ln, mw), "tcms_queues_stats")
    return list(ln), list(mw)


def tcms_simulate(reg, policy, arrival, service, cls):
    a, pa = _arr(arrival)
    s, ps = _arr(service)
    c = np.ascontiguousarray(cls, dtype=np.int32)
    st = np.empty(len(a), np.float64)
    _check(lib().tcms_simulate(C.byref(reg), int(policy), len(a), pa, ps, c.ctypes.data_as(C.POINTER(C.c_int32)),
                               st.ctypes.data_as(_D)), "tcms_simulate")
    return st
