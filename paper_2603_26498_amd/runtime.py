"""Convenience layer over the C ABI: owns device memory through PyTorch (device
memory and streams only) and marshals arguments.  No arithmetic of the method
is done here; all of it runs in libtcmv.so."""
from __future__ import annotations

import ctypes as C
from typing import Dict, Optional, Sequence

import numpy as np
import torch

from . import binding as B


def _require_gpu():
    if not torch.cuda.is_available():
        raise RuntimeError("no GPU visible: the vision path has no CPU fallback")


def _stream_ptr(stream: Optional[torch.cuda.Stream] = None):
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


class Plan:
    def __init__(self, enc: "VisionEncoder", items, frame_tensors):
        self.enc = enc
        self.n_items = len(items)
        self._frames = frame_tensors          # keep device frames alive
        self.handle = B.tcmv_plan_create(enc.ctx, items)
        self.info = B.tcmv_plan_query(self.handle)
        self.cu_seqlens = B.tcmv_plan_cu_seqlens(self.handle, self.n_items)
        # device copy of the plan's index metadata: memory from PyTorch, copy enqueued by the library on the
        # current stream (stage calls on other streams must be ordered after it, see run_pipelined)
        self.meta = None
        if frame_tensors and self.info.meta_bytes:
            self.meta = torch.empty(int(self.info.meta_bytes), dtype=torch.uint8, device=enc.device)
            B.tcmv_plan_upload(enc.ctx, self.handle, self.meta, self.meta.numel(), _stream_ptr())

    def row_map(self, which):
        return B.tcmv_plan_row_map(self.handle, which)

    def close(self):
        if self.handle is not None:
            B.tcmv_plan_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class VisionEncoder:
    """desc: an object with the fields of tcmv_model_desc (e.g. workloads.ModelDesc).
    weights: dict name -> numpy fp32 array, linear weights [out, in]; may be None
    for plan-only (host) use."""

    def __init__(self, desc, weights: Optional[Dict[str, np.ndarray]] = None, device="cuda:0"):
        self.desc = desc
        # Sizes the kernels do not have are reached by zero padding at upload (a layout step: padded q/k
        # elements add nothing to a score, padded v columns and mlp units meet zero weights afterwards):
        # a bf16 head size outside {32, 64, 80, 96} goes to the next one up, with the true softmax scale
        # handed over; an mlp width that is not a multiple of 64 goes to the next multiple.
        self.dh = desc.d // desc.heads
        self.dh_lib, self.mlp_lib, attn_scale = 0, desc.mlp, 0.0
        if desc.dtype == "bf16":
            if self.dh not in (32, 64, 80, 96):
                fits = [h for h in (32, 64, 80, 96) if h >= self.dh]
                if not fits or getattr(desc, "pos", "none") == "rope2d":
                    raise ValueError(f"head size {self.dh} is not available on the bf16 path")
                self.dh_lib, attn_scale = fits[0], 1.0 / float(np.sqrt(self.dh))
            self.mlp_lib = (desc.mlp + 63) // 64 * 64
        self.cdesc = B.make_desc(dtype=desc.dtype, layers=desc.layers, d=desc.d, heads=desc.heads, mlp=self.mlp_lib,
                                 head_dim=self.dh_lib, attn_scale=attn_scale,
                                 patch=desc.patch, tpatch=desc.tpatch, merge=desc.merge, out_dim=desc.out_dim,
                                 use_cls=desc.use_cls, pos=desc.pos, max_pos=desc.max_pos, final_ln=desc.final_ln,
                                 ln_eps=desc.ln_eps, mean=desc.mean, std=desc.std,
                                 norm=getattr(desc, "norm", "layer"), gated=getattr(desc, "gated", 0),
                                 window=getattr(desc, "window", 0), full_every=getattr(desc, "full_every", 0),
                                 rope_theta=getattr(desc, "rope_theta", 10000.0))
        self.ctx = B.tcmv_create(self.cdesc)
        self.k_pad = B.tcmv_k_pad(self.cdesc)
        self.device = device
        self.bf16 = desc.dtype == "bf16"
        self._w = {}
        self._layer_arr = None
        if weights is not None:
            self.set_weights(weights)

    # -- parameters ---------------------------------------------------------------------------
    def _mat(self, a: np.ndarray, pad_to: int = 0) -> torch.Tensor:
        t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
        if pad_to and t.shape[1] < pad_to:
            t = torch.nn.functional.pad(t, (0, pad_to - t.shape[1]))
        t = t.to(self.device)
        return (t.to(torch.bfloat16) if self.bf16 else t).contiguous()

    def _vec(self, a: np.ndarray) -> torch.Tensor:
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(self.device).contiguous()

    def _lib_layout(self, name: str, a: np.ndarray) -> np.ndarray:
        """One layer parameter in the layout the library takes it in (padding and interleaving only)."""
        d = self.desc
        pad_rows = lambda x, n: np.concatenate([x, np.zeros((n - x.shape[0],) + x.shape[1:], x.dtype)], 0) if n > x.shape[0] else x
        if self.dh_lib and name in ("w_qkv", "b_qkv"):
            # [3, heads, dh, ...] -> [3, heads, dh_lib, ...] with zero rows behind every head
            x = a.reshape((3, d.heads, self.dh) + a.shape[1:])
            z = np.zeros((3, d.heads, self.dh_lib - self.dh) + a.shape[1:], a.dtype)
            return np.concatenate([x, z], 2).reshape((3 * d.heads * self.dh_lib,) + a.shape[1:])
        if self.dh_lib and name == "w_o":
            x = a.reshape(a.shape[0], d.heads, self.dh)
            z = np.zeros((a.shape[0], d.heads, self.dh_lib - self.dh), a.dtype)
            return np.concatenate([x, z], 2).reshape(a.shape[0], d.heads * self.dh_lib)
        if name in ("w_1", "b_1"):
            if getattr(d, "gated", 0):
                # gate and up rows interleaved (the caller's array has the gate rows first, then the up rows)
                g, u = pad_rows(a[:d.mlp], self.mlp_lib), pad_rows(a[d.mlp:], self.mlp_lib)
                return np.stack([g, u], axis=1).reshape((2 * self.mlp_lib,) + a.shape[1:])
            return pad_rows(a, self.mlp_lib)
        if name == "w_2" and self.mlp_lib > d.mlp:
            return np.concatenate([a, np.zeros((a.shape[0], self.mlp_lib - d.mlp), a.dtype)], 1)
        return a

    def set_weights(self, w: Dict[str, np.ndarray]):
        _require_gpu()
        d = self.desc
        T = self._w
        T["w_pe"] = self._mat(w["w_pe"], self.k_pad)
        T["b_pe"] = self._vec(w["b_pe"])
        for n in ("cls", "pos0", "pos1", "lnf_g", "lnf_b", "lnm_g", "lnm_b", "b_m1", "b_m2"):
            if n in w:
                T[n] = self._vec(w[n])
        for n in ("w_m1", "w_m2"):
            if n in w:
                T[n] = self._mat(w[n])
        arr = (C.c_void_p * max(1, d.layers * 12))()
        for l in range(d.layers):
            for j, name in enumerate(B.LAYER_FIELDS):
                key = f"l{l}.{name}"
                a = self._lib_layout(name, w[key])
                T[key] = self._mat(a) if name.startswith("w_") else self._vec(a)
                arr[l * 12 + j] = T[key].data_ptr()
        self._layer_arr = arr
        cw = B.tcmv_weights()
        for n in ("w_pe", "b_pe", "cls", "pos0", "pos1", "lnf_g", "lnf_b", "lnm_g", "lnm_b", "w_m1", "b_m1", "w_m2",
                  "b_m2"):
            setattr(cw, n, T[n].data_ptr() if n in T else None)
        cw.layer = C.cast(arr, C.POINTER(C.c_void_p))
        B.tcmv_set_weights(self.ctx, cw)

    # -- requests -----------------------------------------------------------------------------
    def plan(self, items: Sequence, upload: bool = True) -> Plan:
        """items: objects with modality, n_frames, src_h, src_w, dst_h, dst_w, frames (numpy uint8 or None)."""
        rows, keep = [], []
        for it in items:
            ptr = None
            if it.n_frames > 0 and upload:
                _require_gpu()
                t = torch.from_numpy(np.ascontiguousarray(it.frames)).to(self.device)
                keep.append(t)
                ptr = t.data_ptr()
            rows.append((it.modality, it.n_frames, it.src_h, it.src_w, it.dst_h, it.dst_w, ptr))
        return Plan(self, rows, keep)

    def preprocess(self, plan: Plan, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        _require_gpu()
        i = plan.info
        if out is None:
            out = torch.empty((i.n_patch_rows, i.k_pad), dtype=torch.bfloat16 if self.bf16 else torch.float32,
                              device=self.device)
        B.tcmv_preprocess(self.ctx, plan.handle, plan.meta, out, _stream_ptr())
        return out

    def workspace(self, nbytes: int) -> torch.Tensor:
        return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=self.device)

    def encode(self, plan: Plan, patches: torch.Tensor, hidden: Optional[torch.Tensor] = None,
               workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
        _require_gpu()
        i = plan.info
        if hidden is None:
            hidden = torch.empty((i.n_tokens, self.desc.d), dtype=torch.float32, device=self.device)
        if workspace is None:
            workspace = self.workspace(i.encode_workspace_bytes)
        B.tcmv_encode(self.ctx, plan.handle, plan.meta, patches, hidden, workspace, workspace.numel(), _stream_ptr())
        return hidden

    def merge_project(self, plan: Plan, hidden: torch.Tensor, out: Optional[torch.Tensor] = None,
                      workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
        _require_gpu()
        i = plan.info
        if out is None:
            out = torch.empty((i.n_out_tokens, self.desc.out_dim),
                              dtype=torch.bfloat16 if self.bf16 else torch.float32, device=self.device)
        if workspace is None:
            workspace = self.workspace(i.merge_workspace_bytes)
        B.tcmv_merge_project(self.ctx, plan.handle, hidden, out, workspace, workspace.numel(), _stream_ptr())
        return out

    def run(self, plan: Plan) -> torch.Tensor:
        """preprocess -> encode -> merge/project (when the model has a projector) on the current stream."""
        hidden = self.encode(plan, self.preprocess(plan))
        return self.merge_project(plan, hidden) if self.desc.out_dim else hidden

    def run_pipelined(self, plans: Sequence[Plan], side_stream: Optional[torch.cuda.Stream] = None):
        """Runs the plans in order; the preprocessing of plan i+1 is enqueued on a second
        stream (same priority) so that it overlaps the encoding of plan i (preprocess and
        encode are separate stages of a request, Sec. 2.1).  Only stream and event plumbing
        lives here; results are identical to calling run() plan by plan."""
        _require_gpu()
        main = torch.cuda.current_stream()
        side = side_stream if side_stream is not None else torch.cuda.Stream(device=self.device)
        side.wait_stream(main)
        patches = [None] * len(plans)
        ready = [torch.cuda.Event() for _ in plans]

        def stage(i):
            with torch.cuda.stream(side):
                patches[i] = self.preprocess(plans[i])
                ready[i].record(side)
            patches[i].record_stream(main)

        outs = []
        if plans:
            stage(0)
        for i, plan in enumerate(plans):
            if i + 1 < len(plans):
                stage(i + 1)
            main.wait_event(ready[i])
            hidden = self.encode(plan, patches[i])
            outs.append(self.merge_project(plan, hidden) if self.desc.out_dim else hidden)
            patches[i] = None
        return outs

    def close(self):
        if self.ctx is not None:
            B.tcmv_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
