// Scheduling front-end (host code): Impact Estimator fits, Request Classifiers, Priority
// Regulator, Queue Manager and a one-server trace model, after Sections 3.3 - 3.6 of the
// paper.  See tcms.h for the contract of every entry point.
#include "../../include/tcms.h"

#include <algorithm>
#include <cmath>
#include <deque>
#include <limits>
#include <new>
#include <utility>
#include <vector>

namespace {

bool finite_all(const double* v, int64_t n) {
  for (int64_t i = 0; i < n; ++i)
    if (!std::isfinite(v[i])) return false;
  return true;
}

bool valid_regulator(const tcms_regulator* r) {
  if (!r) return false;
  for (int c = 0; c < 3; ++c) {
    if (!(r->static_priority[c] >= 0.0) || !(r->k[c] >= 0.0) || !(r->p[c] > 0.0)) return false;
    if (!std::isfinite(r->static_priority[c]) || !std::isfinite(r->k[c]) || !std::isfinite(r->p[c])) return false;
  }
  return true;
}

double priority_of(const tcms_regulator& r, int c, double wait) {
  if (wait < 0.0) wait = 0.0;
  return r.static_priority[c] + (1.0 - std::exp(-r.k[c] * std::pow(wait, r.p[c])));
}

double score_of(const tcms_regulator& r, int c, double wait) {
  const double pr = priority_of(r, c, wait);
  return pr <= 0.0 ? std::numeric_limits<double>::infinity() : -std::log(pr);
}

struct Waiting {
  int64_t id;
  double arrival;
  int64_t seq;   // push order, breaks ties between equal arrival times
};

// index of the class whose head is served next, or -1
int pick_class(const std::deque<Waiting> (&q)[3], const tcms_regulator& reg, int policy, double now) {
  int best = -1;
  double best_score = 0.0;
  for (int c = 0; c < 3; ++c) {
    if (q[c].empty()) continue;
    const Waiting& h = q[c].front();
    if (policy == TCMS_STATIC) return c;
    if (policy == TCMS_FCFS) {
      if (best < 0 || h.arrival < q[best].front().arrival ||
          (h.arrival == q[best].front().arrival && h.seq < q[best].front().seq))
        best = c;
    } else {
      const double s = score_of(reg, c, now - h.arrival);
      if (best < 0 || s < best_score || (s == best_score && h.seq < q[best].front().seq)) {
        best = c;
        best_score = s;
      }
    }
  }
  return best;
}

}  // namespace

struct tcms_queues {
  tcms_regulator reg;
  int policy;
  int64_t seq;
  std::deque<Waiting> q[3];
};

extern "C" {

int tcms_fit_linear(const double* x, const double* y, int64_t n, double* slope, double* intercept) {
  if (!x || !y || !slope || !intercept || n < 1 || !finite_all(x, n) || !finite_all(y, n)) return TCMS_E_INVALID_ARG;
  double xm = 0.0, ym = 0.0;
  for (int64_t i = 0; i < n; ++i) { xm += x[i]; ym += y[i]; }
  xm /= (double)n;
  ym /= (double)n;
  double sxx = 0.0, sxy = 0.0;
  for (int64_t i = 0; i < n; ++i) {
    sxx += (x[i] - xm) * (x[i] - xm);
    sxy += (x[i] - xm) * (y[i] - ym);
  }
  if (sxx == 0.0) {
    *slope = 0.0;
    *intercept = ym;
  } else {
    *slope = sxy / sxx;
    *intercept = ym - (sxy / sxx) * xm;
  }
  return TCMS_OK;
}

double tcms_pinball_loss(const double* x, const double* y, int64_t n, double q, double slope, double intercept) {
  if (!x || !y || n < 0) return std::numeric_limits<double>::quiet_NaN();
  double s = 0.0;
  for (int64_t i = 0; i < n; ++i) {
    const double r = y[i] - (intercept + slope * x[i]);
    s += r >= 0.0 ? q * r : (q - 1.0) * r;
  }
  return s;
}

int tcms_fit_quantile(const double* x, const double* y, int64_t n, double q, double* slope, double* intercept,
                      double* loss) {
  if (!x || !y || !slope || !intercept || n < 1 || !(q > 0.0 && q < 1.0) || !finite_all(x, n) || !finite_all(y, n))
    return TCMS_E_INVALID_ARG;
  double best_loss = std::numeric_limits<double>::infinity(), best_s = 0.0, best_i = 0.0;
  std::vector<std::pair<double, double>> bp;   // (slope to the other point, |dx|)
  bp.reserve((size_t)n);
  bool any_line = false;
  for (int64_t i = 0; i < n; ++i) {
    // best line through point i: the loss along the slope b is convex and piecewise linear with
    // breakpoints at the slopes to the other points; its derivative starts at g0 and rises by
    // |dx_j| at breakpoint j, the minimum is where it first reaches zero
    bp.clear();
    double g0 = 0.0;
    for (int64_t j = 0; j < n; ++j) {
      const double dx = x[j] - x[i];
      if (dx == 0.0) continue;
      bp.emplace_back((y[j] - y[i]) / dx, std::fabs(dx));
      g0 -= dx > 0.0 ? dx * q : -dx * (1.0 - q);
    }
    if (bp.empty()) continue;
    any_line = true;
    std::sort(bp.begin(), bp.end());
    double g = g0, b = bp.back().first;
    for (const auto& e : bp) {
      g += e.second;
      if (g >= 0.0) { b = e.first; break; }
    }
    const double a = y[i] - b * x[i];
    const double l = tcms_pinball_loss(x, y, n, q, b, a);
    if (l < best_loss) { best_loss = l; best_s = b; best_i = a; }
  }
  if (!any_line) {   // all x equal: a q-quantile of y
    std::vector<double> ys(y, y + n);
    std::sort(ys.begin(), ys.end());
    int64_t k = (int64_t)std::ceil(q * (double)n) - 1;
    k = std::min<int64_t>(std::max<int64_t>(k, 0), n - 1);
    best_s = 0.0;
    best_i = ys[(size_t)k];
    best_loss = tcms_pinball_loss(x, y, n, q, 0.0, best_i);
  }
  *slope = best_s;
  *intercept = best_i;
  if (loss) *loss = best_loss;
  return TCMS_OK;
}

namespace {
// centre and scale the two regressors (x2 reaches 1e9 for long videos); a constant column keeps scale 1
struct Scaled2 {
  std::vector<double> u, v;
  double m1 = 0.0, m2 = 0.0, s1 = 1.0, s2 = 1.0;
  Scaled2(const double* x1, const double* x2, int64_t n) : u((size_t)n), v((size_t)n) {
    for (int64_t i = 0; i < n; ++i) { m1 += x1[i]; m2 += x2[i]; }
    m1 /= (double)n;
    m2 /= (double)n;
    double q1 = 0.0, q2 = 0.0;
    for (int64_t i = 0; i < n; ++i) {
      q1 += (x1[i] - m1) * (x1[i] - m1);
      q2 += (x2[i] - m2) * (x2[i] - m2);
    }
    if (q1 > 0.0) s1 = std::sqrt(q1);
    if (q2 > 0.0) s2 = std::sqrt(q2);
    for (int64_t i = 0; i < n; ++i) {
      u[(size_t)i] = (x1[i] - m1) / s1;
      v[(size_t)i] = (x2[i] - m2) / s2;
    }
  }
  // coefficients of (1, u, v) -> coefficients of (1, x1, x2)
  void unscale(double a0, double a1, double a2, double* coef) const {
    coef[1] = a1 / s1;
    coef[2] = a2 / s2;
    coef[0] = a0 - coef[1] * m1 - coef[2] * m2;
  }
};
}  // namespace

int tcms_fit_linear2(const double* x1, const double* x2, const double* y, int64_t n, double* coef) {
  if (!x1 || !x2 || !y || !coef || n < 1 || !finite_all(x1, n) || !finite_all(x2, n) || !finite_all(y, n))
    return TCMS_E_INVALID_ARG;
  const Scaled2 z(x1, x2, n);
  double ym = 0.0;
  for (int64_t i = 0; i < n; ++i) ym += y[i];
  ym /= (double)n;
  double suu = 0.0, svv = 0.0, suv = 0.0, suy = 0.0, svy = 0.0;
  for (int64_t i = 0; i < n; ++i) {
    const double u = z.u[(size_t)i], v = z.v[(size_t)i], r = y[i] - ym;
    suu += u * u; svv += v * v; suv += u * v; suy += u * r; svy += v * r;
  }
  // the columns have unit length (or are zero): det = 1 - cos^2 of the angle between them
  const double det = suu * svv - suv * suv;
  double a1, a2;
  if (det > 1e-10) {
    a1 = (svv * suy - suv * svy) / det;
    a2 = (suu * svy - suv * suy) / det;
  } else if (suu > 0.0 && svv > 0.0) {   // proportional columns: the minimum-norm solution shares the slope
    a1 = 0.5 * suy;
    a2 = suv > 0.0 ? a1 : -a1;
  } else {                                // a constant column gets no weight
    a1 = suu > 0.0 ? suy : 0.0;
    a2 = svv > 0.0 ? svy : 0.0;
  }
  z.unscale(ym, a1, a2, coef);
  return TCMS_OK;
}

double tcms_pinball_loss2(const double* x1, const double* x2, const double* y, int64_t n, double q,
                          const double* coef) {
  if (!x1 || !x2 || !y || !coef || n < 0) return std::numeric_limits<double>::quiet_NaN();
  double s = 0.0;
  for (int64_t i = 0; i < n; ++i) {
    const double r = y[i] - (coef[0] + coef[1] * x1[i] + coef[2] * x2[i]);
    s += r >= 0.0 ? q * r : (q - 1.0) * r;
  }
  return s;
}

int tcms_fit_quantile2(const double* x1, const double* x2, const double* y, int64_t n, double q, double* coef,
                       double* loss) {
  if (!x1 || !x2 || !y || !coef || n < 1 || n > 4096 || !(q > 0.0 && q < 1.0) || !finite_all(x1, n) ||
      !finite_all(x2, n) || !finite_all(y, n))
    return TCMS_E_INVALID_ARG;
  const Scaled2 z(x1, x2, n);
  const std::vector<double>&u = z.u, &v = z.v;
  auto loss_of = [&](double a0, double a1, double a2) {
    double s = 0.0;
    for (int64_t k = 0; k < n; ++k) {
      const double r = y[k] - (a0 + a1 * u[(size_t)k] + a2 * v[(size_t)k]);
      s += r >= 0.0 ? q * r : (q - 1.0) * r;
    }
    return s;
  };
  double best = std::numeric_limits<double>::infinity(), b0 = 0.0, b1 = 0.0, b2 = 0.0;
  std::vector<std::pair<double, double>> bp;
  bp.reserve((size_t)n);
  // The optimum of the linear program is a plane through three data points.  For every pair of points with
  // different regressors, the planes through both form a one-parameter family (slope vector = p0 + t * nrm);
  // along t the loss is convex and piecewise linear with breakpoints where a third point falls on the plane,
  // and its derivative rises by |b_k| there: the best member is a weighted quantile, as in the one-regressor fit.
  for (int64_t i = 0; i < n; ++i) {
    for (int64_t j = i + 1; j < n; ++j) {
      const double du = u[(size_t)j] - u[(size_t)i], dv = v[(size_t)j] - v[(size_t)i];
      const double dd = du * du + dv * dv;
      if (dd == 0.0) continue;
      const double dy = y[j] - y[i];
      const double p0u = dy * du / dd, p0v = dy * dv / dd, nu = -dv, nv = du;
      bp.clear();
      double g = 0.0;
      for (int64_t k = 0; k < n; ++k) {
        const double eu = u[(size_t)k] - u[(size_t)i], ev = v[(size_t)k] - v[(size_t)i];
        const double b = nu * eu + nv * ev;
        if (b == 0.0) continue;
        const double a = (y[k] - y[i]) - (p0u * eu + p0v * ev);
        bp.emplace_back(a / b, std::fabs(b));
        g -= b > 0.0 ? b * q : -b * (1.0 - q);
      }
      double t = 0.0;
      if (!bp.empty()) {
        std::sort(bp.begin(), bp.end());
        t = bp.back().first;
        for (const auto& e : bp) {
          g += e.second;
          if (g >= 0.0) { t = e.first; break; }
        }
      }
      const double a1 = p0u + t * nu, a2 = p0v + t * nv;
      const double a0 = y[i] - a1 * u[(size_t)i] - a2 * v[(size_t)i];
      const double l = loss_of(a0, a1, a2);
      if (l < best) { best = l; b0 = a0; b1 = a1; b2 = a2; }
    }
  }
  if (!std::isfinite(best)) {   // every point has the same regressors: a q-quantile of y
    std::vector<double> ys(y, y + n);
    std::sort(ys.begin(), ys.end());
    int64_t k = (int64_t)std::ceil(q * (double)n) - 1;
    k = std::min<int64_t>(std::max<int64_t>(k, 0), n - 1);
    b0 = ys[(size_t)k];
    b1 = b2 = 0.0;
  }
  z.unscale(b0, b1, b2, coef);
  if (loss) *loss = tcms_pinball_loss2(x1, x2, y, n, q, coef);
  return TCMS_OK;
}

int tcms_classify_naive(int modality) {
  switch (modality) {
    case 0: return TCMS_MOTORCYCLE;
    case 1: return TCMS_CAR;
    case 2: return TCMS_TRUCK;
    default: return TCMS_E_INVALID_ARG;
  }
}

int tcms_cluster_fit(const double* features, int64_t n, int max_iter, tcms_cluster_model* out) {
  if (!features || !out || n < 3 || max_iter < 1 || !finite_all(features, 2 * n)) return TCMS_E_INVALID_ARG;
  for (int64_t i = 0; i < 2 * n; ++i)
    if (features[i] < 0.0) return TCMS_E_INVALID_ARG;
  std::vector<double> z((size_t)(2 * n));
  tcms_cluster_model m{};
  for (int f = 0; f < 2; ++f) {
    double mean = 0.0;
    for (int64_t i = 0; i < n; ++i) {
      z[(size_t)(2 * i + f)] = std::log1p(features[2 * i + f]);
      mean += z[(size_t)(2 * i + f)];
    }
    mean /= (double)n;
    double var = 0.0;
    for (int64_t i = 0; i < n; ++i) var += (z[(size_t)(2 * i + f)] - mean) * (z[(size_t)(2 * i + f)] - mean);
    double sd = std::sqrt(var / (double)n);
    if (!(sd > 0.0)) sd = 1.0;
    m.mean[f] = mean;
    m.scale[f] = sd;
    for (int64_t i = 0; i < n; ++i) z[(size_t)(2 * i + f)] = (z[(size_t)(2 * i + f)] - mean) / sd;
  }
  std::vector<int64_t> order((size_t)n);
  for (int64_t i = 0; i < n; ++i) order[(size_t)i] = i;
  std::stable_sort(order.begin(), order.end(),
                   [&](int64_t a, int64_t b) { return z[(size_t)(2 * a)] < z[(size_t)(2 * b)]; });
  double cent[3][2];
  for (int j = 0; j < 3; ++j) {
    const int64_t at = order[(size_t)std::min<int64_t>(n - 1, (2 * j + 1) * n / 6)];
    cent[j][0] = z[(size_t)(2 * at)];
    cent[j][1] = z[(size_t)(2 * at + 1)];
  }
  std::vector<int> assign((size_t)n, -1), fresh((size_t)n);
  for (int it = 0; it < max_iter; ++it) {
    bool same = true;
    for (int64_t i = 0; i < n; ++i) {
      int bj = 0;
      double bd = 0.0;
      for (int j = 0; j < 3; ++j) {
        const double d0 = z[(size_t)(2 * i)] - cent[j][0], d1 = z[(size_t)(2 * i + 1)] - cent[j][1];
        const double d = d0 * d0 + d1 * d1;
        if (j == 0 || d < bd) { bd = d; bj = j; }
      }
      fresh[(size_t)i] = bj;
      same = same && bj == assign[(size_t)i];
    }
    if (same) break;
    assign = fresh;
    for (int j = 0; j < 3; ++j) {
      double s0 = 0.0, s1 = 0.0;
      int64_t cnt = 0;
      for (int64_t i = 0; i < n; ++i)
        if (assign[(size_t)i] == j) { s0 += z[(size_t)(2 * i)]; s1 += z[(size_t)(2 * i + 1)]; ++cnt; }
      if (cnt) { cent[j][0] = s0 / (double)cnt; cent[j][1] = s1 / (double)cnt; }   // an empty cluster keeps its centroid
    }
  }
  int idx[3] = {0, 1, 2};
  std::stable_sort(idx, idx + 3, [&](int a, int b) { return cent[a][0] < cent[b][0]; });
  for (int j = 0; j < 3; ++j) { m.centroid[j][0] = cent[idx[j]][0]; m.centroid[j][1] = cent[idx[j]][1]; }
  *out = m;
  return TCMS_OK;
}

int tcms_cluster_assign(const tcms_cluster_model* m, double time, double tokens) {
  if (!m || !(time >= 0.0) || !(tokens >= 0.0) || !std::isfinite(time) || !std::isfinite(tokens)) return TCMS_E_INVALID_ARG;
  const double z0 = (std::log1p(time) - m->mean[0]) / m->scale[0], z1 = (std::log1p(tokens) - m->mean[1]) / m->scale[1];
  int bj = 0;
  double bd = 0.0;
  for (int j = 0; j < 3; ++j) {
    const double d0 = z0 - m->centroid[j][0], d1 = z1 - m->centroid[j][1];
    const double d = d0 * d0 + d1 * d1;
    if (j == 0 || d < bd) { bd = d; bj = j; }
  }
  return bj;
}

void tcms_regulator_default(tcms_regulator* r) {
  if (!r) return;
  const double st[3] = {0.1, 0.05, 0.0}, k[3] = {0.05, 0.003, 0.00075}, p[3] = {3.5, 2.5, 1.1};
  for (int c = 0; c < 3; ++c) { r->static_priority[c] = st[c]; r->k[c] = k[c]; r->p[c] = p[c]; }
}

double tcms_priority(const tcms_regulator* r, int cls, double wait) {
  if (!valid_regulator(r) || cls < 0 || cls > 2 || std::isnan(wait)) return std::numeric_limits<double>::quiet_NaN();
  return priority_of(*r, cls, wait);
}

double tcms_score(const tcms_regulator* r, int cls, double wait) {
  if (!valid_regulator(r) || cls < 0 || cls > 2 || std::isnan(wait)) return std::numeric_limits<double>::quiet_NaN();
  return score_of(*r, cls, wait);
}

tcms_queues* tcms_queues_create(const tcms_regulator* r, int policy) {
  if (!valid_regulator(r) || policy < TCMS_FCFS || policy > TCMS_REGULATED) return nullptr;
  tcms_queues* q = new (std::nothrow) tcms_queues();
  if (!q) return nullptr;
  q->reg = *r;
  q->policy = policy;
  q->seq = 0;
  return q;
}

void tcms_queues_destroy(tcms_queues* q) { delete q; }

int tcms_queues_push(tcms_queues* q, int64_t id, int cls, double arrival) {
  if (!q || cls < 0 || cls > 2 || !std::isfinite(arrival)) return TCMS_E_INVALID_ARG;
  if (!q->q[cls].empty() && arrival < q->q[cls].back().arrival) return TCMS_E_INVALID_ARG;
  try {
    q->q[cls].push_back(Waiting{id, arrival, q->seq++});
  } catch (...) {
    return TCMS_E_INVALID_ARG;
  }
  return TCMS_OK;
}

int tcms_queues_pop(tcms_queues* q, double now, int64_t* id, int* cls, double* arrival) {
  if (!q || !id || std::isnan(now)) return TCMS_E_INVALID_ARG;
  const int c = pick_class(q->q, q->reg, q->policy, now);
  if (c < 0) return TCMS_E_EMPTY;
  const Waiting w = q->q[c].front();
  q->q[c].pop_front();
  *id = w.id;
  if (cls) *cls = c;
  if (arrival) *arrival = w.arrival;
  return TCMS_OK;
}

int tcms_queues_stats(const tcms_queues* q, double now, int64_t length[3], double mean_wait[3]) {
  if (!q || !length || !mean_wait || std::isnan(now)) return TCMS_E_INVALID_ARG;
  for (int c = 0; c < 3; ++c) {
    length[c] = (int64_t)q->q[c].size();
    double s = 0.0;
    for (const Waiting& w : q->q[c]) s += now - w.arrival;
    mean_wait[c] = q->q[c].empty() ? 0.0 : s / (double)q->q[c].size();
  }
  return TCMS_OK;
}

int tcms_simulate(const tcms_regulator* r, int policy, int64_t n, const double* arrival, const double* service,
                  const int32_t* cls, double* start) {
  if (!valid_regulator(r) || policy < TCMS_FCFS || policy > TCMS_REGULATED || n < 0) return TCMS_E_INVALID_ARG;
  if (n == 0) return TCMS_OK;
  if (!arrival || !service || !cls || !start || !finite_all(arrival, n) || !finite_all(service, n)) return TCMS_E_INVALID_ARG;
  for (int64_t i = 0; i < n; ++i) {
    if (cls[i] < 0 || cls[i] > 2 || service[i] < 0.0) return TCMS_E_INVALID_ARG;
    if (i && arrival[i] < arrival[i - 1]) return TCMS_E_INVALID_ARG;
  }
  std::vector<double> st((size_t)n);
  std::deque<Waiting> q[3];
  int64_t nxt = 0, done = 0;
  double now = 0.0;
  try {
    while (done < n) {
      while (nxt < n && arrival[nxt] <= now) {
        q[cls[nxt]].push_back(Waiting{nxt, arrival[nxt], nxt});
        ++nxt;
      }
      const int c = pick_class(q, *r, policy, now);
      if (c < 0) {
        now = arrival[nxt];
        continue;
      }
      const Waiting w = q[c].front();
      q[c].pop_front();
      st[(size_t)w.id] = now;
      now += service[w.id];
      ++done;
    }
  } catch (...) {
    return TCMS_E_INVALID_ARG;
  }
  std::copy(st.begin(), st.end(), start);
  return TCMS_OK;
}

}  // extern "C"
