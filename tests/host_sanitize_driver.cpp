// Exercises the host-only part of the library (descriptions, plans, index maps, attention index data, the
// scheduling front-end) on seeded random inputs.  The test that builds it compiles the library's host code with
// AddressSanitizer and UndefinedBehaviorSanitizer: any out-of-bounds access, overflow or leak ends the run with a
// non-zero status.  It launches nothing on a GPU and needs none.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>
#include "../include/tcmv.h"
#include "../include/tcms.h"

namespace {
uint64_t g_state = 0x9E3779B97F4A7C15ull;
uint32_t rnd() {                                   // splitmix64, upper half
  uint64_t z = (g_state += 0x9E3779B97F4A7C15ull);
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return (uint32_t)((z ^ (z >> 31)) >> 32);
}
int rint_in(int lo, int hi) { return lo + (int)(rnd() % (uint32_t)(hi - lo + 1)); }
double runif() { return (rnd() + 0.5) / 4294967296.0; }

int g_fail = 0;
#define EXPECT(c) do { if (!(c)) { std::printf("FAILED %s:%d: %s\n", __FILE__, __LINE__, #c); ++g_fail; } } while (0)

tcmv_model_desc base_desc(int dtype) {
  tcmv_model_desc d;
  std::memset(&d, 0, sizeof d);
  d.dtype = dtype; d.layers = 2; d.d = 128; d.heads = 2; d.mlp = 256; d.patch = 14; d.tpatch = 1; d.merge = 1;
  d.ln_eps = 1e-6f;
  for (int c = 0; c < 3; ++c) { d.mean[c] = 0.5f; d.std[c] = 0.25f; }
  return d;
}

// Reads every byte / entry the plan exposes, so that a size the library reports too large is an out-of-bounds read.
void walk_plan(const tcmv_plan* p, int n_items) {
  tcmv_plan_info info;
  EXPECT(tcmv_plan_query(p, &info) == 0);
  size_t bytes = 0;
  const unsigned char* meta = (const unsigned char*)tcmv_plan_meta(p, &bytes);
  EXPECT(bytes == info.meta_bytes);
  unsigned sum = 0;
  for (size_t i = 0; i < bytes; ++i) sum += meta[i];
  const int64_t* cu = tcmv_plan_cu_seqlens(p);
  EXPECT(cu != nullptr && cu[0] == 0 && cu[n_items] == info.n_tokens);
  for (int i = 0; i < n_items; ++i) EXPECT(cu[i] <= cu[i + 1]);
  for (int which = 0; which < 3; ++which) {
    const int32_t* m = nullptr;
    const int64_t n = tcmv_plan_row_map(p, which, &m);
    EXPECT(n == info.n_patch_rows);
    for (int64_t i = 0; i < n; ++i) {
      sum += (unsigned)m[i];
      if (which == 1) EXPECT(m[i] >= 0 && m[i] < info.n_tokens);
    }
  }
  const int32_t* m = nullptr;
  EXPECT(tcmv_plan_row_map(p, 3, &m) < 0);
  if (sum == 0xFFFFFFFFu) std::printf(" ");      // keeps the reads alive
}

void plans() {
  struct Variant { const char* name; tcmv_model_desc d; } v[6];
  int nv = 0;
  { Variant a = {"bf16 cls learned-1d", base_desc(TCMV_BF16)}; a.d.use_cls = 1; a.d.pos = TCMV_POS_LEARNED_1D; a.d.max_pos = 600; a.d.final_ln = 1; v[nv++] = a; }
  { Variant a = {"f32 cls learned-1d", base_desc(TCMV_F32)}; a.d.use_cls = 1; a.d.pos = TCMV_POS_LEARNED_1D; a.d.max_pos = 600; v[nv++] = a; }
  { Variant a = {"bf16 merge separable-2d", base_desc(TCMV_BF16)}; a.d.tpatch = 2; a.d.merge = 2; a.d.out_dim = 64; a.d.pos = TCMV_POS_SEPARABLE_2D; a.d.max_pos = 64; a.d.d = 320; a.d.heads = 4; a.d.mlp = 640; v[nv++] = a; }
  { Variant a = {"bf16 windows rotary rms gated", base_desc(TCMV_BF16)}; a.d.tpatch = 2; a.d.merge = 2; a.d.out_dim = 64; a.d.pos = TCMV_POS_ROTARY_2D; a.d.rope_theta = 10000.f; a.d.norm = TCMV_NORM_RMS; a.d.mlp_gated = 1; a.d.window = 8; a.d.full_every = 2; a.d.d = 320; a.d.heads = 4; a.d.mlp = 640; v[nv++] = a; }
  { Variant a = {"bf16 windows only", base_desc(TCMV_BF16)}; a.d.merge = 2; a.d.out_dim = 32; a.d.window = 4; a.d.pos = TCMV_POS_ROTARY_2D; a.d.rope_theta = 10000.f; v[nv++] = a; }
  { Variant a = {"bf16 padded heads", base_desc(TCMV_BF16)}; a.d.merge = 2; a.d.out_dim = 32; a.d.d = 192; a.d.heads = 2; a.d.head_dim = 96; a.d.attn_scale = 0.1f; a.d.mlp = 256; v[nv++] = a; }
  for (int i = 0; i < nv; ++i) {
    tcmv_ctx* ctx = nullptr;
    const int rc = tcmv_create(&v[i].d, &ctx);
    if (rc != 0) { std::printf("create(%s) -> %d (%s)\n", v[i].name, rc, tcmv_last_error(nullptr)); EXPECT(rc == 0); continue; }
    EXPECT(tcmv_k_pad(&v[i].d) >= (int64_t)3 * v[i].d.patch * v[i].d.patch * v[i].d.tpatch);
    const int step = v[i].d.patch * v[i].d.merge;
    int good = 0, bad = 0;
    for (int trial = 0; trial < 60; ++trial) {
      const int n_items = rint_in(0, 9);
      std::vector<tcmv_item> items((size_t)n_items);
      bool ok = true;
      for (auto& it : items) {
        std::memset(&it, 0, sizeof it);
        const int kind = rint_in(0, 9);
        it.modality = kind == 0 ? TCMV_TEXT : (kind < 7 ? TCMV_IMAGE : TCMV_VIDEO);
        if (it.modality == TCMV_TEXT) continue;
        it.n_frames = it.modality == TCMV_IMAGE ? 1 : v[i].d.tpatch * rint_in(1, 4);
        const int gmax = v[i].d.pos == TCMV_POS_LEARNED_1D ? 24 : 20;
        it.dst_h = step * rint_in(1, gmax / v[i].d.merge);
        it.dst_w = step * rint_in(1, gmax / v[i].d.merge);
        if (rint_in(0, 2) == 0) { it.src_h = rint_in(1, 700); it.src_w = rint_in(1, 700); }
        else { it.src_h = it.dst_h; it.src_w = it.dst_w; }
        it.d_frames = reinterpret_cast<const uint8_t*>(uintptr_t(0x1000) * (uintptr_t)rint_in(1, 1000));   // recorded, never read
        if (rint_in(0, 24) == 0) {                       // one of the documented shape errors
          switch (rint_in(0, 3)) {
            case 0: it.dst_h += 1; break;
            case 1: it.dst_w = 0; break;
            case 2: it.src_h = 0; break;
            default: it.dst_h = step * 300; break;       // grid side above 255
          }
          ok = false;
        }
        if (v[i].d.pos == TCMV_POS_LEARNED_1D && ok) {
          const int64_t rows = (int64_t)(it.dst_h / step) * (it.dst_w / step) * (it.n_frames / v[i].d.tpatch) + v[i].d.use_cls;
          if (rows > v[i].d.max_pos) ok = false;
        }
      }
      tcmv_plan* p = nullptr;
      const int prc = tcmv_plan_create(ctx, items.data(), n_items, &p);
      if (ok) {
        if (prc != 0) std::printf("%s: plan_create -> %d (%s)\n", v[i].name, prc, tcmv_last_error(ctx));
        EXPECT(prc == 0);
      } else {
        EXPECT(prc != 0 && p == nullptr);
      }
      if (prc == 0) { walk_plan(p, n_items); tcmv_plan_destroy(p); ++good; } else ++bad;
    }
    std::printf("%-32s %d plans walked, %d rejected\n", v[i].name, good, bad);
    tcmv_destroy(ctx);
  }
}

void attention_index() {
  for (int trial = 0; trial < 40; ++trial) {
    const int heads = rint_in(1, 4), dh = (int[]){32, 64, 80, 96}[rint_in(0, 3)], d = heads * dh;
    const int n_seg = rint_in(0, 12);
    std::vector<int64_t> cu((size_t)n_seg + 1, 0);
    for (int i = 0; i < n_seg; ++i) cu[(size_t)i + 1] = cu[(size_t)i] + (rint_in(0, 5) == 0 ? 0 : rint_in(1, 1500));
    for (int dtype = 0; dtype < 2; ++dtype) {
      if (dtype == TCMV_F32 && dh == 80) continue;
      const size_t ib = tcmv_op_attention_index_bytes(dtype, cu.data(), n_seg, d, heads);
      const size_t wb = tcmv_op_attention_workspace(dtype, cu.data(), n_seg, d, heads);
      (void)wb;
      if (ib == 0) continue;
      std::vector<unsigned char> buf(ib);                // exactly as large as reported
      EXPECT(tcmv_op_attention_index(dtype, cu.data(), n_seg, d, heads, buf.data(), ib) == 0);
      if (ib > 16) EXPECT(tcmv_op_attention_index(dtype, cu.data(), n_seg, d, heads, buf.data(), ib - 16) != 0);
    }
  }
  std::printf("attention index data: done\n");
}

void scheduler() {
  tcms_regulator reg;
  tcms_regulator_default(&reg);
  for (int trial = 0; trial < 30; ++trial) {
    const int64_t n = trial < 4 ? trial : rint_in(3, 400);
    std::vector<double> x1((size_t)n), x2((size_t)n), y((size_t)n), arr((size_t)n), svc((size_t)n), start((size_t)n), feat((size_t)n * 2);
    std::vector<int32_t> cls((size_t)n);
    double t = 0;
    const int shape = rint_in(0, 3);
    for (int64_t i = 0; i < n; ++i) {
      const size_t k = (size_t)i;
      x1[k] = shape == 1 ? 7.0 : std::floor(runif() * 4000);
      x2[k] = shape == 2 ? 3.0 * x1[k] : (shape == 3 ? 0.0 : x1[k] * x1[k] * runif());
      y[k] = 1e-3 * x1[k] + 1e-7 * x2[k] + runif();
      t += runif() * 0.05; arr[k] = t; svc[k] = runif() * 0.04; cls[k] = rint_in(0, 2);
      feat[2 * k] = y[k]; feat[2 * k + 1] = x1[k];
    }
    double s, b, loss, c[3];
    const int e1 = tcms_fit_linear(x1.data(), y.data(), n, &s, &b);
    EXPECT((n >= 1) == (e1 == 0));
    const int e2 = tcms_fit_quantile(x1.data(), y.data(), n, 0.9, &s, &b, &loss);
    if (e2 == 0) EXPECT(std::fabs(tcms_pinball_loss(x1.data(), y.data(), n, 0.9, s, b) - loss) <= 1e-9 * (1 + loss));
    (void)tcms_fit_linear2(x1.data(), x2.data(), y.data(), n, c);
    if (n <= 120) {
      const int e3 = tcms_fit_quantile2(x1.data(), x2.data(), y.data(), n, 0.9, c, &loss);
      if (e3 == 0) EXPECT(std::fabs(tcms_pinball_loss2(x1.data(), x2.data(), y.data(), n, 0.9, c) - loss) <= 1e-9 * (1 + loss));
    }
    EXPECT(tcms_fit_quantile(x1.data(), y.data(), n, 1.5, &s, &b, nullptr) != 0);
    tcms_cluster_model cm;
    if (tcms_cluster_fit(feat.data(), n, 50, &cm) == 0)
      for (int64_t i = 0; i < n; ++i) { const int k = tcms_cluster_assign(&cm, feat[2 * (size_t)i], feat[2 * (size_t)i + 1]); EXPECT(k >= 0 && k <= 2); }
    for (int policy = 0; policy < 3; ++policy) {
      EXPECT(tcms_simulate(&reg, policy, n, arr.data(), svc.data(), cls.data(), start.data()) == 0 || n == 0);
      for (int64_t i = 0; i < n; ++i) EXPECT(start[(size_t)i] >= arr[(size_t)i]);
      tcms_queues* q = tcms_queues_create(&reg, policy);
      EXPECT(q != nullptr);
      int64_t pushed = 0, popped = 0, id, len[3]; int pc; double pa, mw[3];
      for (int64_t i = 0; i < n; ++i) {
        EXPECT(tcms_queues_push(q, i, cls[(size_t)i], arr[(size_t)i]) == 0); ++pushed;
        if (rint_in(0, 2) == 0 && tcms_queues_pop(q, arr[(size_t)i], &id, &pc, &pa) == 0) { ++popped; EXPECT(id >= 0 && id <= i); }
        if ((i & 63) == 0) EXPECT(tcms_queues_stats(q, arr[(size_t)i], len, mw) == 0);
      }
      while (tcms_queues_pop(q, t + 1, &id, &pc, &pa) == 0) ++popped;
      EXPECT(pushed == popped);
      EXPECT(tcms_queues_pop(q, t + 2, &id, &pc, &pa) == TCMS_E_EMPTY);
      tcms_queues_destroy(q);
    }
  }
  EXPECT(tcms_queues_create(&reg, 7) == nullptr);
  EXPECT(tcms_classify_naive(3) < 0 && tcms_classify_naive(2) == TCMS_TRUCK);
  EXPECT(std::isinf(tcms_score(&reg, 2, 0.0)) || tcms_score(&reg, 2, 0.0) > 0);
  std::printf("scheduling front-end: done\n");
}
}  // namespace

int main(int argc, char** argv) {
  if (argc > 1) g_state ^= std::strtoull(argv[1], nullptr, 10) * 0xD1B54A32D192ED03ull;
  EXPECT(tcmv_version() >= 200);
  plans();
  attention_index();
  scheduler();
  std::printf(g_fail ? "%d expectation(s) failed\n" : "all expectations held\n", g_fail);
  return g_fail ? 1 : 0;
}
