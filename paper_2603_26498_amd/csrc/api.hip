// Host side of the C ABI declared in include/tcmv.h: context, plan construction
// (pure host logic), workspace carving and the sequence of kernel launches that
// makes up each stage.  No arithmetic of the method happens here.
#include "../../include/tcmv.h"
#include "tcmv_internal.h"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

using namespace tcmv;

struct tcmv_ctx {
  tcmv_model_desc desc;
  int64_t k, k_pad;
  bool has_weights = false;
  tcmv_weights w;
  std::vector<const void*> layer;   // layers*12 device pointers (copied)
  std::string err;
  // per-kernel timing
  unsigned profile_mask = 0;         // bit c set: launches of kernel class c are bracketed with events
  struct Span { hipEvent_t a, b; int cat; };
  std::vector<Span> spans;          // recorded, not yet read
  std::vector<Span> free_spans;     // event pairs ready for reuse
};

struct tcmv_plan {
  tcmv_ctx* ctx;
  std::vector<ItemDev> items;
  std::vector<int64_t> cu;            // n_items + 1
  std::vector<int32_t> prow_item, prow_thw, prow_dst, prow_pos;
  std::vector<int32_t> row_vcol;      // hidden row -> column in the transposed-V buffer
  std::vector<int32_t> cls_rows;
  std::vector<AttnWork> work;
  // windowed layers: the windows are the attention segments (own work list and transposed-V columns)
  std::vector<int32_t> row_vcol_win;
  std::vector<AttnWork> work_win;
  int64_t t_vpad_win = 0;
  std::vector<float> rope;            // [n_tokens][dh]: (cos, sin) of every element pair of a head
  std::vector<int32_t> row_seg, row_seg_win;   // hidden row -> index of its segment / window (key-norm table row)
  int n_windows = 0;
  int64_t max_win_len = 0;          // longest window (tokens)
  std::vector<float> lut;             // [3][256]
  std::vector<PreStrip> strips;       // preprocessing work of the strip kernel: copied strips, then (appended at the end of planning) the resampled ones
  std::vector<PreStrip> strips_resampled;
  int n_copy_strips = 0;
  bool affine = false;                // bf16 normalisation table == bf16(fma(v, aff_scale, aff_off)) entry by entry
  float aff_scale[3] = {0, 0, 0}, aff_off[3] = {0, 0, 0};
  std::vector<int32_t> run_rows;      // patch rows produced run by run (unaligned frames, other patch sizes, window order)
  int64_t n_patch_rows = 0, n_tokens = 0, t_vpad = 0;
  int n_segments = 0;
  int bq = 0;                         // query rows per attention work item of the full-segment layers
  bool norm_bound = false, norm_bound_win = false;   // worth computing key norms (long segments / long windows)
  std::vector<int32_t> vt_pads;       // (first column, end column) of every padding run of the transposed-V buffer, both layouts
  // index metadata as one blob (host copy owned by the plan; the caller keeps the device copy)
  std::vector<uint8_t> blob;
  size_t off_vt_pads = 0;
  size_t off_items = 0, off_prow_item = 0, off_prow_thw = 0, off_prow_dst = 0, off_prow_pos = 0, off_vcol = 0,
         off_cls = 0, off_work = 0, off_lut = 0, off_strips = 0, off_run_rows = 0, off_vcol_win = 0, off_work_win = 0,
         off_rope = 0, off_row_seg = 0, off_row_seg_win = 0, meta_bytes = 0;
  int64_t ldvt() const { return std::max(t_vpad, t_vpad_win); }
};

namespace {

thread_local std::string g_create_err;   // reason of the last failed tcmv_create on this thread

int fail(tcmv_ctx* ctx, int code, const std::string& msg) {
  if (ctx) ctx->err = msg;
  return code;
}
int fail_hip(tcmv_ctx* ctx, hipError_t e, const char* what) {
  return fail(ctx, TCMV_E_HIP, std::string(what) + ": " + hipGetErrorString(e));
}

// Query rows per attention work item on the bf16 path.  Head sizes up to 80 allow two query
// tiles per wave (256 rows with 4 waves, 512 with 8); 512-row items stage every K/V tile once per
// CU instead of twice and are used when rounding the segments up to 512 rows wastes little.
int attn_bq_bf16(int dh, int heads, const std::vector<int64_t>& seg_len) {
  if (dh > 80) return 128;
  int64_t rows = 0, padded = 0, items256 = 0;
  for (int64_t n : seg_len) { rows += n; padded += (n + 511) / 512 * 512; items256 += (n + 255) / 256; }
  // a single small request: fewer 256-row work items than CUs; 128-row items double the workgroups
  if (items256 * heads < 256) return 128;
  // segments that fill their last 256-row item badly (576 tokens: 3 items for 2.25 items' worth of rows): 128-row
  // items when they cut the padded rows by a tenth or more
  int64_t p256 = 0, p128 = 0;
  for (int64_t n : seg_len) { p256 += (n + 255) / 256 * 256; p128 += (n + 127) / 128 * 128; }
  if (rows > 0 && p256 * 100 > rows * 115 && p128 * 100 <= p256 * 90) return 128;
  return (rows > 0 && padded * 100 <= rows * 103) ? 512 : 256;
}

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

float round_bf16_host(float f) {
  uint32_t u;
  std::memcpy(&u, &f, 4);
  u = (u + 0x7FFFu + ((u >> 16) & 1u)) & 0xFFFF0000u;
  std::memcpy(&f, &u, 4);
  return f;
}

// size of one head as stored in w_qkv / w_o, width of the attention (heads * head size), softmax scale
int head_dim_of(const tcmv_model_desc& d) { return d.head_dim > 0 ? d.head_dim : d.d / d.heads; }
int attn_width_of(const tcmv_model_desc& d) { return d.heads * head_dim_of(d); }
double attn_scale_of(const tcmv_model_desc& d) {
  return d.attn_scale > 0.f ? (double)d.attn_scale : 1.0 / std::sqrt((double)head_dim_of(d));
}

int validate_desc(const tcmv_model_desc* d, std::string& why) {
  if (!d) { why = "null description"; return TCMV_E_INVALID_ARG; }
  if (d->dtype != TCMV_F32 && d->dtype != TCMV_BF16) { why = "unknown dtype"; return TCMV_E_INVALID_ARG; }
  if (d->layers < 0 || d->d <= 0 || d->heads <= 0 || d->mlp <= 0 || d->patch <= 0 || d->tpatch <= 0 ||
      d->out_dim < 0 || d->max_pos < 0) { why = "non-positive size"; return TCMV_E_INVALID_ARG; }
  if (d->merge != 1 && d->merge != 2) { why = "merge must be 1 or 2"; return TCMV_E_INVALID_ARG; }
  if (d->pos < TCMV_POS_NONE || d->pos > TCMV_POS_ROTARY_2D) { why = "unknown position scheme"; return TCMV_E_INVALID_ARG; }
  if ((d->norm != TCMV_NORM_LAYER && d->norm != TCMV_NORM_RMS) || (d->mlp_gated != 0 && d->mlp_gated != 1) ||
      d->window < 0 || d->full_every < 0) { why = "bad encoder-family switch"; return TCMV_E_INVALID_ARG; }
  if (d->window % d->merge) { why = "window must be a multiple of merge"; return TCMV_E_INVALID_ARG; }
  if (d->pos == TCMV_POS_ROTARY_2D && !(d->rope_theta > 0.f && std::isfinite(d->rope_theta))) { why = "rope_theta must be positive"; return TCMV_E_INVALID_ARG; }
  if (d->head_dim < 0 || !(d->attn_scale >= 0.f) || !std::isfinite(d->attn_scale)) { why = "negative head_dim or attn_scale"; return TCMV_E_INVALID_ARG; }
  if (d->head_dim == 0 && d->d % d->heads) { why = "d not divisible by heads"; return TCMV_E_INVALID_ARG; }
  if (!(d->ln_eps >= 0.f)) { why = "negative ln_eps"; return TCMV_E_INVALID_ARG; }
  for (int c = 0; c < 3; ++c)
    if (!(d->std[c] > 0.f) || !std::isfinite(d->mean[c])) { why = "bad mean/std"; return TCMV_E_INVALID_ARG; }
  if ((d->pos == TCMV_POS_LEARNED_1D || d->pos == TCMV_POS_SEPARABLE_2D) && d->max_pos <= 0) { why = "position table without rows"; return TCMV_E_INVALID_ARG; }
  if (d->pos == TCMV_POS_SEPARABLE_2D && d->use_cls) { why = "CLS with separable 2-D positions"; return TCMV_E_UNSUPPORTED; }
  if (d->out_dim && d->use_cls) { why = "projector with CLS rows"; return TCMV_E_UNSUPPORTED; }
  if (d->patch > 32) { why = "patch above 32"; return TCMV_E_UNSUPPORTED; }
  if (d->d % 4 || d->d > 2048) { why = "d must be a multiple of 4, at most 2048"; return TCMV_E_UNSUPPORTED; }
  const int dh = head_dim_of(*d);
  if (d->head_dim && d->dtype != TCMV_BF16) { why = "an explicit head size needs the bf16 path"; return TCMV_E_UNSUPPORTED; }
  if (d->norm || d->mlp_gated || d->window || d->pos == TCMV_POS_ROTARY_2D) {
    if (d->dtype != TCMV_BF16) { why = "RMSNorm, gated MLP, windows and rotary positions need the bf16 path"; return TCMV_E_UNSUPPORTED; }
    if (d->use_cls) { why = "RMSNorm, gated MLP, windows and rotary positions are defined without CLS rows"; return TCMV_E_UNSUPPORTED; }
    if (d->pos == TCMV_POS_ROTARY_2D && dh % 4) { why = "rotary positions need a head size that is a multiple of 4"; return TCMV_E_UNSUPPORTED; }
  }
  if (d->dtype == TCMV_BF16) {
    if (dh != 32 && dh != 64 && dh != 80 && dh != 96) { why = "bf16 head size must be 32, 64, 80 or 96"; return TCMV_E_UNSUPPORTED; }
    if (d->d % 64 || d->mlp % 64 || d->out_dim % 8 || (d->heads * dh) % 64) { why = "bf16 path needs d, mlp and heads*head size multiples of 64 and out_dim of 8"; return TCMV_E_UNSUPPORTED; }
  } else {
    if (dh % 16 || dh > 128) { why = "fp32 head size must be a multiple of 16, at most 128"; return TCMV_E_UNSUPPORTED; }
  }
  return TCMV_OK;
}

int64_t k_of(const tcmv_model_desc& d) { return 3LL * d.tpatch * d.patch * d.patch; }
int64_t k_pad_of(const tcmv_model_desc& d) {
  const int64_t k = k_of(d);
  return d.dtype == TCMV_BF16 ? (k + 63) / 64 * 64 : (k + 1) / 2 * 2;
}

size_t elt(const tcmv_ctx* c) { return c->desc.dtype == TCMV_BF16 ? 2 : 4; }

struct EncodeWs { size_t xn, qkv, vt, h, kmax, kmax_bytes, splitk, splitk_bytes, total; };
EncodeWs encode_ws(const tcmv_plan* p) {
  const tcmv_model_desc& d = p->ctx->desc;
  const size_t e = elt(p->ctx);
  const size_t T = (size_t)p->n_tokens;
  EncodeWs w{};
  size_t off = 0;
  const size_t da = (size_t)attn_width_of(d);
  w.xn = off; off = align_up(off + T * std::max<size_t>(d.d, da) * e, 256);   // LN output [T, d], then attention output [T, da]
  if (d.dtype == TCMV_BF16) {
    w.qkv = off; off = align_up(off + T * 2 * da * e, 256);
    w.vt = off; off = align_up(off + da * p->ldvt() * e, 256);
  } else {
    w.qkv = off; off = align_up(off + T * 3 * d.d * e, 256);
    w.vt = off;
  }
  w.h = off; off = align_up(off + T * d.mlp * e, 256);   // gated MLP: the product silu(gate)*up, also [T, mlp]
  // largest squared key norm per (segment or window, head)
  // (+ one word behind the table: "some workgroup needs the reference-tracking kernel").  Two such blocks: the
  // layers that use the table alternate between them, and the attention kernel of one layer clears the block
  // of the next.
  w.kmax_bytes = align_up(((size_t)std::max(p->n_segments, p->n_windows) * d.heads + 1) * kKmaxStride * 4, 256);
  w.kmax = off; off += d.dtype == TCMV_BF16 ? 2 * w.kmax_bytes : 0;
  // one small request: room for the four k-slices of the fc2 product (see GemmArgs::partial)
  const bool few_rows = d.dtype == TCMV_BF16 && ((T + 127) / 128) * (((size_t)d.d + 127) / 128) < 200;
  w.splitk_bytes = few_rows ? align_up(4 * T * (size_t)d.d * sizeof(float), 256) : 0;
  w.splitk = off; off += w.splitk_bytes;
  w.total = off;
  return w;
}
struct MergeWs { size_t y, h, total; };
MergeWs merge_ws(const tcmv_plan* p) {
  const tcmv_model_desc& d = p->ctx->desc;
  const size_t e = elt(p->ctx);
  const size_t T = (size_t)p->n_tokens;
  MergeWs w{};
  size_t off = 0;
  w.y = off; off = align_up(off + T * d.d * e, 256);
  w.h = off; off = align_up(off + T * d.d * e, 256);   // [T/m2, m2*d]
  w.total = off;
  return w;
}

template <class T>
size_t place(size_t& off, const std::vector<T>& v) {
  const size_t at = off;
  off = align_up(off + std::max<size_t>(v.size() * sizeof(T), 16), 256);
  return at;
}

template <class T>
const T* dev(const void* d_meta, size_t off) { return reinterpret_cast<const T*>(reinterpret_cast<const uint8_t*>(d_meta) + off); }

// checks the caller's device copy of the plan metadata
int check_meta(tcmv_ctx* ctx, const tcmv_plan* p, const void* d_meta) {
  if (p->meta_bytes == 0) return TCMV_OK;
  if (!d_meta) return fail(ctx, TCMV_E_INVALID_ARG, "null plan metadata buffer (see tcmv_plan_upload)");
  if (reinterpret_cast<uintptr_t>(d_meta) % 256) return fail(ctx, TCMV_E_INVALID_ARG, "plan metadata buffer must be 256-byte aligned");
  return TCMV_OK;
}

void build_work(std::vector<AttnWork>& work, const std::vector<int64_t>& seg_start, const std::vector<int64_t>& seg_len,
                const std::vector<int64_t>& seg_v0, int bq) {
  work.clear();
  for (size_t s = 0; s < seg_start.size(); ++s) {
    for (int64_t q = 0; q < seg_len[s]; q += bq) {
      AttnWork w{};
      w.q0 = (int)(seg_start[s] + q);
      w.nq = (int)std::min<int64_t>(bq, seg_len[s] - q);
      w.seg_start = (int)seg_start[s];
      w.seg_len = (int)seg_len[s];
      w.v0 = (int)seg_v0[s];
      w.seg = (int)s;
      work.push_back(w);
    }
  }
  // longest segments first: the work per tile is proportional to the segment length
  std::stable_sort(work.begin(), work.end(), [](const AttnWork& a, const AttnWork& b) { return a.seg_len > b.seg_len; });
}

// Runs `launch` and, when timing is on, brackets it with an event pair.
template <class F>
hipError_t timed(tcmv_ctx* ctx, int cat, hipStream_t s, F&& launch) {
  if (!((ctx->profile_mask >> cat) & 1u)) return launch();
  tcmv_ctx::Span sp{};
  if (!ctx->free_spans.empty()) {
    sp = ctx->free_spans.back();
    ctx->free_spans.pop_back();
  } else {
    hipError_t e = hipEventCreate(&sp.a);
    if (e != hipSuccess) return e;
    e = hipEventCreate(&sp.b);
    if (e != hipSuccess) { (void)hipEventDestroy(sp.a); return e; }
  }
  sp.cat = cat;
  hipError_t e = hipEventRecord(sp.a, s);
  if (e == hipSuccess) e = launch();
  if (e == hipSuccess) e = hipEventRecord(sp.b, s);
  if (e != hipSuccess) { ctx->free_spans.push_back(sp); return e; }
  ctx->spans.push_back(sp);
  return hipSuccess;
}

hipError_t run_gemm(const tcmv_ctx* ctx, const GemmArgs& g, hipStream_t s) {
  return ctx->desc.dtype == TCMV_BF16 ? launch_gemm_bf16(g, s) : launch_gemm_f32(g, s);
}

}  // namespace

extern "C" {

int tcmv_version(void) { return 200; }   // see include/tcmv.h

const char* tcmv_error_name(int code) {
  switch (code) {
    case TCMV_OK: return "TCMV_OK";
    case TCMV_E_INVALID_ARG: return "TCMV_E_INVALID_ARG";
    case TCMV_E_BAD_SHAPE: return "TCMV_E_BAD_SHAPE";
    case TCMV_E_WORKSPACE_TOO_SMALL: return "TCMV_E_WORKSPACE_TOO_SMALL";
    case TCMV_E_NO_WEIGHTS: return "TCMV_E_NO_WEIGHTS";
    case TCMV_E_HIP: return "TCMV_E_HIP";
    case TCMV_E_UNSUPPORTED: return "TCMV_E_UNSUPPORTED";
    default: return "TCMV_E_UNKNOWN";
  }
}

int64_t tcmv_k_pad(const tcmv_model_desc* desc) {
  std::string why;
  const int rc = validate_desc(desc, why);
  if (rc != TCMV_OK) return rc;
  return k_pad_of(*desc);
}

int tcmv_create(const tcmv_model_desc* desc, tcmv_ctx** out) {
  if (!out) return TCMV_E_INVALID_ARG;
  *out = nullptr;
  std::string why;
  const int rc = validate_desc(desc, why);
  if (rc != TCMV_OK) { g_create_err = why; return rc; }
  tcmv_ctx* c = new (std::nothrow) tcmv_ctx();
  if (!c) return TCMV_E_INVALID_ARG;
  c->desc = *desc;
  c->k = k_of(*desc);
  c->k_pad = k_pad_of(*desc);
  std::memset(&c->w, 0, sizeof(c->w));
  *out = c;
  return TCMV_OK;
}

void tcmv_destroy(tcmv_ctx* ctx) {
  if (!ctx) return;
  for (auto* v : {&ctx->spans, &ctx->free_spans})
    for (auto& sp : *v) { (void)hipEventDestroy(sp.a); (void)hipEventDestroy(sp.b); }
  delete ctx;
}

int tcmv_profile_enable(tcmv_ctx* ctx, int classes) {
  if (!ctx) return TCMV_E_INVALID_ARG;
  ctx->profile_mask = classes < 0 ? ~0u : (unsigned)classes;
  return TCMV_OK;
}

int tcmv_profile_read(tcmv_ctx* ctx, double* ms, int64_t* launches) {
  if (!ctx || !ms || !launches) return TCMV_E_INVALID_ARG;
  for (int i = 0; i < TCMV_K_COUNT; ++i) { ms[i] = 0.0; launches[i] = 0; }
  int rc = TCMV_OK;
  for (auto& sp : ctx->spans) {
    hipError_t e = hipEventSynchronize(sp.b);
    float t = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&t, sp.a, sp.b);
    if (e != hipSuccess) rc = fail_hip(ctx, e, "profile read");
    else { ms[sp.cat] += t; launches[sp.cat] += 1; }
    ctx->free_spans.push_back(sp);
  }
  ctx->spans.clear();
  return rc;
}

const char* tcmv_last_error(const tcmv_ctx* ctx) { return ctx ? ctx->err.c_str() : g_create_err.c_str(); }

int tcmv_set_weights(tcmv_ctx* ctx, const tcmv_weights* w) {
  if (!ctx) return TCMV_E_INVALID_ARG;
  if (!w) return fail(ctx, TCMV_E_INVALID_ARG, "null weights");
  const tcmv_model_desc& d = ctx->desc;
  if (!w->w_pe || !w->b_pe) return fail(ctx, TCMV_E_INVALID_ARG, "w_pe / b_pe missing");
  if (d.use_cls && !w->cls) return fail(ctx, TCMV_E_INVALID_ARG, "cls missing");
  if ((d.pos == TCMV_POS_LEARNED_1D || d.pos == TCMV_POS_SEPARABLE_2D) && !w->pos0) return fail(ctx, TCMV_E_INVALID_ARG, "pos0 missing");
  if (d.pos == TCMV_POS_SEPARABLE_2D && !w->pos1) return fail(ctx, TCMV_E_INVALID_ARG, "pos1 missing");
  if (d.layers > 0 && !w->layer) return fail(ctx, TCMV_E_INVALID_ARG, "layer array missing");
  for (int i = 0; i < d.layers * 12; ++i)
    if (!w->layer[i]) return fail(ctx, TCMV_E_INVALID_ARG, "a layer parameter is missing");
  if (d.final_ln && (!w->lnf_g || !w->lnf_b)) return fail(ctx, TCMV_E_INVALID_ARG, "final LayerNorm missing");
  if (d.out_dim && (!w->lnm_g || !w->lnm_b || !w->w_m1 || !w->b_m1 || !w->w_m2 || !w->b_m2))
    return fail(ctx, TCMV_E_INVALID_ARG, "projector parameters missing");
  ctx->w = *w;
  ctx->layer.assign(w->layer, w->layer + (size_t)d.layers * 12);
  ctx->w.layer = ctx->layer.data();
  ctx->has_weights = true;
  return TCMV_OK;
}

int tcmv_plan_create(tcmv_ctx* ctx, const tcmv_item* items, int n_items, tcmv_plan** out) {
  if (!ctx) return TCMV_E_INVALID_ARG;
  if (!out || n_items < 0 || (n_items > 0 && !items)) return fail(ctx, TCMV_E_INVALID_ARG, "bad plan arguments");
  *out = nullptr;
  const tcmv_model_desc& d = ctx->desc;
  const int pm = d.patch * d.merge;
  tcmv_plan* p = new (std::nothrow) tcmv_plan();
  if (!p) return fail(ctx, TCMV_E_INVALID_ARG, "out of host memory");
  p->ctx = ctx;
  p->cu.assign(1, 0);
  std::vector<int64_t> seg_start, seg_len, seg_v0, win_start, win_len, win_v0;
  const int dh_ = head_dim_of(d);
  std::vector<double> rope_freq;      // theta^(-j/(dh/4)), j < dh/4
  if (d.pos == TCMV_POS_ROTARY_2D)
    for (int j = 0; j < dh_ / 4; ++j) rope_freq.push_back(std::pow((double)d.rope_theta, -(double)j / (double)(dh_ / 4)));
  auto bad = [&](const std::string& m) { delete p; return fail(ctx, TCMV_E_BAD_SHAPE, m); };
  for (int i = 0; i < n_items; ++i) {
    const tcmv_item& it = items[i];
    ItemDev di{};
    di.frames = it.d_frames;
    if (it.n_frames < 0) { delete p; return fail(ctx, TCMV_E_INVALID_ARG, "negative frame count"); }
    if (it.modality < TCMV_TEXT || it.modality > TCMV_VIDEO) { delete p; return fail(ctx, TCMV_E_INVALID_ARG, "unknown modality"); }
    if (it.n_frames == 0) {          // text: no tokens
      p->items.push_back(di);
      p->cu.push_back(p->cu.back());
      continue;
    }
    if (it.dst_h <= 0 || it.dst_w <= 0 || it.dst_h % pm || it.dst_w % pm)
      return bad("target size must be a positive multiple of patch*merge (item " + std::to_string(i) + ")");
    if (it.src_h < 1 || it.src_w < 1) return bad("source size below 1");
    if (it.n_frames > 1 && it.n_frames % d.tpatch) return bad("video length not a multiple of the temporal patch");
    di.n_frames = it.n_frames; di.src_h = it.src_h; di.src_w = it.src_w; di.dst_h = it.dst_h; di.dst_w = it.dst_w;
    di.gt = it.n_frames == 1 ? 1 : it.n_frames / d.tpatch;
    di.gh = it.dst_h / d.patch; di.gw = it.dst_w / d.patch;
    di.resized = (it.src_h != it.dst_h) || (it.src_w != it.dst_w);
    if (di.gh > 255 || di.gw > 255 || di.gt > 32767) return bad("grid too large (side above 255 or more than 32767 frame groups)");
    if ((int64_t)it.src_h * it.src_w > (1LL << 28) || (int64_t)it.src_h * it.dst_h > (1LL << 28) ||
        (int64_t)it.src_w * it.dst_w > (1LL << 28)) return bad("frame too large");
    const int64_t n = (int64_t)di.gt * di.gh * di.gw;
    const int64_t rows = n + (d.use_cls ? 1 : 0);
    if (d.pos == TCMV_POS_LEARNED_1D && rows > d.max_pos) return bad("segment longer than the position table");
    if (d.pos == TCMV_POS_SEPARABLE_2D && (di.gh > d.max_pos || di.gw > d.max_pos)) return bad("grid side above the position table");
    if (p->cu.back() + rows > (1LL << 30)) return bad("too many tokens");
    const int64_t row0 = p->cu.back();
    const int item_idx = (int)p->items.size();
    di.row0 = (int)p->prow_item.size();
    {
      // the strip kernel needs a compiled patch size and the plain token order; where it copies lines (no
      // resampling) it also needs them 4-byte aligned
      const bool aligned = (reinterpret_cast<uintptr_t>(it.d_frames) % 4 == 0) && ((int64_t)it.src_w * 3) % 4 == 0 &&
                           ((int64_t)it.src_h * it.src_w * 3) % 4 == 0;
      const bool strip_ok = d.window == 0 && preprocess_has_strip_kernel(d.patch, d.tpatch) && (di.resized || aligned);
      const int64_t n_rows = (int64_t)di.gt * di.gh * di.gw;
      if (strip_ok) {
        const bool still = di.n_frames == 1;
        std::vector<PreStrip>& list = di.resized ? p->strips_resampled : p->strips;
        for (int t = 0; t < di.gt; ++t)
          for (int ph = 0; ph < di.gh; ++ph)
            for (int pw0 = 0; pw0 < di.gw; pw0 += kStripTokens) {
              PreStrip sp{};
              sp.row_stride = di.src_w * 3;
              sp.frame_stride = di.src_h * di.src_w * 3;               // source pixels per frame <= 2^28 (checked above)
              sp.src = di.frames + (size_t)(still ? 0 : t * d.tpatch) * (size_t)sp.frame_stride +
                       (size_t)(ph * d.patch) * (size_t)sp.row_stride + (size_t)pw0 * d.patch * 3;
              // raster order, or merge-group-major order (strips start at even patch columns)
              sp.row_base = d.merge == 2
                  ? (int64_t)di.row0 + ((int64_t)(t * (di.gh >> 1) + (ph >> 1)) * (di.gw >> 1)) * 4 + (ph & 1) * 2 + (pw0 >> 1) * 4
                  : (int64_t)di.row0 + (int64_t)(t * di.gh + ph) * di.gw + pw0;
              sp.ntok = std::min(kStripTokens, di.gw - pw0);
              sp.flags = (still ? kStripStill : 0) | (di.resized ? kStripResampled : 0);
              sp.item = item_idx; sp.t = t; sp.ph = ph; sp.pw0 = pw0;
              list.push_back(sp);
            }
      } else {
        for (int64_t r = 0; r < n_rows; ++r) p->run_rows.push_back((int32_t)(di.row0 + r));
      }
    }
    if (d.use_cls) p->cls_rows.push_back((int32_t)row0);
    int64_t local = d.use_cls ? 1 : 0;
    auto emit = [&](int t, int h, int w) {
      p->prow_item.push_back(item_idx);
      p->prow_thw.push_back((t << 16) | (h << 8) | w);
      p->prow_dst.push_back((int32_t)(row0 + local));
      int32_t pos = 0;
      if (d.pos == TCMV_POS_LEARNED_1D) pos = (int32_t)local;
      else if (d.pos == TCMV_POS_SEPARABLE_2D) pos = h | (w << 16);
      p->prow_pos.push_back(pos);
      if (d.pos == TCMV_POS_ROTARY_2D) {
        for (int ax = 0; ax < 2; ++ax)
          for (int j = 0; j < dh_ / 4; ++j) {
            const double ang = (double)(ax == 0 ? h : w) * rope_freq[(size_t)j];
            p->rope.push_back((float)std::cos(ang));
            p->rope.push_back((float)std::sin(ang));
          }
      }
      ++local;
    };
    // frame groups; inside one, windows in raster order (one window = the whole grid without
    // windows); inside a window, merge groups in raster order, the rows of a group consecutive
    const int wh = d.window ? d.window : di.gh, ww = d.window ? d.window : di.gw;
    for (int t = 0; t < di.gt; ++t)
      for (int h0 = 0; h0 < di.gh; h0 += wh)
        for (int w0 = 0; w0 < di.gw; w0 += ww) {
          const int h1 = std::min(di.gh, h0 + wh), w1 = std::min(di.gw, w0 + ww);
          if (d.window) {
            const int64_t n_win = (int64_t)(h1 - h0) * (w1 - w0);
            win_start.push_back(row0 + local);
            win_len.push_back(n_win);
            win_v0.push_back(p->t_vpad_win);
            if (n_win % kVtAlign) { p->vt_pads.push_back((int32_t)(p->t_vpad_win + (n_win & ~(int64_t)15))); p->vt_pads.push_back((int32_t)(p->t_vpad_win + (n_win + kVtAlign - 1) / kVtAlign * kVtAlign)); }
            for (int64_t r = 0; r < n_win; ++r) {
              p->row_vcol_win.push_back((int32_t)(p->t_vpad_win + vt_col_in_segment(r)));
              p->row_seg_win.push_back((int32_t)(win_start.size() - 1));
            }
            p->t_vpad_win += (n_win + kVtAlign - 1) / kVtAlign * kVtAlign;
          }
          for (int hb = h0; hb < h1; hb += d.merge)
            for (int wb = w0; wb < w1; wb += d.merge)
              for (int hi = 0; hi < d.merge; ++hi)
                for (int wi = 0; wi < d.merge; ++wi) emit(t, hb + hi, wb + wi);
        }
    seg_start.push_back(row0);
    seg_len.push_back(rows);
    seg_v0.push_back(p->t_vpad);
    // columns that no key of the segment is written to: from the last (partly filled) group of 16 keys, whose
    // quarters are interleaved, to the end of the 64-column padding
    if (rows % kVtAlign) { p->vt_pads.push_back((int32_t)(p->t_vpad + (rows & ~(int64_t)15))); p->vt_pads.push_back((int32_t)(p->t_vpad + (rows + kVtAlign - 1) / kVtAlign * kVtAlign)); }
    for (int64_t r = 0; r < rows; ++r) {
      p->row_vcol.push_back((int32_t)(p->t_vpad + vt_col_in_segment(r)));
      p->row_seg.push_back((int32_t)(seg_start.size() - 1));
    }
    p->t_vpad += (rows + kVtAlign - 1) / kVtAlign * kVtAlign;
    p->items.push_back(di);
    p->cu.push_back(row0 + rows);
  }
  p->n_patch_rows = (int64_t)p->prow_item.size();
  p->n_tokens = p->cu.back();
  {
    // the kernels keep element offsets into the activation matrices in 32 bits
    const int64_t m2 = (int64_t)d.merge * d.merge;
    const int64_t widest = std::max<int64_t>({3LL * d.d, 3LL * attn_width_of(d), (int64_t)d.mlp, m2 * d.d, k_pad_of(d)});
    if ((double)(p->t_vpad + kVtAlign) * (double)widest >= 4294967296.0)
      return bad("too many tokens in one plan: tokens x widest activation row (max of 3d, mlp, merge^2 d, k_pad) must stay below 2^32");
    // the attention kernel addresses its operands in bytes, 32 bits: the keys (rows of 2 x attention width) ...
    if ((double)(p->t_vpad + kVtAlign) * 2.0 * (double)attn_width_of(d) >= 2147483648.0)
      return bad("too many tokens in one plan: tokens x 2 x attention width must stay below 2^31 elements");
    // ... and the transposed values: heads x head size rows of ldvt() columns (every window padded to 64 columns)
    if ((double)(p->ldvt() + kVtAlign) * (double)attn_width_of(d) >= 2147483648.0)
      return bad("too many tokens in one plan: the transposed values (padded columns x attention width) must stay below 2^31 elements");
  }
  p->n_segments = (int)seg_start.size();
  p->bq = d.dtype == TCMV_BF16 ? attn_bq_bf16(head_dim_of(d), d.heads, seg_len) : kAttnBQ_f32;
  build_work(p->work, seg_start, seg_len, seg_v0, p->bq);
  if (d.window) build_work(p->work_win, win_start, win_len, win_v0, kAttnBQ_window);
  // The key norms come out of the QKV epilogue (a few table updates per tile) and the second attention launch costs a
  // few microseconds; what the reference-free loop saves grows with the number of keys per query.  Measured: it pays
  // from about 1024 keys per query on average (64 stills of 1024 tokens: attention 15.7 -> 12.9 ms per step) and
  // costs time on batches of 577- or 729-token images, which run one query tile per wave.
  auto long_enough = [](const std::vector<int64_t>& len) {
    double rows = 0, pairs = 0;
    for (int64_t n : len) { rows += (double)n; pairs += (double)n * (double)n; }
    return rows > 0 && pairs >= 1024.0 * rows;
  };
  p->norm_bound = d.dtype == TCMV_BF16 && long_enough(seg_len);
  p->norm_bound_win = d.dtype == TCMV_BF16 && long_enough(win_len);
  p->n_windows = (int)win_start.size();
  for (int64_t n : win_len) p->max_win_len = std::max(p->max_win_len, n);
  // normalisation table: (v/255 - mean)/std in double, rounded to fp32, then to bf16 for bf16 models
  p->lut.resize(3 * 256);
  for (int c = 0; c < 3; ++c)
    for (int v = 0; v < 256; ++v) {
      float x = (float)(((double)v / 255.0 - (double)d.mean[c]) / (double)d.std[c]);
      if (d.dtype == TCMV_BF16) x = round_bf16_host(x);
      p->lut[c * 256 + v] = x;
    }
  // The bf16 strip kernel may compute the normalised value (one fused multiply-add, then the conversion to bf16,
  // both correctly rounded on host and device alike) instead of looking it up - but only if that reproduces the
  // table, which holds the contract's arithmetic, in all 768 entries.
  p->affine = d.dtype == TCMV_BF16;
  for (int c = 0; c < 3 && p->affine; ++c) {
    p->aff_scale[c] = (float)(1.0 / (255.0 * (double)d.std[c]));
    p->aff_off[c] = (float)(-(double)d.mean[c] / (double)d.std[c]);
    for (int v = 0; v < 256; ++v)
      if (round_bf16_host(std::fmaf((float)v, p->aff_scale[c], p->aff_off[c])) != p->lut[c * 256 + v]) p->affine = false;
  }
  p->n_copy_strips = (int)p->strips.size();
  p->strips.insert(p->strips.end(), p->strips_resampled.begin(), p->strips_resampled.end());
  p->strips_resampled.clear();
  size_t off = 0;
  p->off_items = place(off, p->items);
  p->off_prow_item = place(off, p->prow_item);
  p->off_prow_thw = place(off, p->prow_thw);
  p->off_prow_dst = place(off, p->prow_dst);
  p->off_prow_pos = place(off, p->prow_pos);
  p->off_vcol = place(off, p->row_vcol);
  p->off_cls = place(off, p->cls_rows);
  p->off_work = place(off, p->work);
  p->off_lut = place(off, p->lut);
  p->off_strips = place(off, p->strips);
  p->off_run_rows = place(off, p->run_rows);
  p->off_vcol_win = place(off, p->row_vcol_win);
  p->off_work_win = place(off, p->work_win);
  p->off_rope = place(off, p->rope);
  p->off_row_seg = place(off, p->row_seg);
  p->off_row_seg_win = place(off, p->row_seg_win);
  p->off_vt_pads = place(off, p->vt_pads);
  p->meta_bytes = p->n_patch_rows > 0 ? off : 0;
  {
    p->blob.assign(p->meta_bytes, 0);
    auto put = [&](size_t at, const void* src, size_t n) { if (n && p->meta_bytes) std::memcpy(p->blob.data() + at, src, n); };
    put(p->off_items, p->items.data(), p->items.size() * sizeof(ItemDev));
    put(p->off_prow_item, p->prow_item.data(), p->prow_item.size() * 4);
    put(p->off_prow_thw, p->prow_thw.data(), p->prow_thw.size() * 4);
    put(p->off_prow_dst, p->prow_dst.data(), p->prow_dst.size() * 4);
    put(p->off_prow_pos, p->prow_pos.data(), p->prow_pos.size() * 4);
    put(p->off_vcol, p->row_vcol.data(), p->row_vcol.size() * 4);
    put(p->off_cls, p->cls_rows.data(), p->cls_rows.size() * 4);
    put(p->off_work, p->work.data(), p->work.size() * sizeof(AttnWork));
    put(p->off_lut, p->lut.data(), p->lut.size() * 4);
    put(p->off_strips, p->strips.data(), p->strips.size() * sizeof(PreStrip));
    put(p->off_run_rows, p->run_rows.data(), p->run_rows.size() * 4);
    put(p->off_vcol_win, p->row_vcol_win.data(), p->row_vcol_win.size() * 4);
    put(p->off_work_win, p->work_win.data(), p->work_win.size() * sizeof(AttnWork));
    put(p->off_rope, p->rope.data(), p->rope.size() * 4);
    put(p->off_row_seg, p->row_seg.data(), p->row_seg.size() * 4);
    put(p->off_row_seg_win, p->row_seg_win.data(), p->row_seg_win.size() * 4);
    put(p->off_vt_pads, p->vt_pads.data(), p->vt_pads.size() * 4);
  }
  *out = p;
  return TCMV_OK;
}

void tcmv_plan_destroy(tcmv_plan* plan) { delete plan; }

const void* tcmv_plan_meta(const tcmv_plan* p, size_t* bytes) {
  if (!p) return nullptr;
  if (bytes) *bytes = p->meta_bytes;
  return p->meta_bytes ? p->blob.data() : nullptr;
}

int tcmv_plan_upload(const tcmv_plan* p, void* d_meta, size_t meta_bytes, void* stream) {
  if (!p) return TCMV_E_INVALID_ARG;
  tcmv_ctx* ctx = p->ctx;
  if (p->meta_bytes == 0) return TCMV_OK;
  if (!d_meta) return fail(ctx, TCMV_E_INVALID_ARG, "null plan metadata buffer");
  if (reinterpret_cast<uintptr_t>(d_meta) % 256) return fail(ctx, TCMV_E_INVALID_ARG, "plan metadata buffer must be 256-byte aligned");
  if (meta_bytes < p->meta_bytes) return fail(ctx, TCMV_E_WORKSPACE_TOO_SMALL, "plan metadata buffer too small");
  const hipError_t e = hipMemcpyAsync(d_meta, p->blob.data(), p->meta_bytes, hipMemcpyHostToDevice, (hipStream_t)stream);
  if (e != hipSuccess) return fail_hip(ctx, e, "hipMemcpyAsync(plan metadata)");
  return TCMV_OK;
}

int tcmv_plan_query(const tcmv_plan* p, tcmv_plan_info* info) {
  if (!p || !info) return TCMV_E_INVALID_ARG;
  const tcmv_model_desc& d = p->ctx->desc;
  std::memset(info, 0, sizeof(*info));
  info->n_patch_rows = p->n_patch_rows;
  info->n_tokens = p->n_tokens;
  const int m2 = d.merge * d.merge;
  info->n_out_tokens = d.out_dim ? p->n_tokens / m2 : 0;
  info->k = p->ctx->k;
  info->k_pad = p->ctx->k_pad;
  info->patches_bytes = (size_t)p->n_patch_rows * p->ctx->k_pad * elt(p->ctx);
  info->hidden_bytes = (size_t)p->n_tokens * d.d * 4;
  info->out_bytes = (size_t)info->n_out_tokens * d.out_dim * elt(p->ctx);
  info->encode_workspace_bytes = encode_ws(p).total;
  info->merge_workspace_bytes = d.out_dim ? merge_ws(p).total : 0;
  info->n_items = (int)p->items.size();
  info->n_segments = p->n_segments;
  info->meta_bytes = p->meta_bytes;
  return TCMV_OK;
}

const int64_t* tcmv_plan_cu_seqlens(const tcmv_plan* p) { return p ? p->cu.data() : nullptr; }

int64_t tcmv_plan_row_map(const tcmv_plan* p, int which, const int32_t** out) {
  if (!p || !out) return TCMV_E_INVALID_ARG;
  const std::vector<int32_t>* v = nullptr;
  switch (which) {
    case 0: v = &p->prow_thw; break;
    case 1: v = &p->prow_dst; break;
    case 2: v = &p->prow_pos; break;
    default: return TCMV_E_INVALID_ARG;
  }
  *out = v->data();
  return (int64_t)v->size();
}

int tcmv_preprocess(tcmv_ctx* ctx, const tcmv_plan* p, const void* d_meta, void* d_patches, void* stream) {
  if (!ctx) return TCMV_E_INVALID_ARG;
  if (!p || p->ctx != ctx) return fail(ctx, TCMV_E_INVALID_ARG, "plan does not belong to this context");
  if (p->n_patch_rows == 0) return TCMV_OK;
  if (!d_patches) return fail(ctx, TCMV_E_INVALID_ARG, "null patch buffer");
  if (reinterpret_cast<uintptr_t>(d_patches) % 16) return fail(ctx, TCMV_E_INVALID_ARG, "patch buffer must be 16-byte aligned");
  for (const ItemDev& it : p->items)
    if (it.n_frames > 0 && !it.frames) return fail(ctx, TCMV_E_INVALID_ARG, "an item with frames has a null frame pointer");
  const int rc = check_meta(ctx, p, d_meta);
  if (rc != TCMV_OK) return rc;
  PreprocArgs a{};
  a.items = dev<ItemDev>(d_meta, p->off_items);
  a.prow_item = dev<int32_t>(d_meta, p->off_prow_item);
  a.prow_thw = dev<int32_t>(d_meta, p->off_prow_thw);
  a.lut = dev<float>(d_meta, p->off_lut);
  a.patches = d_patches;
  a.rows = p->n_patch_rows;
  a.patch = ctx->desc.patch; a.tpatch = ctx->desc.tpatch;
  a.k = (int)ctx->k; a.k_pad = (int)ctx->k_pad;
  a.out_bf16 = ctx->desc.dtype == TCMV_BF16;
  a.merge = ctx->desc.merge;
  a.strips = dev<PreStrip>(d_meta, p->off_strips); a.n_strips = (int)p->strips.size();
  a.n_copy_strips = p->n_copy_strips;
  a.affine = p->affine;
  for (int c = 0; c < 3; ++c) { a.aff_scale[c] = p->aff_scale[c]; a.aff_off[c] = p->aff_off[c]; }
  a.run_rows = dev<int32_t>(d_meta, p->off_run_rows); a.n_run_rows = (int64_t)p->run_rows.size();
  hipError_t e = timed(ctx, TCMV_K_PREPROCESS, (hipStream_t)stream, [&] { return launch_preprocess(a, (hipStream_t)stream); });
  if (e != hipSuccess) return fail_hip(ctx, e, "preprocess launch");
  return TCMV_OK;
}

int tcmv_encode(tcmv_ctx* ctx, const tcmv_plan* p, const void* d_meta, const void* d_patches, void* d_hidden,
                void* d_workspace, size_t workspace_bytes, void* stream) {
  if (!ctx) return TCMV_E_INVALID_ARG;
  if (!p || p->ctx != ctx) return fail(ctx, TCMV_E_INVALID_ARG, "plan does not belong to this context");
  if (!ctx->has_weights) return fail(ctx, TCMV_E_NO_WEIGHTS, "tcmv_set_weights has not been called");
  if (p->n_tokens == 0) return TCMV_OK;
  if (!d_patches || !d_hidden || !d_workspace) return fail(ctx, TCMV_E_INVALID_ARG, "null buffer");
  if (reinterpret_cast<uintptr_t>(d_workspace) % 256) return fail(ctx, TCMV_E_INVALID_ARG, "workspace not 256-byte aligned");
  const EncodeWs ws = encode_ws(p);
  if (workspace_bytes < ws.total) return fail(ctx, TCMV_E_WORKSPACE_TOO_SMALL, "encode workspace too small");
  const int rc = check_meta(ctx, p, d_meta);
  if (rc != TCMV_OK) return rc;

  const tcmv_model_desc& d = ctx->desc;
  const bool bf = d.dtype == TCMV_BF16;
  hipStream_t s = (hipStream_t)stream;
  uint8_t* wsb = reinterpret_cast<uint8_t*>(d_workspace);
  void* xn = wsb + ws.xn;
  void* qkv = wsb + ws.qkv;
  void* vt = wsb + ws.vt;
  void* hbuf = wsb + ws.h;
  float* x = reinterpret_cast<float*>(d_hidden);
  const int64_t T = p->n_tokens;
  const int dh = head_dim_of(d);
  const int da = attn_width_of(d);               // width of q, k, v and of the attention output (= d unless head_dim is set)
  hipError_t e;
#define TCMV_CHECK(call, what) do { e = (call); if (e != hipSuccess) return fail_hip(ctx, e, what); } while (0)

  // The padding columns of the transposed-V buffer must never hold NaN or infinity bit patterns (their
  // probabilities are zero, and 0 * NaN is NaN): they are cleared once, for both column layouts.  Both key-norm
  // blocks start at zero.
  if (bf)
    TCMV_CHECK(timed(ctx, TCMV_K_OTHER, s, [&] {
                 return launch_attn_prepare(vt, p->ldvt(), da, dev<int32_t>(d_meta, p->off_vt_pads), (int)(p->vt_pads.size() / 2),
                                            reinterpret_cast<uint32_t*>(wsb + ws.kmax), (int)(2 * ws.kmax_bytes / 4), s); }),
               "attention set-up");
  int kblock = 0;                                  // key-norm block of the next layer that uses one
  // patch embedding (+ position), CLS rows
  {
    GemmArgs g{};
    g.a = d_patches; g.lda = ctx->k_pad; g.w = ctx->w.w_pe; g.bias = reinterpret_cast<const float*>(ctx->w.b_pe);
    g.c = x; g.ldc = d.d; g.m = p->n_patch_rows; g.n = d.d; g.k = (int)ctx->k_pad; g.epi = EPI_EMBED;
    g.dst_row = dev<int32_t>(d_meta, p->off_prow_dst); g.pos_idx = dev<int32_t>(d_meta, p->off_prow_pos);
    g.pos0 = reinterpret_cast<const float*>(ctx->w.pos0); g.pos1 = reinterpret_cast<const float*>(ctx->w.pos1);
    g.pos_kind = d.pos;
    TCMV_CHECK(timed(ctx, TCMV_K_EMBED_GEMM, s, [&] { return run_gemm(ctx, g, s); }), "patch-embed GEMM");
    if (d.use_cls)
      TCMV_CHECK(timed(ctx, TCMV_K_OTHER, s, [&] {
                   return launch_cls_rows(x, dev<int32_t>(d_meta, p->off_cls), (int)p->cls_rows.size(),
                                          reinterpret_cast<const float*>(ctx->w.cls),
                                          d.pos == TCMV_POS_LEARNED_1D ? reinterpret_cast<const float*>(ctx->w.pos0) : nullptr,
                                          d.d, s); }), "CLS rows");
  }
  for (int l = 0; l < d.layers; ++l) {
    const void* const* L = ctx->layer.data() + (size_t)l * 12;
    auto f = [&](int j) { return reinterpret_cast<const float*>(L[j]); };
    const bool windowed = d.window && !(d.full_every && (l + 1) % d.full_every == 0);
    TCMV_CHECK(timed(ctx, TCMV_K_LAYERNORM, s, [&] { return launch_layernorm(x, f(0), f(1), xn, T, d.d, d.ln_eps, bf, s, d.norm); }), "LN1");
    bool use_kmax = false, kmax_fused = false;
    uint32_t *kmax = nullptr, *kmax_other = nullptr;
    const int32_t* row_seg = nullptr;
    {
      GemmArgs g{};
      g.a = xn; g.lda = d.d; g.w = L[2]; g.bias = f(3); g.m = T; g.n = 3 * da; g.k = d.d;
      g.c = qkv; g.epi = EPI_QKV;
      if (bf) {
        g.ldc = 2 * da; g.split = 2 * da; g.vt = vt; g.ldvt = p->ldvt();
        g.vcol = dev<int32_t>(d_meta, windowed ? p->off_vcol_win : p->off_vcol);
        if (d.pos == TCMV_POS_ROTARY_2D) { g.rope = dev<float>(d_meta, p->off_rope); g.rope_dh = dh; }
        // the queries leave the projection already multiplied by softmax scale * log2(e)
        g.qcols = da; g.qscale = (float)(1.4426950408889634 * attn_scale_of(d));
        // largest key norm per (segment, head): lets the attention kernel drop the running maximum where the
        // scores are provably small.  The projection's epilogue computes it where its tiles line up with the heads.
        const bool short_windows = windowed && p->max_win_len <= 64;
        use_kmax = !short_windows && (windowed ? p->norm_bound_win : p->norm_bound);
        if (use_kmax) {
          kmax = reinterpret_cast<uint32_t*>(wsb + ws.kmax + (size_t)kblock * ws.kmax_bytes);
          kmax_other = reinterpret_cast<uint32_t*>(wsb + ws.kmax + (size_t)(kblock ^ 1) * ws.kmax_bytes);
          kblock ^= 1;
          row_seg = dev<int32_t>(d_meta, windowed ? p->off_row_seg_win : p->off_row_seg);
          if (gemm_bf16_can_fuse_key_norms(T, 3 * da, d.d, da, dh)) {
            g.kmax2 = kmax; g.row_seg = row_seg; g.kn_dh = dh; g.kn_heads = d.heads;
            kmax_fused = true;
          }
        }
      }
      else { g.ldc = 3 * d.d; }
      TCMV_CHECK(timed(ctx, TCMV_K_QKV_GEMM, s, [&] { return run_gemm(ctx, g, s); }), "QKV GEMM");
    }
    {
      AttnArgs a{};
      if (windowed) { a.work = dev<AttnWork>(d_meta, p->off_work_win); a.n_work = (int)p->work_win.size(); }
      else { a.work = dev<AttnWork>(d_meta, p->off_work); a.n_work = (int)p->work.size(); }
      a.heads = d.heads; a.dh = dh; a.t_total = T; a.out = xn; a.ldo = da;
      a.bq = windowed ? kAttnBQ_window : p->bq;
      if (bf) {
        const uint16_t* qk = reinterpret_cast<const uint16_t*>(qkv);
        a.q = qk; a.k = qk + da; a.ldqk = 2 * da; a.v = vt; a.ldv = p->ldvt();
        a.scale = 1.0f; a.prescaled = 1;
        // windows of at most 64 tokens (8 x 8 patches): one small workgroup per window and head
        const bool short_windows = windowed && p->max_win_len <= 64;
        if (use_kmax) {
          if (!kmax_fused)
            TCMV_CHECK(timed(ctx, TCMV_K_ATTENTION, s, [&] { return launch_knorm(qk + da, 2 * da, T, d.heads, dh, row_seg, kmax, s); }),
                       "key norms");
          a.kmax2 = kmax;
          a.any_left = kmax + (size_t)std::max(p->n_segments, p->n_windows) * d.heads * kKmaxStride;
          a.kmax_clear = kmax_other; a.n_clear = (int)(ws.kmax_bytes / 4);
        }
        TCMV_CHECK(timed(ctx, TCMV_K_ATTENTION, s, [&] { return short_windows ? launch_attn_window_bf16(a, s) : launch_attn_bf16(a, s); }),
                   "attention");
      } else {
        const float* q3 = reinterpret_cast<const float*>(qkv);
        a.q = q3; a.k = q3 + d.d; a.ldqk = 3 * d.d; a.v = q3 + 2 * d.d; a.ldv = 3 * d.d;
        a.scale = (float)attn_scale_of(d);
        TCMV_CHECK(timed(ctx, TCMV_K_ATTENTION, s, [&] { return launch_attn_f32(a, s); }), "attention");
      }
    }
    {
      GemmArgs g{};
      g.a = xn; g.lda = da; g.w = L[4]; g.bias = f(5); g.c = x; g.ldc = d.d; g.m = T; g.n = d.d; g.k = da;
      g.epi = EPI_RESID;
      TCMV_CHECK(timed(ctx, TCMV_K_OUT_GEMM, s, [&] { return run_gemm(ctx, g, s); }), "out-proj GEMM");
    }
    TCMV_CHECK(timed(ctx, TCMV_K_LAYERNORM, s, [&] { return launch_layernorm(x, f(6), f(7), xn, T, d.d, d.ln_eps, bf, s, d.norm); }), "LN2");
    {
      GemmArgs g{};
      g.a = xn; g.lda = d.d; g.w = L[8]; g.bias = f(9); g.c = hbuf; g.ldc = d.mlp; g.m = T; g.k = d.d;
      if (d.mlp_gated) { g.n = 2 * d.mlp; g.epi = EPI_GATED; }      // (gate, up) column pairs -> one column of hbuf
      else { g.n = d.mlp; g.epi = EPI_GELU; }
      TCMV_CHECK(timed(ctx, TCMV_K_FC1_GEMM, s, [&] { return run_gemm(ctx, g, s); }), "fc1 GEMM");
    }
    {
      GemmArgs g{};
      g.a = hbuf; g.lda = d.mlp; g.w = L[10]; g.bias = f(11); g.c = x; g.ldc = d.d; g.m = T; g.n = d.d; g.k = d.mlp;
      g.epi = EPI_RESID;
      if (ws.splitk_bytes) g.partial = reinterpret_cast<float*>(wsb + ws.splitk);
      TCMV_CHECK(timed(ctx, TCMV_K_FC2_GEMM, s, [&] { return run_gemm(ctx, g, s); }), "fc2 GEMM");
    }
  }
  if (d.final_ln)
    TCMV_CHECK(timed(ctx, TCMV_K_LAYERNORM, s, [&] {
                 return launch_layernorm(x, reinterpret_cast<const float*>(ctx->w.lnf_g),
                                         reinterpret_cast<const float*>(ctx->w.lnf_b), x, T, d.d, d.ln_eps, 0, s, d.norm); }),
               "final LN");
  return TCMV_OK;
}

int tcmv_merge_project(tcmv_ctx* ctx, const tcmv_plan* p, const void* d_hidden, void* d_out, void* d_workspace,
                       size_t workspace_bytes, void* stream) {
  if (!ctx) return TCMV_E_INVALID_ARG;
  if (!p || p->ctx != ctx) return fail(ctx, TCMV_E_INVALID_ARG, "plan does not belong to this context");
  const tcmv_model_desc& d = ctx->desc;
  if (!d.out_dim) return fail(ctx, TCMV_E_UNSUPPORTED, "model has no projector");
  if (!ctx->has_weights) return fail(ctx, TCMV_E_NO_WEIGHTS, "tcmv_set_weights has not been called");
  if (p->n_tokens == 0) return TCMV_OK;
  if (!d_hidden || !d_out || !d_workspace) return fail(ctx, TCMV_E_INVALID_ARG, "null buffer");
  if (reinterpret_cast<uintptr_t>(d_workspace) % 256) return fail(ctx, TCMV_E_INVALID_ARG, "workspace not 256-byte aligned");
  const MergeWs ws = merge_ws(p);
  if (workspace_bytes < ws.total) return fail(ctx, TCMV_E_WORKSPACE_TOO_SMALL, "merge workspace too small");
  const bool bf = d.dtype == TCMV_BF16;
  hipStream_t s = (hipStream_t)stream;
  uint8_t* wsb = reinterpret_cast<uint8_t*>(d_workspace);
  void* y = wsb + ws.y;
  void* h = wsb + ws.h;
  const int m2 = d.merge * d.merge;
  const int64_t T = p->n_tokens, Tm = T / m2;
  const int dm = d.d * m2;
  hipError_t e;
  TCMV_CHECK(timed(ctx, TCMV_K_LAYERNORM, s, [&] {
               return launch_layernorm(reinterpret_cast<const float*>(d_hidden), reinterpret_cast<const float*>(ctx->w.lnm_g),
                                       reinterpret_cast<const float*>(ctx->w.lnm_b), y, T, d.d, d.ln_eps, bf, s, d.norm); }),
             "merger LN");
  {
    GemmArgs g{};
    g.a = y; g.lda = dm; g.w = ctx->w.w_m1; g.bias = reinterpret_cast<const float*>(ctx->w.b_m1);
    g.c = h; g.ldc = dm; g.m = Tm; g.n = dm; g.k = dm; g.epi = EPI_GELU;
    TCMV_CHECK(timed(ctx, TCMV_K_MERGE_GEMM, s, [&] { return run_gemm(ctx, g, s); }), "merger fc1 GEMM");
  }
  {
    GemmArgs g{};
    g.a = h; g.lda = dm; g.w = ctx->w.w_m2; g.bias = reinterpret_cast<const float*>(ctx->w.b_m2);
    g.c = d_out; g.ldc = d.out_dim; g.m = Tm; g.n = d.out_dim; g.k = dm; g.epi = EPI_STORE;
    TCMV_CHECK(timed(ctx, TCMV_K_MERGE_GEMM, s, [&] { return run_gemm(ctx, g, s); }), "merger fc2 GEMM");
  }
  return TCMV_OK;
}

// ---- single operators ------------------------------------------------------

int tcmv_op_layernorm(int dtype, const float* d_x, const float* d_gamma, const float* d_beta, void* d_y,
                      int64_t rows, int d, float eps, void* stream) {
  if ((dtype != TCMV_F32 && dtype != TCMV_BF16) || rows < 0 || d <= 0) return TCMV_E_INVALID_ARG;
  if (rows == 0) return TCMV_OK;
  if (!d_x || !d_gamma || !d_y) return TCMV_E_INVALID_ARG;
  if (d % 4 || d > 2048) return TCMV_E_UNSUPPORTED;
  return launch_layernorm(d_x, d_gamma, d_beta, d_y, rows, d, eps, dtype == TCMV_BF16, (hipStream_t)stream,
                          d_beta ? 0 : 1) == hipSuccess
             ? TCMV_OK : TCMV_E_HIP;
}

int tcmv_op_stream(const void* d_in, size_t in_bytes, void* d_out, size_t out_bytes, void* stream) {
  if ((in_bytes && !d_in) || (out_bytes && !d_out)) return TCMV_E_INVALID_ARG;
  if (in_bytes % 16 || out_bytes % 16 || reinterpret_cast<uintptr_t>(d_in) % 16 || reinterpret_cast<uintptr_t>(d_out) % 16)
    return TCMV_E_INVALID_ARG;
  return launch_stream_ref(d_in, in_bytes, d_out, out_bytes, (hipStream_t)stream) == hipSuccess ? TCMV_OK : TCMV_E_HIP;
}

int tcmv_op_gemm(int dtype, int epilogue, const void* d_a, const void* d_w, const float* d_bias, void* d_c,
                 int64_t m, int n, int k, void* stream) {
  const bool gated = epilogue == EPI_GATED;
  if ((dtype != TCMV_F32 && dtype != TCMV_BF16) || epilogue < 0 || (epilogue > 2 && !gated) || m < 0 || n <= 0 || k <= 0)
    return TCMV_E_INVALID_ARG;
  if (m == 0) return TCMV_OK;
  if (!d_a || !d_w || !d_c) return TCMV_E_INVALID_ARG;
  if (dtype == TCMV_BF16 && (k % 64 || n % 8)) return TCMV_E_UNSUPPORTED;
  if (gated && dtype != TCMV_BF16) return TCMV_E_UNSUPPORTED;
  GemmArgs g{};
  g.a = d_a; g.lda = k; g.w = d_w; g.bias = d_bias; g.c = d_c; g.ldc = gated ? n / 2 : n; g.m = m; g.n = n; g.k = k;
  g.epi = epilogue;
  const hipError_t e = dtype == TCMV_BF16 ? launch_gemm_bf16(g, (hipStream_t)stream) : launch_gemm_f32(g, (hipStream_t)stream);
  return e == hipSuccess ? TCMV_OK : TCMV_E_HIP;
}

namespace {
// Index data (built on the host, uploaded by the caller): [row -> transposed-V column][work list][row -> segment].
// Scratch: [transposed V][key-norm table + flag].
struct OpAttnLayout { size_t vcol, work, rseg, index_total; size_t vt, kmax, kmax_bytes, ws_total; int64_t t_vpad; int64_t T; int bq; size_t n_seg; size_t n_work; };
OpAttnLayout op_attn_layout(int dtype, const int64_t* cu, int n_seg, int d, int heads, std::vector<int32_t>* vcol,
                            std::vector<AttnWork>* work, std::vector<int32_t>* rseg = nullptr) {
  OpAttnLayout L{};
  std::vector<int64_t> ss, sl, sv;
  int64_t vp = 0;
  for (int s = 0; s < n_seg; ++s) {
    const int64_t len = cu[s + 1] - cu[s];
    if (len <= 0) continue;
    ss.push_back(cu[s]); sl.push_back(len); sv.push_back(vp);
    vp += (len + kVtAlign - 1) / kVtAlign * kVtAlign;
  }
  L.T = n_seg > 0 ? cu[n_seg] : 0;
  L.t_vpad = vp;
  std::vector<AttnWork> wtmp;
  L.bq = dtype == TCMV_BF16 ? attn_bq_bf16(d / heads, heads, sl) : kAttnBQ_f32;
  build_work(wtmp, ss, sl, sv, L.bq);
  if (vcol) {
    vcol->assign((size_t)L.T, 0);
    for (size_t s = 0; s < ss.size(); ++s)
      for (int64_t r = 0; r < sl[s]; ++r) (*vcol)[(size_t)(ss[s] + r)] = (int32_t)(sv[s] + vt_col_in_segment(r));
  }
  if (rseg) {
    rseg->assign((size_t)L.T, 0);
    for (size_t s = 0; s < ss.size(); ++s)
      for (int64_t r = 0; r < sl[s]; ++r) (*rseg)[(size_t)(ss[s] + r)] = (int32_t)s;
  }
  size_t off = 0;
  L.vcol = off; off = align_up(off + std::max<size_t>((size_t)L.T * 4, 16), 256);
  L.work = off; off = align_up(off + std::max<size_t>(wtmp.size() * sizeof(AttnWork), 16), 256);
  L.rseg = off; off = align_up(off + std::max<size_t>((size_t)L.T * 4, 16), 256);
  L.index_total = off;
  off = 0;
  L.vt = off;
  if (dtype == TCMV_BF16) off = align_up(off + (size_t)d * vp * 2, 256);
  L.kmax_bytes = align_up((ss.size() * (size_t)heads + 1) * kKmaxStride * 4, 256);
  L.kmax = off; off += L.kmax_bytes;
  L.ws_total = off;
  L.n_seg = ss.size();
  L.n_work = wtmp.size();
  if (work) work->swap(wtmp);
  return L;
}
bool cu_ok(const int64_t* cu, int n_seg) {
  if (!cu || n_seg < 0) return false;
  if (cu[0] != 0) return false;
  for (int s = 0; s < n_seg; ++s)
    if (cu[s + 1] < cu[s]) return false;
  return cu[n_seg] < (1LL << 30);
}
bool op_attn_args_ok(int dtype, const int64_t* cu, int n_seg, int d, int heads) {
  return (dtype == TCMV_F32 || dtype == TCMV_BF16) && cu_ok(cu, n_seg) && d > 0 && heads > 0 && d % heads == 0;
}

// the launches of tcmv_op_attention; `scratch` holds L.ws_total bytes
int op_attention_run(int dtype, const void* d_qkv, int d, int heads, const OpAttnLayout& L, const void* d_index, void* d_out,
                     uint8_t* scratch, hipStream_t s) {
  const int dh = d / heads;
  const uint8_t* idx = reinterpret_cast<const uint8_t*>(d_index);
  AttnArgs a{};
  a.work = reinterpret_cast<const AttnWork*>(idx + L.work); a.n_work = (int)L.n_work;
  a.heads = heads; a.dh = dh; a.t_total = L.T; a.out = d_out; a.ldo = d;
  a.bq = L.bq;
  hipError_t e;
  if (dtype == TCMV_BF16) {
    const uint16_t* q = reinterpret_cast<const uint16_t*>(d_qkv);
    e = launch_fill_zero(scratch + L.vt, (size_t)d * L.t_vpad * 2, s);
    if (e != hipSuccess) return TCMV_E_HIP;
    e = launch_transpose_v(q + 2 * d, 3 * d, reinterpret_cast<const int32_t*>(idx + L.vcol), scratch + L.vt, L.t_vpad, L.T, d, s);
    if (e != hipSuccess) return TCMV_E_HIP;
    a.q = q; a.k = q + d; a.ldqk = 3 * d; a.v = scratch + L.vt; a.ldv = L.t_vpad;
    a.scale = (float)(1.4426950408889634 / std::sqrt((double)dh));
    a.prescaled = 0;                               // the caller's queries are unscaled
    uint32_t* kmax = reinterpret_cast<uint32_t*>(scratch + L.kmax);
    e = launch_fill_zero(kmax, L.kmax_bytes, s);
    if (e != hipSuccess) return TCMV_E_HIP;
    e = launch_knorm(q + d, 3 * d, L.T, heads, dh, reinterpret_cast<const int32_t*>(idx + L.rseg), kmax, s);
    if (e != hipSuccess) return TCMV_E_HIP;
    a.kmax2 = kmax;
    a.any_left = kmax + L.n_seg * (size_t)heads * kKmaxStride;
    e = launch_attn_bf16(a, s);
  } else {
    const float* q = reinterpret_cast<const float*>(d_qkv);
    a.q = q; a.k = q + d; a.ldqk = 3 * d; a.v = q + 2 * d; a.ldv = 3 * d;
    a.scale = (float)(1.0 / std::sqrt((double)dh));
    e = launch_attn_f32(a, s);
  }
  return e == hipSuccess ? TCMV_OK : TCMV_E_HIP;
}

// shape checks shared by the two attention entry points; fills L
int op_attention_check(int dtype, const void* d_qkv, const int64_t* cu_seqlens, int n_seg, int d, int heads, const void* d_index,
                       const void* d_out, OpAttnLayout* L) {
  if (!op_attn_args_ok(dtype, cu_seqlens, n_seg, d, heads)) return TCMV_E_INVALID_ARG;
  const int dh = d / heads;
  if (dtype == TCMV_BF16 ? !(dh == 32 || dh == 64 || dh == 80 || dh == 96) : (dh % 16 || dh > 128)) return TCMV_E_UNSUPPORTED;
  *L = op_attn_layout(dtype, cu_seqlens, n_seg, d, heads, nullptr, nullptr);
  if (L->T == 0) return TCMV_OK;
  // the kernels keep byte offsets into qkv and into the transposed values in 32 bits
  if ((double)(L->t_vpad + kVtAlign) * 3.0 * (double)d >= 2147483648.0) return TCMV_E_UNSUPPORTED;
  if (!d_qkv || !d_out || !d_index) return TCMV_E_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(d_index) % 256) return TCMV_E_INVALID_ARG;
  return TCMV_OK;
}
}  // namespace

size_t tcmv_op_attention_workspace(int dtype, const int64_t* cu_seqlens, int n_seg, int d, int heads) {
  if (!op_attn_args_ok(dtype, cu_seqlens, n_seg, d, heads)) return 0;
  return op_attn_layout(dtype, cu_seqlens, n_seg, d, heads, nullptr, nullptr).ws_total;
}

size_t tcmv_op_attention_index_bytes(int dtype, const int64_t* cu_seqlens, int n_seg, int d, int heads) {
  if (!op_attn_args_ok(dtype, cu_seqlens, n_seg, d, heads)) return 0;
  return op_attn_layout(dtype, cu_seqlens, n_seg, d, heads, nullptr, nullptr).index_total;
}

int tcmv_op_attention_index(int dtype, const int64_t* cu_seqlens, int n_seg, int d, int heads, void* h_index, size_t index_bytes) {
  if (!op_attn_args_ok(dtype, cu_seqlens, n_seg, d, heads) || !h_index) return TCMV_E_INVALID_ARG;
  std::vector<int32_t> vcol, rseg;
  std::vector<AttnWork> work;
  const OpAttnLayout L = op_attn_layout(dtype, cu_seqlens, n_seg, d, heads, &vcol, &work, &rseg);
  if (index_bytes < L.index_total) return TCMV_E_WORKSPACE_TOO_SMALL;
  uint8_t* h = reinterpret_cast<uint8_t*>(h_index);
  std::memset(h, 0, L.index_total);
  if (!vcol.empty()) std::memcpy(h + L.vcol, vcol.data(), vcol.size() * 4);
  if (!work.empty()) std::memcpy(h + L.work, work.data(), work.size() * sizeof(AttnWork));
  if (!rseg.empty()) std::memcpy(h + L.rseg, rseg.data(), rseg.size() * 4);
  return TCMV_OK;
}

// ---- the attention operator for callers that cannot allocate: its scratch is a fixed array in device memory ----
namespace {
static __device__ __align__(256) unsigned char scratch[TCMV_NOALLOC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
uint8_t* g_scratch_ptr[kMaxDevices] = {};          // device address of each GPU's own copy of `scratch`
std::mutex g_scratch_mu;

// Address of the current device's copy of `scratch` (looked up once per device, with that device current).
int scratch_of_current_device(uint8_t** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return TCMV_E_HIP;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return TCMV_E_HIP;
    g_scratch_ptr[dev] = reinterpret_cast<uint8_t*>(ptr);
  }
  *out = g_scratch_ptr[dev];
  return TCMV_OK;
}
}  // namespace

int tcmv_op_attention_noalloc(int dtype, const void* d_qkv, const int64_t* cu_seqlens, int n_seg, int d, int heads,
                              const void* d_index, void* d_out, void* stream) {
  OpAttnLayout L{};
  const int rc = op_attention_check(dtype, d_qkv, cu_seqlens, n_seg, d, heads, d_index, d_out, &L);
  if (rc != TCMV_OK || L.T == 0) return rc;
  if (L.ws_total > (size_t)TCMV_NOALLOC_SCRATCH_BYTES) return TCMV_E_WORKSPACE_TOO_SMALL;   // beyond the fixed scratch
  uint8_t* ptr = nullptr;
  const int rs = scratch_of_current_device(&ptr);
  if (rs != TCMV_OK) return rs;
  // the kernels zero-fill what they read before writing it (transposed-V padding, key-norm table): the array keeps
  // the previous call's contents
  return op_attention_run(dtype, d_qkv, d, heads, L, d_index, d_out, ptr, (hipStream_t)stream);
}

int tcmv_op_attention(int dtype, const void* d_qkv, const int64_t* cu_seqlens, int n_seg, int d, int heads,
                      const void* d_index, void* d_out, void* d_workspace, size_t workspace_bytes, void* stream) {
  OpAttnLayout L{};
  const int rc = op_attention_check(dtype, d_qkv, cu_seqlens, n_seg, d, heads, d_index, d_out, &L);
  if (rc != TCMV_OK || L.T == 0) return rc;
  if (!d_workspace || reinterpret_cast<uintptr_t>(d_workspace) % 256) return TCMV_E_INVALID_ARG;
  if (workspace_bytes < L.ws_total) return TCMV_E_WORKSPACE_TOO_SMALL;
  return op_attention_run(dtype, d_qkv, d, heads, L, d_index, d_out, reinterpret_cast<uint8_t*>(d_workspace), (hipStream_t)stream);
}

}  // extern "C"
