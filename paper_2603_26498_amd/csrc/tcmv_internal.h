// Internal declarations shared by the host API and the kernel launchers.
// Everything here is private to the library; the public surface is include/tcmv.h.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

namespace tcmv {

// Words between neighbouring entries of the key-norm table: every (segment, head) entry has a 128-byte line (and so an
// L2 channel) to itself; thousands of waves check and raise these words while the QKV projection runs.
constexpr int kKmaxStride = 32;


// ---- device-visible descriptors (plain data, uploaded with a plan) ----------
struct ItemDev {
  const uint8_t* frames;   // [n_frames, src_h, src_w, 3]
  int n_frames, src_h, src_w, dst_h, dst_w;
  int gt, gh, gw;          // token grid
  int resized;             // src size differs from dst size
  int row0;                // first patch row of this request
};

// One unit of preprocessing work of the strip kernel: up to kStripTokens horizontally
// adjacent patches of one patch line of one frame group.  A copied strip (source size ==
// target size) is described completely here, so that a workgroup needs one scalar load
// and no dependent second one before it can request its pixels; a resampled strip also
// reads its request's ItemDev.
struct PreStrip {
  const uint8_t* src;       // copied strips: first byte of the strip in its first source line (first frame of the group)
  int64_t row_base;         // patch row of the strip's first token
  int32_t row_stride;       // bytes between source lines
  int32_t frame_stride;     // bytes between frames
  int32_t ntok;             // tokens of the strip (1..kStripTokens)
  int32_t flags;            // bit 0: still image (its one frame fills the temporal patch), bit 1: resampled
  int32_t item, t, ph, pw0; // request, frame group, patch line, first patch column
};
constexpr int kStripStill = 1, kStripResampled = 2;
constexpr int kStripTokens = 16;

// One unit of attention work: a tile of query rows of one segment.
struct AttnWork {
  int q0;        // first query row (global row index)
  int nq;        // valid query rows in this tile
  int seg_start; // first row of the segment
  int seg_len;   // rows of the segment
  int v0;        // first column of the segment in the transposed-V buffer
  int seg;       // index of the segment (row of the key-norm table)
  int pad_[2];
};

enum Epilogue {
  EPI_STORE = 0,   // C = acc + bias                      (bf16 or fp32 by path)
  EPI_GELU = 1,    // C = gelu(acc + bias)
  EPI_RESID = 2,   // C(fp32) += acc + bias
  EPI_EMBED = 3,   // C(fp32)[dst_row[r]] = acc + bias + position term
  EPI_QKV = 4,     // columns < split: C ; columns >= split: transposed-V buffer
  EPI_GATED = 5,   // columns come in (gate, up) pairs: C[:, j] = silu(gate_j) * up_j   (C has n/2 columns)
  EPI_PARTIAL = 6, // internal: raw fp32 sums of one slice of k into partial[slice][m][n] (see GemmArgs::partial)
  EPI_RESID_AHEAD = 7  // internal: EPI_RESID for outputs too large to stay cached; old values requested one group ahead
};

struct GemmArgs {
  const void* a; int64_t lda;      // [m, k]
  const void* w;                   // [n, k], ld = k
  const float* bias;               // [n] or null
  void* c; int64_t ldc;
  int64_t m; int n; int k;
  int epi;
  // EPI_EMBED
  const int32_t* dst_row; const int32_t* pos_idx; const float* pos0; const float* pos1; int pos_kind;
  // EPI_QKV (bf16 path): q|k columns go to c (ldc), v columns to vt[col - split][vcol[row]]
  int split; void* vt; int64_t ldvt; const int32_t* vcol;
  // EPI_QKV with rotary positions: rope[row][p] = (cos, sin) of pair p of a head, p < rope_dh/2;
  // applied to the columns below split (q and k)
  const float* rope; int rope_dh;
  // EPI_QKV: columns below qcols (the queries) are multiplied by qscale before rounding (0 columns = off)
  int qcols; float qscale;
  // EPI_QKV, optional (see gemm_bf16_can_fuse_key_norms): kmax2[row_seg[r]][h] = max(.., 1.008 * |k row r, head h|^2)
  // over the key columns [qcols, split); kn_dh = head size, kn_heads = heads; float bits, table zeroed by the caller
  uint32_t* kmax2; const int32_t* row_seg; int kn_dh; int kn_heads;   // kmax2: one word per (segment, head), kKmaxStride words apart
  // EPI_RESID with few rows and a long contraction (one small request): when `partial` is given (fp32,
  // room for 4 * m * n values) the launcher may cut k into 4 slices computed by 4 times as many workgroups
  // and add the slices to C in slice order in a second kernel (same result from run to run)
  float* partial; int ksplit;
};

struct AttnArgs {
  const void* q; const void* k; int64_t ldqk;   // row stride (elements) of q and k
  const void* v; int64_t ldv;                    // bf16 path: transposed V [d, ldv]; fp32 path: V rows [T, ldv]
  void* out; int64_t ldo;
  const AttnWork* work; int n_work;
  int heads, dh;
  int bq;                                        // query rows per work item the list was built with (bf16: 128, 256 or 512)
  int64_t t_total;                               // rows of q/k (for clamping)
  float scale;                                   // softmax scale * log2(e); 1 when the queries already carry it
  int prescaled;                                 // bf16 path: the queries already carry the scale
  const uint32_t* kmax2;                         // bf16 path, may be null: [segments][heads] largest squared key norm (float bits)
  uint32_t* any_left;                            // with kmax2, may be null: zeroed word; set when a workgroup needs the reference-tracking copy
  uint32_t* kmax_clear; int n_clear;             // with kmax2, may be null: n_clear words that the first kernel of the launch zeroes
                                                 // (the key-norm block of the next layer)
};

struct PreprocArgs {
  const ItemDev* items;
  const int32_t* prow_item;   // [rows]
  const int32_t* prow_thw;    // [rows] t<<16 | h<<8 | w
  const float* lut;           // [3][256] normalised values (already rounded to the storage type)
  void* patches;              // [rows, k_pad]
  int64_t rows;
  int patch, tpatch, k, k_pad;
  int out_bf16;
  int merge;
  const PreStrip* strips; int n_strips;         // strips staged through LDS: n_copy_strips copied ones first, then the resampled ones
  int n_copy_strips;
  // bf16 output: every table entry equals bf16(fma(v, aff_scale[c], aff_off[c])) (checked by the host for all 768),
  // so the kernel may compute instead of looking up
  int affine; float aff_scale[3], aff_off[3];
  const int32_t* run_rows; int64_t n_run_rows;  // patch rows produced run by run (resampled or unaligned requests)
};

hipError_t launch_preprocess(const PreprocArgs& a, hipStream_t s);
bool preprocess_has_strip_kernel(int patch, int tpatch);
// rms != 0: RMSNorm (no mean subtraction, b is not read)
hipError_t launch_layernorm(const float* x, const float* g, const float* b, void* y, int64_t rows, int d,
                            float eps, int out_bf16, hipStream_t s, int rms = 0);
hipError_t launch_stream_ref(const void* in, size_t in_bytes, void* out, size_t out_bytes, hipStream_t s);
hipError_t launch_gemm_bf16(const GemmArgs& a, hipStream_t s);
// true when launch_gemm_bf16 computes the key-norm maxima in the epilogue of an m x n x k QKV projection whose key
// columns are [qcols, 2 qcols) with heads of dh columns (the wave tiles must line up with the heads)
bool gemm_bf16_can_fuse_key_norms(int64_t m, int n, int k, int qcols, int dh);
hipError_t launch_gemm_f32(const GemmArgs& a, hipStream_t s);
hipError_t launch_attn_bf16(const AttnArgs& a, hipStream_t s);
// windowed layers whose windows hold at most 64 tokens: every work item is one whole window (bf16, prescaled queries)
hipError_t launch_attn_window_bf16(const AttnArgs& a, hipStream_t s);
hipError_t launch_attn_f32(const AttnArgs& a, hipStream_t s);
// vt[c][vcol[r]] = v[r][c] for r < rows, c < d  (bf16)
hipError_t launch_transpose_v(const void* v, int64_t ldv, const int32_t* vcol, void* vt, int64_t ldvt,
                              int64_t rows, int d, hipStream_t s);
// kmax2[row_seg[r]][h] = max(kmax2[..], |k[r, h*dh .. (h+1)*dh)|^2) over all rows (bf16 keys, row stride ldk elements);
// kmax2 holds float bits and must be zero-filled before the call
hipError_t launch_knorm(const void* k, int64_t ldk, int64_t rows, int heads, int dh, const int32_t* row_seg,
                        uint32_t* kmax2, hipStream_t s);
// zero fill of a 16-byte aligned region whose size is a multiple of 16
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s);
// start of an encode on the bf16 path: zeroes the columns [pads[2i], pads[2i+1]) of every row of vt [rows, ldvt]
// (bf16) and n_words 32-bit words at `words`
hipError_t launch_attn_prepare(void* vt, int64_t ldvt, int rows, const int32_t* pads, int n_pads, uint32_t* words,
                               int n_words, hipStream_t s);
// hidden[cls_rows[i]] = cls + pos0[0] (if pos0)
hipError_t launch_cls_rows(float* hidden, const int32_t* cls_rows, int n, const float* cls,
                           const float* pos0, int d, hipStream_t s);

// Tile sizes the host must know about.
constexpr int kAttnBQ_f32 = 64;     // query rows per attention workgroup, fp32 path
constexpr int kAttnBQ_window = 128; // bf16 path, windowed layers (windows are short segments: one query tile per wave)
constexpr int kVtAlign = 64;        // segment starts in the transposed-V buffer are multiples of this

// Column of key r (row inside its segment) in the transposed-V buffer, relative to the
// segment's first column: inside every aligned group of 16 keys the four quarters are
// stored in the order 0, 2, 1, 3 (the order the attention kernel's MFMA operand wants).
inline int64_t vt_col_in_segment(int64_t r) {
  const int64_t kk = r & 15;
  const int64_t q = kk >> 2;
  const int64_t nq = (q == 1) ? 2 : (q == 2 ? 1 : q);
  return (r & ~(int64_t)15) + nq * 4 + (kk & 3);
}

}  // namespace tcmv
