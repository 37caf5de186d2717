// C = epilogue(A * W^T + bias) on bf16 MFMA (gfx950), fp32 accumulation.
//
// A [m, k] and W [n, k] are both contiguous along k, so both operands are staged
// the same way: direct global -> LDS loads (16 bytes per lane, no registers in
// between) into tiles of 64 k-elements per row (128 bytes), with the 16-byte
// chunk index XOR-swizzled by (row/2)%8 so that the per-lane 16-byte MFMA operand
// reads are conflict-free.  LDS is double buffered and the next tile's loads are
// issued before the current tile's MFMAs.  Each wave owns a (BM/WM) x (BN/WN)
// sub-tile built from v_mfma_f32_32x32x16_bf16.
//
// The MFMA is issued with W as the row operand and A as the column operand, so
// the accumulator holds C^T: a lane owns ONE output row (token) and, per 32x32
// tile, four groups of four consecutive output columns.  Written out like that a
// store instruction would touch 32 rows; each wave therefore passes its sub-tile
// through a private LDS buffer (32 rows x 64 columns at a time) and comes back
// with lanes running along the row, 8 consecutive columns per lane: bias /
// position adds, GELU, the gated product, the rotary rotation, the fp32 residual
// read-modify-write and the stores all work on 16 or 32 contiguous bytes per
// lane.  All reads of a group (staged sums, old residual values) are issued
// before the first result is computed, so their round trips overlap instead of
// queueing behind each other.  Only the transposed-V columns of the QKV
// projection leave from registers (consecutive lanes = consecutive tokens = the
// contiguous direction of that buffer).
//
// Large products run on a PERSISTENT kernel: one workgroup of 8 waves per CU walks
// a list of 256x320 (or 256x256) tiles.  While it finishes the k-loop of one tile
// it already requests the first k-tile of its next tile, the tile is written out
// from the stage that is free by then, and the stores drain while the next
// k-loop runs.  Operands are read through buffer descriptors (base and size in
// SGPRs, one 32-bit lane offset per operand, everything else in the scalar
// offset), and the last tile of a dimension is shifted back to end at the matrix
// edge so that no load ever leaves the operand (its repeated rows / columns are
// skipped when it is written out).
// Smaller products use one workgroup per tile: 128x128 (4 waves, two per CU),
// 64x64 (2 waves) for a single small request; a long contraction over few rows
// that accumulates into the residual stream is cut into four slices of k whose
// fp32 partial sums a second kernel adds in slice order.
//
// Workgroups are numbered so that the eight XCDs (workgroup id mod 8) each walk
// a contiguous range of tiles: neighbouring tiles share A rows or W rows in the
// XCD's own L2.
#include <algorithm>
#include <type_traits>
#include "tcmv_internal.h"
#include "device_utils.h"

namespace tcmv {

namespace {
typedef __attribute__((address_space(1))) const void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;
constexpr int kEpStride = 68;                      // floats per row of a wave's staging buffer (64 columns + 4: conflict-free)
constexpr int kEpWaveBytes = 32 * kEpStride * 4;   // staging bytes per wave
}  // namespace

// Lane exchanges inside a row of 16 lanes through the data-parallel path of the vector ALU (no LDS round trip):
// value of lane (l ^ 1), lane (l ^ 2), lane (l + 4), lane (l + 8); lanes that would read past the row get 0.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}
__device__ __forceinline__ float lane_xor1(float v) { return dpp_move<0xB1>(v); }   // quad_perm [1,0,3,2]
__device__ __forceinline__ float lane_xor2(float v) { return dpp_move<0x4E>(v); }   // quad_perm [2,3,0,1]
__device__ __forceinline__ float lane_up4(float v) { return dpp_move<0x104>(v); }   // row_shl:4
__device__ __forceinline__ float lane_up8(float v) { return dpp_move<0x108>(v); }   // row_shl:8

// Rows and columns of the output that a workgroup may write: [row_lo, row_hi) x [col_lo, col_hi).
struct TileBounds { int64_t row_lo, row_hi; int col_lo, col_hi; int slice; };

// Writes one wave's sub-tile (MI x NI accumulator tiles of 32 x 32, first row m_base, first column wcol0).  In the
// accumulator a lane holds row (lane & 31) and columns 8*(v/4) + 4*(lane>>5) + v%4 of each tile.  The sub-tile
// leaves through the wave's private LDS buffer `ep` (32 rows x 64 columns of fp32 at a time) and comes back with
// lanes running along the rows, 8 consecutive columns per lane.  FULL: every element is inside the bounds.
//
// Key-norm maxima (EPI_QKV with g.kmax2, wave tiles of key columns that hold whole heads): on their way out the
// lanes square and sum their 8 values, the lanes of a row are added per head in a fixed order, and one lane per row
// accumulates the sums in the four spare floats at the end of the row's line in the staging buffer.  After the
// last column group of a 32-row block, the largest row of each segment goes to kmax2[segment][head] (the sums are
// >= 0, so their float bits order like unsigned integers).  The sums are taken before the rotary rotation (which
// preserves the norm of every pair) and before rounding to bf16 (which changes a squared norm by less than 2^-7 of
// itself): the factor 1.008 keeps the result an upper bound of the norm of the stored keys.
template <int EPI, int MI, int NI, bool FULL>
__device__ __forceinline__ void wave_epilogue(f32x16 (&acc)[MI][NI], const GemmArgs& g, float* ep, int64_t m_base, int wcol0,
                                              int lane, const TileBounds& tb) {
  constexpr int EPS = kEpStride;
  constexpr int TN = NI * 32;
  const int lr = lane & 31, lg = lane >> 5;
  const bool kn = EPI == EPI_QKV && g.kmax2 != nullptr && wcol0 >= g.qcols && wcol0 < g.split;
  // old values of a group of the output (residual epilogues)
  auto load_old = [&](auto ngc, int nb, int64_t rbase, float4 (&o)[4][2]) {
    constexpr int NGT = decltype(ngc)::value;
    constexpr int LPR = NGT * 4, RPP = 64 / LPR, NP = 32 / RPP;
    const int col = wcol0 + nb * 32 + (lane % LPR) * 8;
    const int r0 = lane / LPR;
    const bool col_ok = FULL || (col >= tb.col_lo && col < tb.col_hi);
#pragma unroll
    for (int ps = 0; ps < NP; ++ps) {
      const int64_t row = rbase + ps * RPP + r0;
      if (FULL || (row >= tb.row_lo && row < tb.row_hi && col_ok)) {
        const float4* c = reinterpret_cast<const float4*>(reinterpret_cast<const float*>(g.c) + (size_t)row * g.ldc + col);
        o[ps][0] = c[0]; o[ps][1] = c[1];
      }
    }
  };
  // `ahead` (EPI_RESID_AHEAD): old values of this group, requested while the previous group was written out;
  // `prefetch` requests those of the next group once this group's accumulators are in LDS and their registers free
  auto flush = [&](auto ngc, int mi, int nb, int64_t rbase, float4 (&ahead)[4][2], auto&& prefetch) {
    constexpr int NGT = decltype(ngc)::value;
    constexpr int LPR = NGT * 4;                   // lanes per row (8 columns each)
    constexpr int RPP = 64 / LPR;                  // rows per pass
    constexpr int NP = 32 / RPP;                   // passes
    const int c8 = (lane % LPR) * 8;
    const int col = wcol0 + nb * 32 + c8;
    const int r0 = lane / LPR;
    const bool col_ok = FULL || (col >= tb.col_lo && col < tb.col_hi);
    float4 here[4][2];
    if (EPI == EPI_RESID) load_old(ngc, nb, rbase, here);
    float4 (&o)[4][2] = EPI == EPI_RESID_AHEAD ? ahead : here;
#pragma unroll
    for (int ni = 0; ni < NGT; ++ni)
#pragma unroll
      for (int vq = 0; vq < 4; ++vq)
        *reinterpret_cast<float4*>(ep + lr * EPS + ni * 32 + 8 * vq + 4 * lg) =
            make_float4(acc[mi][nb + ni][4 * vq], acc[mi][nb + ni][4 * vq + 1], acc[mi][nb + ni][4 * vq + 2], acc[mi][nb + ni][4 * vq + 3]);
    prefetch();
    float4 b0 = make_float4(0.f, 0.f, 0.f, 0.f), b1 = b0;
    if (EPI != EPI_PARTIAL && g.bias && col_ok) { b0 = *reinterpret_cast<const float4*>(g.bias + col); b1 = *reinterpret_cast<const float4*>(g.bias + col + 4); }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    // plain stores read all staged values of the group first; the epilogues that keep other values in registers
    // (old residual values, rotary factors, key-norm sums) read them pass by pass
    constexpr bool BATCH = EPI == EPI_STORE || EPI == EPI_GELU || EPI == EPI_GATED || EPI == EPI_PARTIAL;
    float4 v[NP][2];
    if (BATCH) {
#pragma unroll
      for (int ps = 0; ps < NP; ++ps) {
        const int r = ps * RPP + r0;
        v[ps][0] = *reinterpret_cast<const float4*>(ep + r * EPS + c8);
        v[ps][1] = *reinterpret_cast<const float4*>(ep + r * EPS + c8 + 4);
      }
    }
    if (EPI == EPI_QKV && kn) {
      // this group's share of the squared key norms: per row, the lanes of the first head of the group and the
      // lanes of the second (a group of 64 columns meets at most two heads of 64 or more columns)
      const int h_first = (nb * 32) / g.kn_dh;
      const bool second = (nb * 32 + c8) / g.kn_dh != h_first;
#pragma unroll
      for (int ps = 0; ps < NP; ++ps) {
        const int r = ps * RPP + r0;
        const int64_t row = rbase + r;
        const bool ok = FULL || (row >= tb.row_lo && row < tb.row_hi && col_ok);
        const float4 va = *reinterpret_cast<const float4*>(ep + r * EPS + c8), vb = *reinterpret_cast<const float4*>(ep + r * EPS + c8 + 4);
        const float y[8] = {va.x + b0.x, va.y + b0.y, va.z + b0.z, va.w + b0.w, vb.x + b1.x, vb.y + b1.y, vb.z + b1.z, vb.w + b1.w};
        float sq = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) sq = fmaf(y[j], y[j], sq);
        if (!ok) sq = 0.f;
        float s0 = second ? 0.f : sq, s1 = second ? sq : 0.f;
        // sums over the LPR (4 or 8) lanes of a row, in a fixed order; valid in the first lane of the row
        s0 += lane_xor1(s0); s1 += lane_xor1(s1);
        s0 += lane_xor2(s0); s1 += lane_xor2(s1);
        if (LPR == 8) { s0 += lane_up4(s0); s1 += lane_up4(s1); }
        if (lane % LPR == 0) {
          float* acc2 = ep + r * EPS + 64 + h_first;
          acc2[0] += s0;
          if ((nb * 32 + NGT * 32 - 1) / g.kn_dh != h_first) acc2[1] += s1;
        }
      }
    }
#pragma unroll
    for (int ps = 0; ps < NP; ++ps) {
      const int64_t row = rbase + ps * RPP + r0;
      if (!FULL && (row < tb.row_lo || row >= tb.row_hi || !col_ok)) continue;
      if (!BATCH) {
        const int r = ps * RPP + r0;
        v[ps][0] = *reinterpret_cast<const float4*>(ep + r * EPS + c8);
        v[ps][1] = *reinterpret_cast<const float4*>(ep + r * EPS + c8 + 4);
      }
      float x[8] = {v[ps][0].x + b0.x, v[ps][0].y + b0.y, v[ps][0].z + b0.z, v[ps][0].w + b0.w,
                    v[ps][1].x + b1.x, v[ps][1].y + b1.y, v[ps][1].z + b1.z, v[ps][1].w + b1.w};
      if (EPI == EPI_GATED) {
        uint2 pk;
        float h[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) h[j] = x[2 * j] / (1.0f + __expf(-x[2 * j])) * x[2 * j + 1];
        pk.x = pack_bf16x2(h[0], h[1]); pk.y = pack_bf16x2(h[2], h[3]);
        *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(g.c) + (size_t)row * g.ldc + (col >> 1)) = pk;
      } else if (EPI == EPI_STORE || EPI == EPI_GELU || EPI == EPI_QKV) {
        if (EPI == EPI_QKV && col >= g.split) continue;
        if (EPI == EPI_QKV && col < g.qcols) {
#pragma unroll
          for (int j = 0; j < 8; ++j) x[j] *= g.qscale;
        }
        if (EPI == EPI_QKV && g.rope) {
          const int p2 = ((col % g.rope_dh) >> 1) * 2;
          const float4* cs = reinterpret_cast<const float4*>(g.rope + (size_t)row * g.rope_dh + p2);
          const float4 c0 = cs[0], c1 = cs[1];
          const float a0 = x[0], a1 = x[1], a2 = x[2], a3 = x[3], a4 = x[4], a5 = x[5], a6 = x[6], a7 = x[7];
          x[0] = a0 * c0.x - a1 * c0.y; x[1] = a0 * c0.y + a1 * c0.x;
          x[2] = a2 * c0.z - a3 * c0.w; x[3] = a2 * c0.w + a3 * c0.z;
          x[4] = a4 * c1.x - a5 * c1.y; x[5] = a4 * c1.y + a5 * c1.x;
          x[6] = a6 * c1.z - a7 * c1.w; x[7] = a6 * c1.w + a7 * c1.z;
        }
        if (EPI == EPI_GELU) {
#pragma unroll
          for (int j = 0; j < 8; ++j) x[j] = gelu_bf16(x[j]);
        }
        uint4 pk;
        pk.x = pack_bf16x2(x[0], x[1]); pk.y = pack_bf16x2(x[2], x[3]); pk.z = pack_bf16x2(x[4], x[5]); pk.w = pack_bf16x2(x[6], x[7]);
        *reinterpret_cast<uint4*>(reinterpret_cast<uint16_t*>(g.c) + (size_t)row * g.ldc + col) = pk;
      } else if (EPI == EPI_PARTIAL) {
        float4* c = reinterpret_cast<float4*>(g.partial + ((size_t)tb.slice * g.m + row) * g.n + col);
        c[0] = make_float4(x[0], x[1], x[2], x[3]);
        c[1] = make_float4(x[4], x[5], x[6], x[7]);
      } else if (EPI == EPI_RESID || EPI == EPI_RESID_AHEAD) {
        float4* c = reinterpret_cast<float4*>(reinterpret_cast<float*>(g.c) + (size_t)row * g.ldc + col);
        c[0] = make_float4(o[ps][0].x + x[0], o[ps][0].y + x[1], o[ps][0].z + x[2], o[ps][0].w + x[3]);
        c[1] = make_float4(o[ps][1].x + x[4], o[ps][1].y + x[5], o[ps][1].z + x[6], o[ps][1].w + x[7]);
      } else if (EPI == EPI_EMBED) {
        const int pi = g.pos_idx ? g.pos_idx[row] : 0;
        if (g.pos_kind == 1) {
          const float4* p0 = reinterpret_cast<const float4*>(g.pos0 + (size_t)pi * g.n + col);
          const float4 pa = p0[0], pb = p0[1];
          x[0] += pa.x; x[1] += pa.y; x[2] += pa.z; x[3] += pa.w; x[4] += pb.x; x[5] += pb.y; x[6] += pb.z; x[7] += pb.w;
        } else if (g.pos_kind == 2) {
          const float4* p0 = reinterpret_cast<const float4*>(g.pos0 + (size_t)(pi & 0xFFFF) * g.n + col);
          const float4* p1 = reinterpret_cast<const float4*>(g.pos1 + (size_t)(pi >> 16) * g.n + col);
          const float4 pa = p0[0], pb = p0[1], qa = p1[0], qb = p1[1];
          x[0] += pa.x + qa.x; x[1] += pa.y + qa.y; x[2] += pa.z + qa.z; x[3] += pa.w + qa.w;
          x[4] += pb.x + qb.x; x[5] += pb.y + qb.y; x[6] += pb.z + qb.z; x[7] += pb.w + qb.w;
        }
        const int64_t dst = g.dst_row ? (int64_t)g.dst_row[row] : row;
        float4* c = reinterpret_cast<float4*>(reinterpret_cast<float*>(g.c) + (size_t)dst * g.ldc + col);
        c[0] = make_float4(x[0], x[1], x[2], x[3]);
        c[1] = make_float4(x[4], x[5], x[6], x[7]);
      }
    }
    asm volatile("" ::: "memory");
  };

  if constexpr (EPI == EPI_RESID_AHEAD) {
    // Outputs that do not stay cached between the kernels that update them (hundreds of megabytes of residual stream):
    // all groups of the wave tile in one sequence, the old values of group i+1 on their way while group i is written out.
    // It costs registers (two sets of old values; the compiler spills a few dozen), which is why outputs that do stay
    // cached keep the plain form: measured 14 % faster on fc2 at 100 k tokens (0.5 GB), 1 - 3 % slower at 32 k and 65 k
    // tokens (0.17 and 0.34 GB), hence the launcher's threshold of 0.4 GB.
    constexpr int G = NI / 2 + (NI & 1);           // groups per 32-row block: pairs of 32-column tiles, then a single one
    float4 oa[4][2], ob[4][2];
    load_old(std::integral_constant<int, (NI >= 2 ? 2 : 1)>{}, 0, m_base, oa);
    static_for<MI * G>([&](auto gc) {
      constexpr int gi = decltype(gc)::value;
      constexpr int mi = gi / G, k = gi % G, nb = 2 * k, NGT = (nb + 2 <= NI) ? 2 : 1;
      auto pre = [&]() {
        if constexpr (gi + 1 < MI * G) {
          constexpr int mi2 = (gi + 1) / G, k2 = (gi + 1) % G, nb2 = 2 * k2, NGT2 = (nb2 + 2 <= NI) ? 2 : 1;
          if constexpr (gi % 2 == 0) load_old(std::integral_constant<int, NGT2>{}, nb2, m_base + mi2 * 32, ob);
          else load_old(std::integral_constant<int, NGT2>{}, nb2, m_base + mi2 * 32, oa);
        }
      };
      if constexpr (gi % 2 == 0) flush(std::integral_constant<int, NGT>{}, mi, nb, m_base + mi * 32, oa, pre);
      else flush(std::integral_constant<int, NGT>{}, mi, nb, m_base + mi * 32, ob, pre);
    });
    return;
  }
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) {
    const int64_t rbase = m_base + mi * 32;
    if (EPI == EPI_QKV && kn && lane < 32) *reinterpret_cast<float4*>(ep + lane * EPS + 64) = make_float4(0.f, 0.f, 0.f, 0.f);
    if (EPI == EPI_QKV && wcol0 + TN > g.split) {
      const int64_t row = rbase + lr;
      if (FULL || (row >= tb.row_lo && row < tb.row_hi)) {
        const int vc = g.vcol[row];
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
          for (int vq = 0; vq < 4; ++vq) {
            const int col = wcol0 + ni * 32 + 8 * vq + 4 * lg;
            if (col >= g.split && (FULL || (col >= tb.col_lo && col < tb.col_hi))) {
              float4 b4 = make_float4(0.f, 0.f, 0.f, 0.f);
              if (g.bias) b4 = *reinterpret_cast<const float4*>(g.bias + col);
              uint16_t* vt = reinterpret_cast<uint16_t*>(g.vt) + (size_t)(col - g.split) * g.ldvt + vc;
              vt[0] = f32_to_bf16(acc[mi][ni][4 * vq] + b4.x);
              vt[g.ldvt] = f32_to_bf16(acc[mi][ni][4 * vq + 1] + b4.y);
              vt[2 * g.ldvt] = f32_to_bf16(acc[mi][ni][4 * vq + 2] + b4.z);
              vt[3 * g.ldvt] = f32_to_bf16(acc[mi][ni][4 * vq + 3] + b4.w);
            }
          }
      }
      if (wcol0 >= g.split) continue;
    }
    {
      float4 none[4][2];
#pragma unroll
      for (int nb = 0; nb + 2 <= NI; nb += 2) flush(std::integral_constant<int, 2>{}, mi, nb, rbase, none, [] {});
      if (NI & 1) flush(std::integral_constant<int, 1>{}, mi, NI - 1, rbase, none, [] {});
    }
    if (EPI == EPI_QKV && kn) {
      // rows of this block -> table.  Lane l < 32 reads the sums of row l (up to four heads per wave tile).
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      const float4 sums = *reinterpret_cast<const float4*>(ep + lr * EPS + 64);
      const float hs[4] = {sums.x, sums.y, sums.z, sums.w};
      const int64_t row = rbase + lr;
      const bool row_ok = FULL || (row >= tb.row_lo && row < tb.row_hi);
      const int seg = row_ok ? g.row_seg[row] : -1;
      const int seg_a = __builtin_amdgcn_readlane(seg, 0), seg_b = __builtin_amdgcn_readlane(seg, 31);
      const bool one_segment = __all(row_ok) && seg_a == seg_b;        // rows are ordered by segment
      const int head0 = (wcol0 - g.qcols) / g.kn_dh;
      const int nh = TN / g.kn_dh;
      // all table words of the block are read before any is compared: one memory round trip per block, not one per head
      uint32_t bits[4] = {0u, 0u, 0u, 0u}, seen[4] = {0u, 0u, 0u, 0u};
      const bool writer = one_segment ? lane == 0 : (row_ok && lg == 0);
      uint32_t* word = g.kmax2 + ((size_t)(one_segment ? seg_a : (row_ok ? seg : 0)) * g.kn_heads + head0) * kKmaxStride;
#pragma unroll
      for (int h = 0; h < 4; ++h) {
        if (h < nh) {
          float vmax = hs[h] * 1.008f;
          if (one_segment) {
            // largest of the 32 rows (lanes 0..31): inside each row of 16 lanes, then lanes 0 and 16
            vmax = fmaxf(vmax, lane_xor1(vmax));
            vmax = fmaxf(vmax, lane_xor2(vmax));
            vmax = fmaxf(vmax, lane_up4(vmax));
            vmax = fmaxf(vmax, lane_up8(vmax));
            vmax = fmaxf(__builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, vmax), 0)),
                         __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, vmax), 16)));
          }
          bits[h] = __float_as_uint(vmax);
          if (writer) seen[h] = __hip_atomic_load(word + h * kKmaxStride, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
      }
      // *p = max(*p, v).  Thousands of waves update the few words of one table: the atomic is only issued when the
      // word, as this wave has just seen it, is smaller (a stale view only costs an atomic that changes nothing),
      // which leaves a handful of atomics per word instead of one per wave queued behind each other.
#pragma unroll
      for (int h = 0; h < 4; ++h)
        if (h < nh && writer && seen[h] < bits[h]) atomicMax(word + h * kKmaxStride, bits[h]);
    }
  }
}


template <int BM, int BN, int WM, int WN, int BK, int NSTAGE, int MINB, int EPI>
__global__ __launch_bounds__(WM* WN * 64, MINB) void gemm_bf16_kernel(GemmArgs g) {
  constexpr int TM = BM / WM, TN = BN / WN, MI = TM / 32, NI = TN / 32;
  constexpr int ROWB = BK * 2;                     // bytes per staged row
  constexpr int CPR = BK / 8;                      // 16-byte chunks per row (8 or 4)
  constexpr int SW_SHIFT = (CPR == 8) ? 1 : 2;     // rows that share a swizzle value (span 256 bytes = all banks)
  constexpr int RPL = 64 / CPR;                    // rows covered by one wave-wide load
  static_assert(BK == 64 || BK == 32, "BK");
  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
  constexpr int A_BYTES = BM * ROWB, B_BYTES = BN * ROWB, STAGE = A_BYTES + B_BYTES;

  const int tiles_n = (g.n + BN - 1) / BN;
  const int tiles_m = (int)((g.m + BM - 1) / BM);
  const int nslice = (EPI == EPI_PARTIAL) ? g.ksplit : 1;   // slices of k (neighbouring workgroups take the slices of a tile)
  const int total = tiles_m * tiles_n * nslice;
  const int chunk = (total + 7) >> 3;
  const int pq = (int)(blockIdx.x & 7) * chunk + (int)(blockIdx.x >> 3);
  if (pq >= total) return;
  const int p = pq / nslice, slice = pq - p * nslice;
  // tiles are walked in groups of GM rows of tiles, column by column inside a group: the
  // workgroups that run at the same time on one XCD then form a roughly square block of
  // tiles and share both A rows and W rows in that XCD's L2
  constexpr int GM = 8;
  const int per_group = GM * tiles_n;
  const int grp = p / per_group, within = p - grp * per_group;
  const int gm_eff = min(GM, tiles_m - grp * GM);
  const int tn = within / gm_eff;
  const int tm = grp * GM + (within - tn * gm_eff);
  const int64_t m0 = (int64_t)tm * BM;
  const int n0 = tn * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const uint16_t* A = reinterpret_cast<const uint16_t*>(g.a);
  const uint16_t* W = reinterpret_cast<const uint16_t*>(g.w);

  // Tile staging: global -> LDS directly.  One wave-wide load writes 64 consecutive
  // 16-byte chunks (RPL rows) of the stage; each lane fetches the global chunk that
  // belongs at its swizzled LDS position.  Rows past the end of the operand are
  // clamped to its last row (they only feed outputs that are never stored).
  constexpr int WAVES = WM * WN;
  constexpr int NLA = BM / RPL / WAVES, NLB = BN / RPL / WAVES;      // wave-loads per wave and k-tile
  static_assert(BM % (RPL * WAVES) == 0 && BN % (RPL * WAVES) == 0, "tile/waves mismatch");
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  uint32_t offa[NLA], offb[NLB];
  {
    const int rl = lane / CPR, pc = lane % CPR;
#pragma unroll
    for (int i = 0; i < NLA; ++i) {
      const int row = (wave_u + WAVES * i) * RPL + rl;
      int64_t gr = m0 + row;
      if (gr > g.m - 1) gr = g.m - 1;
      offa[i] = (uint32_t)(gr * g.lda) + ((pc ^ ((row >> SW_SHIFT) & (CPR - 1))) << 3);
    }
#pragma unroll
    for (int i = 0; i < NLB; ++i) {
      const int row = (wave_u + WAVES * i) * RPL + rl;
      int gn = n0 + row;
      if (gn > g.n - 1) gn = g.n - 1;
      offb[i] = (uint32_t)gn * (uint32_t)g.k + ((pc ^ ((row >> SW_SHIFT) & (CPR - 1))) << 3);
    }
  }
  const int nk = g.k / BK / nslice;               // k-tiles of this workgroup
  const int k_first = slice * nk;
  auto load_tiles = [&](int kt, int buf) {
    uint8_t* sa = smem + buf * STAGE;
    uint8_t* sb = sa + A_BYTES;
    const uint16_t* ak = A + (size_t)(k_first + kt) * BK;
    const uint16_t* wk = W + (size_t)(k_first + kt) * BK;
#pragma unroll
    for (int i = 0; i < NLA; ++i)
      __builtin_amdgcn_global_load_lds((gptr_t)(ak + offa[i]), (lptr_t)(sa + (wave_u + WAVES * i) * 1024), 16, 0, 0);
#pragma unroll
    for (int i = 0; i < NLB; ++i)
      __builtin_amdgcn_global_load_lds((gptr_t)(wk + offb[i]), (lptr_t)(sb + (wave_u + WAVES * i) * 1024), 16, 0, 0);
  };

  f32x16 acc[MI][NI];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;

  // Two LDS stages.  The barrier of a k-tile sits before its LAST k-step, not before its first: by then every
  // wave has read all of the tile's fragments into registers (so the tile's stage can be refilled with tile
  // kt+2 right after the barrier) and tile kt+1, requested a tile earlier, has had three quarters of an
  // iteration to land.  After the barrier a wave asks for the first fragments of tile kt+1 and then still has
  // the MFMAs of the last k-step of tile kt to issue, so no wave sits behind a barrier with nothing to do while
  // its fragments travel.
  static_assert(NSTAGE == 2 && BK / 16 >= 2, "the k-loop is written for two stages");
  const int lr = lane & 31, lg = lane >> 5;
  bf16x8 af[2][MI], bfr[2][NI];        // fragments double-buffered in registers
  auto frags = [&](int stage, int kk, int b) {
    const uint8_t* sa = smem + stage * STAGE;
    const uint8_t* sb = sa + A_BYTES;
    const int ch = kk * 2 + lg;
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
      const int row = wm * TM + mi * 32 + lr;
      af[b][mi] = *reinterpret_cast<const bf16x8*>(sa + row * ROWB + ((ch ^ ((row >> SW_SHIFT) & (CPR - 1))) << 4));
    }
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
      const int row = wn * TN + ni * 32 + lr;
      bfr[b][ni] = *reinterpret_cast<const bf16x8*>(sb + row * ROWB + ((ch ^ ((row >> SW_SHIFT) & (CPR - 1))) << 4));
    }
  };
  auto mfmas = [&](int b) {
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[b][ni], af[b][mi], acc[mi][ni], 0, 0, 0);
  };
  constexpr int KK = BK / 16;
  load_tiles(0, 0);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();                     // tile 0 visible to all waves
  if (1 < nk) load_tiles(1, 1);
  frags(0, 0, 0);
  // mode 2: tile kt+2 exists and is requested; 1: tile kt+1 is the last; 0: tile kt is the last
  auto iteration = [&](int kt, auto mode_c) {
    constexpr int MODE = decltype(mode_c)::value;
    const int cur = kt & 1;
#pragma unroll
    for (int kk = 0; kk + 1 < KK; ++kk) {
      frags(cur, kk + 1, (kk + 1) & 1);
      mfmas(kk & 1);
      {
        // issue order of this k-step: one LDS read after each MFMA while reads are left, then the other MFMAs
        // (instead of all reads first): 2-5 % on the large products
        constexpr int NR = MI + NI, NM = MI * NI;
#pragma unroll
        for (int i = 0; i < NR; ++i) {
          if (i < NM) __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        if (NM > NR) __builtin_amdgcn_sched_group_barrier(0x008, NM - NR, 0);
      }
    }
    if (MODE >= 1) {
      asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
      __syncthreads();
      if (MODE == 2) load_tiles(kt + 2, cur);
      frags(cur ^ 1, 0, KK & 1);
    }
    mfmas((KK - 1) & 1);
    if (MODE >= 1) {
      // after the barrier: an MFMA first, then the tile loads and fragment reads one by one between the MFMAs
      constexpr int NR = MI + NI, NM = MI * NI, NV = (MODE == 2) ? NLA + NLB : 0;
#pragma unroll
      for (int i = 0; i < NM; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        if (i < NV) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        if (i < NR) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
    }
  };
  {
    int kt = 0;
    for (; kt + 2 < nk; ++kt) iteration(kt, std::integral_constant<int, 2>{});
    if (kt + 1 < nk) { iteration(kt, std::integral_constant<int, 1>{}); ++kt; }
    iteration(kt, std::integral_constant<int, 0>{});
  }

  // ---- epilogue: through the operand stages, which every wave has finished with
  static_assert(WAVES * kEpWaveBytes <= NSTAGE * STAGE, "epilogue staging does not fit in the operand stages");
  __syncthreads();
  {
    float* ep = reinterpret_cast<float*>(smem + wave * kEpWaveBytes);
    const TileBounds tb{0, g.m, 0, g.n, slice};
    const int64_t m_base = m0 + wm * TM;
    const int wcol0 = n0 + wn * TN;
    if (m0 + BM <= g.m && n0 + BN <= g.n) wave_epilogue<EPI, MI, NI, true>(acc, g, ep, m_base, wcol0, lane, tb);
    else wave_epilogue<EPI, MI, NI, false>(acc, g, ep, m_base, wcol0, lane, tb);
  }
}

template <int BM, int BN, int WM, int WN, int BK, int NSTAGE, int MINB>
static hipError_t launch_cfg(const GemmArgs& a, hipStream_t s) {
  const int tiles_n = (a.n + BN - 1) / BN;
  const int64_t tiles_m = (a.m + BM - 1) / BM;
  const int64_t total = tiles_m * tiles_n * (a.epi == EPI_PARTIAL ? a.ksplit : 1);
  if (total <= 0) return hipSuccess;
  if (total > (1 << 30)) return hipErrorInvalidValue;
  const unsigned grid = (unsigned)(((total + 7) / 8) * 8);
  const size_t lds = (size_t)NSTAGE * (BM + BN) * BK * 2;
  dim3 block(WM * WN * 64);
#define TCMV_GEMM_CASE(E)                                                                              \
  case E: {                                                                                            \
    auto kern = gemm_bf16_kernel<BM, BN, WM, WN, BK, NSTAGE, MINB, E>;                                 \
    if (lds > 64 * 1024) {                                                                             \
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                          \
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);        \
      if (e != hipSuccess) return e;                                                                   \
    }                                                                                                  \
    hipLaunchKernelGGL(kern, dim3(grid), block, lds, s, a);                                            \
    break;                                                                                             \
  }
  switch (a.epi) {
    TCMV_GEMM_CASE(EPI_STORE) TCMV_GEMM_CASE(EPI_GELU) TCMV_GEMM_CASE(EPI_RESID)
    TCMV_GEMM_CASE(EPI_EMBED) TCMV_GEMM_CASE(EPI_QKV) TCMV_GEMM_CASE(EPI_GATED) TCMV_GEMM_CASE(EPI_PARTIAL)
    default: return hipErrorInvalidValue;
  }
#undef TCMV_GEMM_CASE
  return hipGetLastError();
}

// C += bias + slice 0 + slice 1 + ... (in this order), 16 bytes per lane
__global__ __launch_bounds__(256) void splitk_reduce_kernel(float* c, int64_t ldc, const float* partial, const float* bias,
                                                            int64_t m, int n, int nslice) {
  const int n4 = n >> 2;
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= m * n4) return;
  const int64_t row = i / n4;
  const int col = (int)(i - row * n4) * 4;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  if (bias) acc = *reinterpret_cast<const float4*>(bias + col);
  for (int sl = 0; sl < nslice; ++sl) {
    const float4 v = *reinterpret_cast<const float4*>(partial + ((size_t)sl * m + row) * n + col);
    acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
  }
  float4* dst = reinterpret_cast<float4*>(c + (size_t)row * ldc + col);
  float4 old = *dst;
  old.x += acc.x; old.y += acc.y; old.z += acc.z; old.w += acc.w;
  *dst = old;
}

// One wave-wide 16-byte-per-lane load global -> LDS through a buffer descriptor over `bytes` bytes at `base` (base,
// size and `soff` are wave-uniform and live in SGPRs; `voff` is the lane's byte offset).  Lane l writes 16 bytes
// at lds + 16 l.
__device__ __forceinline__ void buffer_load_lds16(const void* base, uint32_t bytes, void* lds, uint32_t voff, uint32_t soff) {
  const uint64_t v = reinterpret_cast<uint64_t>(base);
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<void*>(((uint64_t)hi << 32) | lo), 0,
                                                                      (int)__builtin_amdgcn_readfirstlane(bytes), 0x00020000);
  __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lptr_t)lds, 16, voff, soff, 0, 0);
}

template <int BM, int BN, int WM, int WN, int EPI>
__global__ __launch_bounds__(WM* WN * 64, 1) void gemm_bf16_persist_kernel(GemmArgs g) {
  constexpr int BK = 64, TM = BM / WM, TN = BN / WN, MI = TM / 32, NI = TN / 32;
  constexpr int ROWB = BK * 2, CPR = 8, RPL = 8, WAVES = WM * WN, KK = BK / 16;
  constexpr int A_BYTES = BM * ROWB, B_BYTES = BN * ROWB, STAGE = A_BYTES + B_BYTES;
  constexpr int EP_WAVE = kEpWaveBytes, EP_BYTES = WAVES * EP_WAVE;
  constexpr int EXTRA = EP_BYTES > STAGE ? (EP_BYTES - STAGE + 255) / 256 * 256 : 0;
  constexpr int NLA = BM / RPL / WAVES, NLB = BN / RPL / WAVES;
  static_assert(BM % (RPL * WAVES) == 0 && BN % (RPL * WAVES) == 0, "tile/waves mismatch");
  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];      // [stage 0][extra][stage 1]

  const int tiles_n = (g.n + BN - 1) / BN;
  const int tiles_m = (int)((g.m + BM - 1) / BM);
  const int total = tiles_m * tiles_n;
  const int chunk = (total + 7) >> 3;
  const int xcd = (int)(blockIdx.x & 7), slot = (int)(blockIdx.x >> 3), nslot = (int)(gridDim.x >> 3);
  int pq = xcd * chunk + slot;
  const int pq_end = min((xcd + 1) * chunk, total);
  if (pq >= pq_end) return;
  constexpr int GM = 8;
  auto tile_of = [&](int p, int& tm, int& tn) {
    const int per_group = GM * tiles_n;
    const int grp = p / per_group, within = p - grp * per_group;
    const int gm_eff = min(GM, tiles_m - grp * GM);
    tn = within / gm_eff;
    tm = grp * GM + (within - tn * gm_eff);
  };

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  const int wm = wave_u / WN, wn = wave_u % WN;
  const uint16_t* A = reinterpret_cast<const uint16_t*>(g.a);
  const uint16_t* W = reinterpret_cast<const uint16_t*>(g.w);
  const int nk = g.k / BK;

  // sizes of the operands in bytes (below 2^32: checked by the launcher)
  const uint32_t bytes_a = (uint32_t)(((uint64_t)(g.m - 1) * (uint64_t)g.lda + (uint64_t)g.k) * 2ull);
  const uint32_t bytes_w = (uint32_t)((uint64_t)g.n * (uint64_t)g.k * 2ull);
  // Tile loads: lane l of a wave-wide load fetches 16 bytes of row l/8 of an 8-row slab; the slab's first row, the
  // k offset and the slab index go into the scalar offset of the instruction, so one VGPR per operand is enough.
  // The last tile of a dimension is shifted back to end at the matrix edge (its first rows / columns then repeat
  // the previous tile's and are skipped when the tile is written out), so every load stays inside the operand.
  const int rl = lane / CPR, pc = lane % CPR;
  const int swz = ((rl >> 1) + 4 * (wave_u & 1)) & 7;            // (row >> 1) & 7 for row = (wave + 8 i) * 8 + rl
  const uint32_t lane_a = (uint32_t)rl * (uint32_t)g.lda * 2u + ((pc ^ swz) << 4);
  const uint32_t lane_w = (uint32_t)rl * (uint32_t)g.k * 2u + ((pc ^ swz) << 4);
  uint32_t tile_a = 0, tile_w = 0;                               // byte offset of the tile's first row (scalars)
  int row_lo = 0, col_lo = 0;                                    // first row / column this tile owns
  int64_t m0 = 0; int n0 = 0;
  auto set_tile = [&](int tm_, int tn_) {
    row_lo = tm_ * BM; col_lo = tn_ * BN;
    m0 = min((int64_t)row_lo, g.m - BM); n0 = min(col_lo, g.n - BN);
    tile_a = (uint32_t)(m0 * g.lda) * 2u;
    tile_w = (uint32_t)n0 * (uint32_t)g.k * 2u;
  };
  auto stage_ptr = [&](int s) { return smem + (s ? STAGE + EXTRA : 0); };
  auto load_tiles = [&](int kt, int s, uint32_t ta, uint32_t tw) {
    uint8_t* sa = stage_ptr(s);
    uint8_t* sb = sa + A_BYTES;
    const uint32_t koff = (uint32_t)kt * (BK * 2);
    const uint32_t slab_a = (uint32_t)(8 * g.lda * 2), slab_w = (uint32_t)(8 * g.k * 2);
#pragma unroll
    for (int i = 0; i < NLA; ++i)
      buffer_load_lds16(A, bytes_a, sa + (wave_u + WAVES * i) * 1024, lane_a, ta + koff + (uint32_t)(wave_u + WAVES * i) * slab_a);
#pragma unroll
    for (int i = 0; i < NLB; ++i)
      buffer_load_lds16(W, bytes_w, sb + (wave_u + WAVES * i) * 1024, lane_w, tw + koff + (uint32_t)(wave_u + WAVES * i) * slab_w);
  };

  f32x16 acc[MI][NI];
  const int lr = lane & 31, lg = lane >> 5;
  bf16x8 af[2][MI], bfr[2][NI];
  auto frags = [&](int s, int kk, int b) {
    const uint8_t* sa = stage_ptr(s);
    const uint8_t* sb = sa + A_BYTES;
    const int ch = kk * 2 + lg;
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
      const int row = wm * TM + mi * 32 + lr;
      af[b][mi] = *reinterpret_cast<const bf16x8*>(sa + row * ROWB + ((ch ^ ((row >> 1) & 7)) << 4));
    }
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
      const int row = wn * TN + ni * 32 + lr;
      bfr[b][ni] = *reinterpret_cast<const bf16x8*>(sb + row * ROWB + ((ch ^ ((row >> 1) & 7)) << 4));
    }
  };
  auto mfmas = [&](int b) {
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[b][ni], af[b][mi], acc[mi][ni], 0, 0, 0);
  };

  {
    int tm, tn;
    tile_of(pq, tm, tn);
    set_tile(tm, tn);
  }
  int base = 0;                                  // stage of k-tile kt of the current tile = (kt + base) & 1
  load_tiles(0, 0, tile_a, tile_w);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (nk > 1) load_tiles(1, 1, tile_a, tile_w);
  frags(0, 0, 0);

  // MODE 2: after the barrier request k-tile kt+2 of this tile; 3: request k-tile 0 of the next tile (if there is one);
  // 0: last k-tile, nothing after it
  auto iteration = [&](int kt, auto mode_c, int np, bool has_next) {
    constexpr int MODE = decltype(mode_c)::value;
    const int cur = (kt + base) & 1;
#pragma unroll
    for (int kk = 0; kk + 1 < KK; ++kk) {
      frags(cur, kk + 1, (kk + 1) & 1);
      mfmas(kk & 1);
      {
        constexpr int NR = MI + NI, NM = MI * NI;
#pragma unroll
        for (int i = 0; i < NR; ++i) {
          if (i < NM) __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        if (NM > NR) __builtin_amdgcn_sched_group_barrier(0x008, NM - NR, 0);
      }
    }
    if (MODE >= 2) {
      asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
      __syncthreads();
      if (MODE == 2) load_tiles(kt + 2, cur, tile_a, tile_w);
      if (MODE == 3 && has_next) {
        int tm2, tn2;
        tile_of(np, tm2, tn2);
        const int64_t m2 = min((int64_t)tm2 * BM, g.m - BM);
        const int n2 = min(tn2 * BN, g.n - BN);
        load_tiles(0, cur, (uint32_t)(m2 * g.lda) * 2u, (uint32_t)n2 * (uint32_t)g.k * 2u);
      }
      frags(cur ^ 1, 0, KK & 1);
    }
    mfmas((KK - 1) & 1);
    if (MODE == 2) {
      constexpr int NR = MI + NI, NM = MI * NI, NV = NLA + NLB;
#pragma unroll
      for (int i = 0; i < NM; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        if (i < NV) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        if (i < NR) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
    }
  };

  for (;;) {
    const int np = pq + nslot;
    const bool has_next = np < pq_end;
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;
    {
      int kt = 0;
      for (; kt + 2 < nk; ++kt) iteration(kt, std::integral_constant<int, 2>{}, np, has_next);
      if (kt + 1 < nk) { iteration(kt, std::integral_constant<int, 3>{}, np, has_next); ++kt; }
      iteration(kt, std::integral_constant<int, 0>{}, np, has_next);
    }
    const int s_last = (nk - 1 + base) & 1;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();                               // every wave is done with the last stage; the next tile's first k-tile has landed
    {
      float* ep = reinterpret_cast<float*>(smem + (s_last ? STAGE : 0) + wave_u * EP_WAVE);
      const int64_t m_base = m0 + wm * TM;
      const int wcol0 = n0 + wn * TN;
      // The epilogue reads its arguments (a dozen pointers and sizes that the k-loop never touches) from the kernel
      // argument segment again, through a pointer the compiler cannot trace back: kept live across the k-loop they
      // overflow the scalar registers and come back from scratch memory one dependent load at a time.
      const __attribute__((address_space(4))) GemmArgs* ge =
          (const __attribute__((address_space(4))) GemmArgs*)__builtin_amdgcn_kernarg_segment_ptr();
      asm volatile("" : "+s"(ge) : : "memory");
      const GemmArgs& g2 = *(const GemmArgs*)ge;
      // likewise the lane number: the epilogue's per-lane offsets are the same for every tile, and the compiler
      // would compute them once before the first k-loop and carry them through it
      int lane_e = lane;
      asm volatile("" : "+v"(lane_e));
      const TileBounds tb{row_lo, g2.m, col_lo, g2.n, 0};
      if (m0 == row_lo && n0 == col_lo) wave_epilogue<EPI, MI, NI, true>(acc, g2, ep, m_base, wcol0, lane_e, tb);
      else wave_epilogue<EPI, MI, NI, false>(acc, g2, ep, m_base, wcol0, lane_e, tb);
    }
    if (!has_next) break;
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __syncthreads();                               // the staging area is free again
    pq = np;
    {
      int tm, tn;
      tile_of(pq, tm, tn);
      set_tile(tm, tn);
    }
    base = (base + nk) & 1;
    if (nk > 1) load_tiles(1, (1 + base) & 1, tile_a, tile_w);
    frags(base & 1, 0, 0);
  }
}

template <int BM, int BN, int WM, int WN>
static hipError_t launch_persist(const GemmArgs& a, hipStream_t s) {
  const int tiles_n = (a.n + BN - 1) / BN;
  const int64_t tiles_m = (a.m + BM - 1) / BM;
  const int64_t total = tiles_m * tiles_n;
  if (total <= 0) return hipSuccess;
  if (total > (1 << 30)) return hipErrorInvalidValue;
  constexpr int STAGE = (BM + BN) * 128, EP_BYTES = WM * WN * kEpWaveBytes;
  constexpr int EXTRA = EP_BYTES > STAGE ? (EP_BYTES - STAGE + 255) / 256 * 256 : 0;
  const size_t lds = 2 * STAGE + EXTRA;
  const unsigned grid = (unsigned)std::min<int64_t>(256, (total + 7) / 8 * 8);
  dim3 block(WM * WN * 64);
#define TCMV_PGEMM_CASE(E)                                                                             \
  case E: {                                                                                            \
    auto kern = gemm_bf16_persist_kernel<BM, BN, WM, WN, E>;                                           \
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                            \
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);          \
    if (e != hipSuccess) return e;                                                                     \
    hipLaunchKernelGGL(kern, dim3(grid), block, lds, s, a);                                            \
    break;                                                                                             \
  }
  switch (a.epi) {
    TCMV_PGEMM_CASE(EPI_STORE) TCMV_PGEMM_CASE(EPI_GELU) TCMV_PGEMM_CASE(EPI_RESID) TCMV_PGEMM_CASE(EPI_RESID_AHEAD)
    TCMV_PGEMM_CASE(EPI_EMBED) TCMV_PGEMM_CASE(EPI_QKV) TCMV_PGEMM_CASE(EPI_GATED)
    default: return hipErrorInvalidValue;
  }
#undef TCMV_PGEMM_CASE
  return hipGetLastError();
}


namespace {
enum GemmKernel { GK_INVALID, GK_P320, GK_P256, GK_SPLITK, GK_T64, GK_T128 };
// which kernel a product runs on, and the width of its wave tiles
GemmKernel choose_kernel(const GemmArgs& a, int* wave_tile_n, int* block_n) {
  if (a.k <= 0 || a.k % 64 || a.lda % 8 || a.n <= 0 || a.n % 8 || a.ldc % 4) return GK_INVALID;
  if (a.epi == EPI_QKV && (a.split % 8)) return GK_INVALID;
  if (a.epi == EPI_QKV && a.rope && (a.rope_dh % 8 || a.rope_dh <= 0)) return GK_INVALID;
  if (a.epi == EPI_GATED && (a.ldc % 4)) return GK_INVALID;
  // operand element offsets are kept in 32 bits
  if ((double)a.m * (double)a.lda >= 4294967296.0 || (double)a.n * (double)a.k >= 4294967296.0) return GK_INVALID;
  // Persistent 256-row tiles (8 waves, one workgroup per CU) from about one and a half rounds of them over the 256
  // CUs.  A tile 320 columns wide is taken where it needs no more tile area x rounds than a 256-wide one (hidden
  // sizes that are multiples of 320 but not of 256, such as 1280).  That kernel addresses its operands in bytes,
  // 32 bits.
  const int64_t big_tiles = ((a.m + 255) / 256) * ((a.n + 255) / 256);
  if (big_tiles >= 400 && a.k >= 128 && a.m >= 256 && a.n >= 320 && a.epi != EPI_PARTIAL &&
      (double)a.m * (double)a.lda < 2147483648.0 && (double)a.n * (double)a.k < 2147483648.0) {
    auto area = [&](int64_t bm, int64_t bn) {
      const int64_t t = ((a.m + bm - 1) / bm) * ((a.n + bn - 1) / bn);
      return ((t + 255) / 256) * bm * bn;
    };
    if (area(256, 320) <= area(256, 256)) { *wave_tile_n = 160; *block_n = 320; return GK_P320; }
    *wave_tile_n = 64; *block_n = 256;
    return GK_P256;
  }
  // a single small request: fewer than 200 tiles of 128x128 leave most CUs idle; 64x64 tiles
  // (2 waves) quadruple the number of workgroups
  const int64_t mid_tiles = ((a.m + 127) / 128) * ((a.n + 127) / 128);
  *wave_tile_n = 64; *block_n = 128;
  // a long contraction over few rows (fc2 of one small request): 64x64 tiles would each walk all of k and
  // re-read both operands from L2 twice as often; 128x128 tiles over a quarter of k each give as many
  // workgroups with a quarter of the iterations.  The slices are added to C in a fixed order afterwards.
  if (mid_tiles < 200 && a.epi == EPI_RESID && a.partial && a.k >= 2048 && (a.k / 64) % 4 == 0) return GK_SPLITK;
  if (mid_tiles < 200) { *wave_tile_n = 32; *block_n = 64; return GK_T64; }
  return GK_T128;
}
}  // namespace

bool gemm_bf16_can_fuse_key_norms(int64_t m, int n, int k, int qcols, int dh) {
  if (dh != 64 && dh != 80) return false;
  GemmArgs a{};
  a.m = m; a.n = n; a.k = k; a.lda = k; a.ldc = 2 * qcols; a.epi = EPI_QKV; a.split = 2 * qcols; a.qcols = qcols;
  int tn = 0, bn = 0;
  const GemmKernel gk = choose_kernel(a, &tn, &bn);
  if (gk == GK_INVALID || gk == GK_SPLITK) return false;
  // whole heads per wave tile, wave tiles that start at head boundaries, no shifted last tile
  return tn % dh == 0 && tn / dh <= 4 && qcols % tn == 0 && ((gk != GK_P320 && gk != GK_P256) || n % bn == 0);
}

hipError_t launch_gemm_bf16(const GemmArgs& a, hipStream_t s) {
  if (a.m == 0 || a.n == 0) return hipSuccess;
  int tn = 0, bn = 0;
  const GemmKernel gk = choose_kernel(a, &tn, &bn);
  if (a.epi == EPI_QKV && a.kmax2 &&
      !(gk != GK_INVALID && (a.kn_dh == 64 || a.kn_dh == 80) && tn % a.kn_dh == 0 && a.qcols % tn == 0 &&
        a.split == 2 * a.qcols && a.row_seg && ((gk != GK_P320 && gk != GK_P256) || a.n % bn == 0)))
    return hipErrorInvalidValue;
  if ((gk == GK_P320 || gk == GK_P256) && a.epi == EPI_RESID && (double)a.m * (double)a.n * 4.0 > 400e6) {
    GemmArgs g = a;                                 // an output larger than the last-level cache: see wave_epilogue
    g.epi = EPI_RESID_AHEAD;
    return gk == GK_P320 ? launch_persist<256, 320, 4, 2>(g, s) : launch_persist<256, 256, 2, 4>(g, s);
  }
  switch (gk) {
    case GK_P320: return launch_persist<256, 320, 4, 2>(a, s);
    case GK_P256: return launch_persist<256, 256, 2, 4>(a, s);
    case GK_SPLITK: {
      GemmArgs g = a;
      g.epi = EPI_PARTIAL; g.ksplit = 4;
      const hipError_t e = launch_cfg<128, 128, 2, 2, 64, 2, 2>(g, s);
      if (e != hipSuccess) return e;
      const int64_t n4 = (int64_t)a.m * (a.n / 4);
      hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, s,
                         reinterpret_cast<float*>(a.c), a.ldc, a.partial, a.bias, a.m, a.n, 4);
      return hipGetLastError();
    }
    case GK_T64: return launch_cfg<64, 64, 1, 2, 64, 2, 4>(a, s);
    case GK_T128: return launch_cfg<128, 128, 2, 2, 64, 2, 2>(a, s);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace tcmv
