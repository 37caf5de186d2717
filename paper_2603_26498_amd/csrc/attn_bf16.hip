// Bidirectional block-diagonal attention on bf16 MFMA (gfx950), flash style:
// scores are never written to memory; softmax statistics are kept per query in
// fp32 and updated tile by tile (online softmax).
//
// Work decomposition: one workgroup (4 waves) = 128 query rows of one segment
// and one head; each wave owns 32 query rows.  K and V^T tiles of 64 keys are
// staged in LDS (double buffered, next tile's global loads in flight during the
// MFMAs) and shared by the four waves.
//
// The kernel computes S^T = K * Q^T (keys are the MFMA row dimension).  In the
// 32x32 accumulator layout a lane then holds ONE query column and 16 keys, so
//   * the running max / rescale factor are one scalar per lane,
//   * the exponentiated scores, packed to bf16 in place, already have the
//     register layout of the B operand of O^T += V^T * P^T (the contraction
//     index only has to be enumerated in the same order on both operands, so V^T
//     is read from LDS in the key order the accumulator happens to have),
//   * P never goes through LDS.
// V arrives already transposed ([head_dim, keys], keys contiguous) so the V^T
// operand is two 8-byte LDS reads per MFMA.
//
// When head_dim is an odd multiple of 16 the V^T tile is padded to a multiple of
// 32 rows; the first padding row is filled with ones, which makes the MFMA
// produce the softmax denominator (sum of the bf16-rounded probabilities) for
// free; otherwise the denominator is accumulated on the vector ALU.
#include "tcmv_internal.h"
#include "device_utils.h"

namespace tcmv {

namespace {
constexpr int BQ = kAttnBQ_bf16;
constexpr int BKV = 64;
constexpr int NTHREADS = 256;
}  // namespace

template <int DH>
struct AttnCfg {
  static constexpr int KS = DH / 16;                       // MFMA k-steps of the score product
  static constexpr int DHP = (DH + 31) / 32 * 32;          // V^T rows incl. padding
  static constexpr int MT = DHP / 32;                      // 32-row tiles of O^T
  static constexpr bool ONES = (DH % 32) == 16;            // denominator from the MFMA
  static constexpr int KCH = DH / 8;                       // 16-byte chunks per K row
  static constexpr int KSTR = (KCH | 1) * 16;              // K row stride in LDS (odd number of chunks)
  static constexpr int K_BYTES = BKV * KSTR;
  static constexpr int V_BYTES = DHP * BKV * 2;
  static constexpr int STAGE = K_BYTES + V_BYTES;
  static constexpr int NCH_K = BKV * KCH, NCH_V = DH * (BKV / 8);
  static constexpr int NLOAD = (NCH_K + NCH_V) / NTHREADS;   // 16-byte global loads per thread per tile
  static_assert((NCH_K + NCH_V) % NTHREADS == 0, "tile does not split evenly over the workgroup");
};

// V^T tile in LDS: row = head-dim index (128 bytes = 64 keys).  Inside a row the
// keys are stored in the order the PV MFMA wants them: 16-byte chunk (2G + g)
// holds keys {16G + 4g + 0..3, 16G + 8 + 4g + 0..3}, i.e. exactly the 8 keys a
// lane of half-wave g contributes to k-step G.  Chunks are XOR-swizzled by the
// row so that 32 lanes reading the same chunk of 32 different rows hit all banks.
template <int DH>
__global__ __launch_bounds__(NTHREADS, 2) void attn_bf16_kernel(AttnArgs a) {
  using C = AttnCfg<DH>;
  __shared__ __attribute__((aligned(16))) uint8_t smem[2 * C::STAGE];

  const int total = a.n_work * a.heads;
  const int chunk = (total + 7) >> 3;
  const int p = (int)(blockIdx.x & 7) * chunk + (int)(blockIdx.x >> 3);
  if (p >= total) return;
  const int head = p / a.n_work;
  const AttnWork w = a.work[p - head * a.n_work];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  __builtin_assume(tid >= 0 && tid < NTHREADS);
  const int lr = lane & 31, lg = lane >> 5;
  const uint16_t* Q = reinterpret_cast<const uint16_t*>(a.q);
  const uint16_t* K = reinterpret_cast<const uint16_t*>(a.k);
  const uint16_t* VT = reinterpret_cast<const uint16_t*>(a.v);

  // padding rows of the V^T tiles: ones row (denominator) then zeros
  if (C::DHP > DH) {
    for (int i = tid; i < 2 * (C::DHP - DH) * (BKV / 2); i += NTHREADS) {
      const int buf = i / ((C::DHP - DH) * (BKV / 2));
      const int rem = i - buf * ((C::DHP - DH) * (BKV / 2));
      const int row = DH + rem / (BKV / 2), c2 = rem % (BKV / 2);
      const uint32_t val = (C::ONES && row == DH) ? 0x3F803F80u : 0u;
      *reinterpret_cast<uint32_t*>(smem + buf * C::STAGE + C::K_BYTES + row * (BKV * 2) + c2 * 4) = val;
    }
  }

  // query fragments (B operand of S^T = K Q^T), kept in registers for the whole kernel
  bf16x8 qf[C::KS];
  {
    int qi = wave * 32 + lr;
    if (qi >= w.nq) qi = w.nq - 1;
    const uint16_t* qp = Q + (size_t)(w.q0 + qi) * a.ldqk + head * DH + lg * 8;
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks) qf[ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 16);
  }

  // global -> register staging of one K / V^T tile: NLOAD 16-byte chunks per thread;
  // chunk ids [0, NCH_K) are K, the rest V^T.  Source pointers and LDS offsets are
  // selected arithmetically (no divergent control flow) and computed once.
  uint4 rg[C::NLOAD];
  const uint16_t* gsrc[C::NLOAD];   // source of tile 0; K advances by 64 rows, V^T by 64 columns per tile
  int lds_lo[C::NLOAD], lds_hi[C::NLOAD];   // byte offsets of the two 8-byte halves inside a stage
  int vkey0[C::NLOAD];              // V^T chunks: first key of the chunk inside the tile, K chunks: -1
  int krow[C::NLOAD];               // K chunks: row inside the tile
#pragma unroll
  for (int i = 0; i < C::NLOAD; ++i) {
    const int c = tid + i * NTHREADS;
    const bool is_k = c < C::NCH_K;
    const int rowk = c / C::KCH, cck = c - rowk * C::KCH;
    const int cv = c - C::NCH_K;
    const int rowv = cv >> 3, ccv = cv & 7;
    const int G = ccv >> 1, h = ccv & 1, sw = rowv & 7;
    const int vb = C::K_BYTES + rowv * (BKV * 2) + h * 8;
    lds_lo[i] = is_k ? rowk * C::KSTR + cck * 16 : vb + (((2 * G) ^ sw) << 4);
    lds_hi[i] = is_k ? rowk * C::KSTR + cck * 16 + 8 : vb + (((2 * G + 1) ^ sw) << 4);
    vkey0[i] = is_k ? -1 : ccv * 8;
    krow[i] = is_k ? rowk : 0;
    const uint16_t* ks = K + (size_t)head * DH + (size_t)(w.seg_start + rowk) * a.ldqk + cck * 8;
    const uint16_t* vs = VT + ((size_t)head * DH + rowv) * a.ldv + w.v0 + ccv * 8;
    gsrc[i] = is_k ? ks : vs;
  }
  const int64_t kstep = (int64_t)BKV * a.ldqk;
  auto load_tile = [&](int t, bool tail) {
#pragma unroll
    for (int i = 0; i < C::NLOAD; ++i) {
      const bool is_k = vkey0[i] < 0;
      const uint16_t* src = gsrc[i] + (is_k ? (int64_t)t * kstep : (int64_t)t * BKV);
      if (tail && is_k) {   // last tile: rows past the end of the buffer are clamped (their scores are masked)
        const int64_t over = (int64_t)w.seg_start + t * BKV + krow[i] - (a.t_total - 1);
        if (over > 0) src -= over * a.ldqk;
      }
      uint4 v = *reinterpret_cast<const uint4*>(src);
      if (tail && !is_k) {  // keys beyond the segment: force exact zeros (the buffer may hold anything there)
        const int valid = w.seg_len - (t * BKV + vkey0[i]);
        v.x = (valid <= 0) ? 0u : (valid == 1 ? (v.x & 0xFFFFu) : v.x);
        v.y = (valid <= 2) ? 0u : (valid == 3 ? (v.y & 0xFFFFu) : v.y);
        v.z = (valid <= 4) ? 0u : (valid == 5 ? (v.z & 0xFFFFu) : v.z);
        v.w = (valid <= 6) ? 0u : (valid == 7 ? (v.w & 0xFFFFu) : v.w);
      }
      rg[i] = v;
    }
  };
  auto store_tile = [&](int buf) {
    uint8_t* st = smem + buf * C::STAGE;
#pragma unroll
    for (int i = 0; i < C::NLOAD; ++i) {
      *reinterpret_cast<uint2*>(st + lds_lo[i]) = make_uint2(rg[i].x, rg[i].y);
      *reinterpret_cast<uint2*>(st + lds_hi[i]) = make_uint2(rg[i].z, rg[i].w);
    }
  };

  f32x16 o[C::MT];
#pragma unroll
  for (int mt = 0; mt < C::MT; ++mt)
#pragma unroll
    for (int v = 0; v < 16; ++v) o[mt][v] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const float cs = a.scale;   // softmax scale * log2(e)

  const int n_tiles = (w.seg_len + BKV - 1) / BKV;
  const bool ragged = (w.seg_len % BKV) != 0;
  load_tile(0, ragged && n_tiles == 1);
  store_tile(0);
  __syncthreads();

  for (int t = 0; t < n_tiles; ++t) {
    const int j0 = t * BKV;
    if (t + 1 < n_tiles) load_tile(t + 1, ragged && (t + 2 == n_tiles));
    const uint8_t* sk = smem + (t & 1) * C::STAGE;
    const uint8_t* sv = sk + C::K_BYTES;

    // ---- S^T tile: 64 keys x 32 queries.  All K fragments are requested first so
    // that the LDS latency overlaps; the two key blocks alternate on the MFMA pipe.
    bf16x8 kf[2][C::KS];
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks)
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
        kf[kb][ks] = *reinterpret_cast<const bf16x8*>(sk + (kb * 32 + lr) * C::KSTR + (2 * ks + lg) * 16);
    f32x16 s[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int v = 0; v < 16; ++v) s[kb][v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks)
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
        s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kb][ks], qf[ks], s[kb], 0, 0, 0);

    // V^T fragments of the first two k-steps are requested before the softmax arithmetic
    bf16x8 vf[C::MT][4];
    auto load_vf = [&](int G) {
#pragma unroll
      for (int mt = 0; mt < C::MT; ++mt) {
        const int row = mt * 32 + lr;
        vf[mt][G] = *reinterpret_cast<const bf16x8*>(sv + row * (BKV * 2) + (((2 * G + lg) ^ (row & 7)) << 4));
      }
    };
    load_vf(0);
    load_vf(1);

    if (ragged && t + 1 == n_tiles) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int key = j0 + kb * 32 + 8 * (v >> 2) + 4 * lg + (v & 3);
          if (key >= w.seg_len) s[kb][v] = -INFINITY;
        }
    }
    // ---- online softmax (per lane = per query column)
    float mx = s[0][0];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s[kb][v]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx);
    const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * cs);
    m_run = m_new;
    const float mc = m_new * cs;
    bf16x8 pf[4];     // pf[G]: keys of k-step G = 2*kb + j
    float psum = 0.f;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        uint32_t pk[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float p0 = __builtin_amdgcn_exp2f(fmaf(s[kb][8 * j + 2 * e], cs, -mc));
          const float p1 = __builtin_amdgcn_exp2f(fmaf(s[kb][8 * j + 2 * e + 1], cs, -mc));
          if (!C::ONES) psum += p0 + p1;
          pk[e] = pack_bf16x2(p0, p1);
        }
        uint4 u = make_uint4(pk[0], pk[1], pk[2], pk[3]);
        pf[2 * kb + j] = __builtin_bit_cast(bf16x8, u);
      }
    if (!C::ONES) l_run = l_run * alpha + psum;
    if (__any(alpha != 1.0f)) {
#pragma unroll
      for (int mt = 0; mt < C::MT; ++mt)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[mt][v] *= alpha;
    }
    // ---- O^T += V^T P^T  (independent accumulators alternate on the MFMA pipe)
    load_vf(2);
    load_vf(3);
#pragma unroll
    for (int G = 0; G < 4; ++G)
#pragma unroll
      for (int mt = 0; mt < C::MT; ++mt)
        o[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[mt][G], pf[G], o[mt], 0, 0, 0);

    if (t + 1 < n_tiles) store_tile((t + 1) & 1);
    __syncthreads();
  }

  // ---- normalise and store: lane holds query (lane & 31), head-dim rows 8*(v/4) + 4*lg + v%4
  float l;
  if (C::ONES) {
    constexpr int r = DH % 32;                       // row of the ones line inside its tile (16)
    l = __shfl(o[DH / 32][4 * (r / 8)], lr, 64);     // held by the lanes of the lower half-wave
  } else {
    l = l_run + __shfl_xor(l_run, 32, 64);
  }
  const float inv = 1.0f / l;
  const int qi = wave * 32 + lr;
  if (qi < w.nq) {
    uint16_t* op = reinterpret_cast<uint16_t*>(a.out) + (size_t)(w.q0 + qi) * a.ldo + head * DH;
#pragma unroll
    for (int mt = 0; mt < C::MT; ++mt)
#pragma unroll
      for (int vq = 0; vq < 4; ++vq) {
        const int dh0 = mt * 32 + 8 * vq + 4 * lg;
        if (dh0 < DH) {
          uint2 pk;
          pk.x = pack_bf16x2(o[mt][4 * vq] * inv, o[mt][4 * vq + 1] * inv);
          pk.y = pack_bf16x2(o[mt][4 * vq + 2] * inv, o[mt][4 * vq + 3] * inv);
          *reinterpret_cast<uint2*>(op + dh0) = pk;
        }
      }
  }
}

hipError_t launch_attn_bf16(const AttnArgs& a, hipStream_t s) {
  if (a.n_work == 0 || a.heads == 0) return hipSuccess;
  const int64_t total = (int64_t)a.n_work * a.heads;
  if (total > (1 << 30)) return hipErrorInvalidValue;
  if (a.ldqk % 8 || a.ldv % 8 || a.ldo % 4) return hipErrorInvalidValue;
  const unsigned grid = (unsigned)(((total + 7) / 8) * 8);
#define TCMV_ATTN_CASE(D)                                                                      \
  case D:                                                                                      \
    hipLaunchKernelGGL((attn_bf16_kernel<D>), dim3(grid), dim3(NTHREADS), 0, s, a);            \
    break;
  switch (a.dh) {
    TCMV_ATTN_CASE(32) TCMV_ATTN_CASE(64) TCMV_ATTN_CASE(80) TCMV_ATTN_CASE(96)
    default: return hipErrorInvalidValue;
  }
#undef TCMV_ATTN_CASE
  return hipGetLastError();
}

// vt[c][vcol[r]] = v[r][c]: staging through LDS so that both sides are coalesced.
__global__ __launch_bounds__(256) void transpose_v_kernel(const uint16_t* v, int64_t ldv, const int32_t* vcol,
                                                          uint16_t* vt, int64_t ldvt, int64_t rows, int d) {
  __shared__ uint16_t tile[64][65];
  const int64_t r0 = (int64_t)blockIdx.x * 64;
  const int c0 = blockIdx.y * 64;
  for (int i = threadIdx.x; i < 64 * 64; i += 256) {
    const int r = i >> 6, c = i & 63;
    tile[r][c] = (r0 + r < rows && c0 + c < d) ? v[(size_t)(r0 + r) * ldv + c0 + c] : (uint16_t)0;
  }
  __syncthreads();
  for (int i = threadIdx.x; i < 64 * 64; i += 256) {
    const int c = i >> 6, r = i & 63;
    if (r0 + r < rows && c0 + c < d) vt[(size_t)(c0 + c) * ldvt + vcol[r0 + r]] = tile[r][c];
  }
}

hipError_t launch_transpose_v(const void* v, int64_t ldv, const int32_t* vcol, void* vt, int64_t ldvt, int64_t rows,
                              int d, hipStream_t s) {
  if (rows == 0) return hipSuccess;
  dim3 grid((unsigned)((rows + 63) / 64), (unsigned)((d + 63) / 64));
  hipLaunchKernelGGL(transpose_v_kernel, grid, dim3(256), 0, s, reinterpret_cast<const uint16_t*>(v), ldv, vcol,
                     reinterpret_cast<uint16_t*>(vt), ldvt, rows, d);
  return hipGetLastError();
}

}  // namespace tcmv
