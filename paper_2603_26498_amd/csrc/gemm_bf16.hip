// C = epilogue(A * W^T + bias) on bf16 MFMA (gfx950), fp32 accumulation.
//
// A [m, k] and W [n, k] are both contiguous along k, so both operands are staged
// the same way: direct global -> LDS loads (16 bytes per lane, no registers in
// between) into tiles of 64 k-elements per row (128 bytes), with the 16-byte
// chunk index XOR-swizzled by (row/2)%8 so that the per-lane 16-byte MFMA operand
// reads are conflict-free: the LDS serves 16 lanes x 16 bytes per clock over 64
// banks, two 128-byte rows span the banks, so 16 consecutive rows reading the
// same logical chunk must land on 16 different 16-byte bank groups.  LDS is double buffered and
// the next tile's loads are issued before the current tile's MFMAs.  Each wave owns a (BM/WM) x (BN/WN) sub-tile
// built from v_mfma_f32_32x32x16_bf16.
//
// The MFMA is issued with W as the row operand and A as the column operand, so
// the accumulator holds C^T: a lane owns ONE output row (token) and, per 32x32
// tile, four groups of four consecutive output columns.  Written out like that a
// store instruction would touch 32 rows; each wave therefore passes its sub-tile
// through a private LDS buffer (32 rows at a time, in column groups of at most 256)
// and comes back with lanes running along the row: bias / position adds, GELU,
// the gated product, the rotary rotation, the fp32 residual read-modify-write and
// the bf16 stores all work on 16 contiguous bytes per lane.  Only the transposed-V
// columns of the QKV projection leave from registers (consecutive lanes =
// consecutive tokens = the contiguous direction of that buffer).
//
// Tiles: 256x256 or 256x320 (8 waves, one workgroup per CU) for large products,
// 128x128 (4 waves, two per CU), 64x64 (2 waves) for a single small request; a long
// contraction over few rows that accumulates into the residual stream is cut into
// four slices of k whose fp32 partial sums a second kernel adds in slice order.
//
// Workgroups are numbered so that the eight XCDs (workgroup id mod 8) each walk
// a contiguous range of tiles: neighbouring tiles share A rows or W rows in the
// XCD's own L2.
#include <type_traits>
#include "tcmv_internal.h"
#include "device_utils.h"

namespace tcmv {

namespace {
typedef __attribute__((address_space(1))) const void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;
}  // namespace

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

  // ---- epilogue.  In the accumulator a lane holds row (lane & 31) and columns
  // 8*(v/4) + 4*(lane>>5) + v%4 of each 32x32 tile: writing that to a row-major matrix
  // directly would touch 32 cache lines per store instruction.  Each wave therefore
  // passes its sub-tile through a private LDS buffer, 32 rows at a time, and comes
  // back with lanes running along the row (16 bytes per lane): stores and the fp32
  // residual read-modify-write are full contiguous segments.  Only the transposed-V
  // part of the QKV projection keeps the register layout (there consecutive lanes =
  // consecutive tokens is exactly the contiguous direction).
  // A wave tile whose width divides 256 columns goes through the buffer in one piece; any
  // other width (160 columns of the 256x320 tile) in groups of two 32-column tiles, the odd
  // one last.
  constexpr int GN = (256 % TN == 0) ? NI : 2;     // 32-column tiles per group
  constexpr int EPS = GN * 32 + 4;                 // padded row stride of the staging buffer (floats)
  static_assert(WAVES * 32 * EPS * 4 <= NSTAGE * STAGE, "epilogue staging does not fit in the operand stages");
  static_assert(TN % 32 == 0, "wave tile width");
  __syncthreads();                                 // every wave is done with the operand stages
  float* ep = reinterpret_cast<float*>(smem) + wave * (32 * EPS);
  const int wcol0 = n0 + wn * TN;

  // one group of NGT tiles (columns nb*32 .. nb*32 + NGT*32 of the wave tile) of 32 rows: registers -> LDS -> global
  auto flush = [&](auto ngc, int mi, int nb, int64_t rbase) {
    constexpr int NGT = decltype(ngc)::value;
    constexpr int LPR = NGT * 8;                   // lanes per row when reading back
    constexpr int RPP = 64 / LPR;                  // rows per read pass
    // registers -> LDS (lane = row)
#pragma unroll
    for (int ni = 0; ni < NGT; ++ni)
#pragma unroll
      for (int vq = 0; vq < 4; ++vq)
        *reinterpret_cast<float4*>(ep + lr * EPS + ni * 32 + 8 * vq + 4 * lg) =
            make_float4(acc[mi][nb + ni][4 * vq], acc[mi][nb + ni][4 * vq + 1], acc[mi][nb + ni][4 * vq + 2],
                        acc[mi][nb + ni][4 * vq + 3]);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // same-wave LDS ops complete in order; keep the compiler from reordering
    // LDS -> global (lanes along the row)
    const int c4 = (lane % LPR) * 4;
    const int col = wcol0 + nb * 32 + c4;
    float4 b4 = make_float4(0.f, 0.f, 0.f, 0.f);
    if (EPI != EPI_PARTIAL && g.bias && col < g.n) b4 = *reinterpret_cast<const float4*>(g.bias + col);
#pragma unroll
    for (int ps = 0; ps < 32 / RPP; ++ps) {
      const int r = ps * RPP + lane / LPR;
      const int64_t row = rbase + r;
      float4 val = *reinterpret_cast<const float4*>(ep + r * EPS + c4);
      if (row >= g.m || col >= g.n) continue;
      val.x += b4.x; val.y += b4.y; val.z += b4.z; val.w += b4.w;
      if (EPI == EPI_GATED) {
        // columns (col, col+1) and (col+2, col+3) are (gate, up) pairs of output columns col/2 and col/2 + 1
        const float h0 = val.x / (1.0f + __expf(-val.x)) * val.y;
        const float h1 = val.z / (1.0f + __expf(-val.z)) * val.w;
        *reinterpret_cast<uint32_t*>(reinterpret_cast<uint16_t*>(g.c) + (size_t)row * g.ldc + (col >> 1)) = pack_bf16x2(h0, h1);
      } else if (EPI == EPI_STORE || EPI == EPI_GELU || EPI == EPI_QKV) {
        if (EPI == EPI_QKV && col >= g.split) continue;
        if (EPI == EPI_QKV && col < g.qcols) { val.x *= g.qscale; val.y *= g.qscale; val.z *= g.qscale; val.w *= g.qscale; }
        if (EPI == EPI_QKV && g.rope) {
          // rotary positions: the lane holds element pairs p and p+1 of one head (col % 4 == 0, head size % 4 == 0)
          const int p2 = ((col % g.rope_dh) >> 1) * 2;
          const float4 cs = *reinterpret_cast<const float4*>(g.rope + (size_t)row * g.rope_dh + p2);   // cos, sin, cos, sin
          const float x0 = val.x, x1 = val.y, x2 = val.z, x3 = val.w;
          val.x = x0 * cs.x - x1 * cs.y; val.y = x0 * cs.y + x1 * cs.x;
          val.z = x2 * cs.z - x3 * cs.w; val.w = x2 * cs.w + x3 * cs.z;
        }
        if (EPI == EPI_GELU) {
          val.x = gelu_fast(val.x); val.y = gelu_fast(val.y); val.z = gelu_fast(val.z); val.w = gelu_fast(val.w);
        }
        uint2 pk;
        pk.x = pack_bf16x2(val.x, val.y);
        pk.y = pack_bf16x2(val.z, val.w);
        *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(g.c) + (size_t)row * g.ldc + col) = pk;
      } else if (EPI == EPI_PARTIAL) {
        *reinterpret_cast<float4*>(g.partial + ((size_t)slice * g.m + row) * g.n + col) = val;
      } else if (EPI == EPI_RESID) {
        float4* c = reinterpret_cast<float4*>(reinterpret_cast<float*>(g.c) + (size_t)row * g.ldc + col);
        float4 old = *c;
        old.x += val.x; old.y += val.y; old.z += val.z; old.w += val.w;
        *c = old;
      } else if (EPI == EPI_EMBED) {
        const int pi = g.pos_idx ? g.pos_idx[row] : 0;
        if (g.pos_kind == 1) {
          const float4 p0 = *reinterpret_cast<const float4*>(g.pos0 + (size_t)pi * g.n + col);
          val.x += p0.x; val.y += p0.y; val.z += p0.z; val.w += p0.w;
        } else if (g.pos_kind == 2) {
          const float4 p0 = *reinterpret_cast<const float4*>(g.pos0 + (size_t)(pi & 0xFFFF) * g.n + col);
          const float4 p1 = *reinterpret_cast<const float4*>(g.pos1 + (size_t)(pi >> 16) * g.n + col);
          val.x += p0.x + p1.x; val.y += p0.y + p1.y; val.z += p0.z + p1.z; val.w += p0.w + p1.w;
        }
        const int64_t dst = g.dst_row ? (int64_t)g.dst_row[row] : row;
        *reinterpret_cast<float4*>(reinterpret_cast<float*>(g.c) + (size_t)dst * g.ldc + col) = val;
      }
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // reads done before the next group overwrites the buffer
  };

#pragma unroll
  for (int mi = 0; mi < MI; ++mi) {
    const int64_t rbase = m0 + wm * TM + mi * 32;
    if (EPI == EPI_QKV && wcol0 + TN > g.split) {
      // transposed-V columns straight from registers
      const int64_t row = rbase + lr;
      if (row < g.m) {
        const int vc = g.vcol[row];
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
          for (int vq = 0; vq < 4; ++vq) {
            const int col = wcol0 + ni * 32 + 8 * vq + 4 * lg;
            if (col >= g.split && col < g.n) {
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
      if (wcol0 >= g.split) continue;              // nothing else in this wave tile
    }
#pragma unroll
    for (int nb = 0; nb < NI; nb += GN) {
      if (nb + GN <= NI) flush(std::integral_constant<int, GN>{}, mi, nb, rbase);
      else flush(std::integral_constant<int, 1>{}, mi, nb, rbase);
    }
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

hipError_t launch_gemm_bf16(const GemmArgs& a, hipStream_t s) {
  if (a.m == 0 || a.n == 0) return hipSuccess;
  if (a.k <= 0 || a.k % 64 || a.lda % 8 || a.n <= 0 || a.n % 8 || a.ldc % 4) return hipErrorInvalidValue;
  if (a.epi == EPI_QKV && (a.split % 4)) return hipErrorInvalidValue;
  if (a.epi == EPI_QKV && a.rope && (a.rope_dh % 4 || a.rope_dh <= 0)) return hipErrorInvalidValue;
  if (a.epi == EPI_GATED && (a.ldc % 2)) return hipErrorInvalidValue;
  // operand element offsets are kept in 32 bits
  if ((double)a.m * (double)a.lda >= 4294967296.0 || (double)a.n * (double)a.k >= 4294967296.0) return hipErrorInvalidValue;
  // 256x256 tiles (8 waves, one workgroup per CU) when there are at least two full rounds of
  // them and the output is wide or the contraction long, or at least four rounds whatever the
  // shape; 128x128 tiles (4 waves, two workgroups per CU) otherwise.  (Measured on the
  // encoder's shapes.)
  const int64_t big_tiles = ((a.m + 255) / 256) * ((a.n + 255) / 256);
  if (big_tiles >= 512 && (a.n >= 2560 || a.k >= 2560 || big_tiles >= 1024)) {
    // one workgroup per CU and 256 CUs: the launch takes ceil(tiles / 256) rounds of one tile
    // time each.  A tile 320 columns wide is taken where it saves rounds' worth of tile area
    // (hidden sizes that are multiples of 320 but not of 256, such as 1280).
    auto area = [&](int64_t bm, int64_t bn) {
      const int64_t t = ((a.m + bm - 1) / bm) * ((a.n + bn - 1) / bn);
      return ((t + 255) / 256) * bm * bn;
    };
    if (area(256, 320) * 100 < area(256, 256) * 97) return launch_cfg<256, 320, 4, 2, 64, 2, 1>(a, s);
    return launch_cfg<256, 256, 2, 4, 64, 2, 1>(a, s);
  }
  // a single small request: fewer than 200 tiles of 128x128 leave most CUs idle; 64x64 tiles
  // (2 waves) quadruple the number of workgroups
  const int64_t mid_tiles = ((a.m + 127) / 128) * ((a.n + 127) / 128);
  if (mid_tiles < 200 && a.epi == EPI_RESID && a.partial && a.k >= 2048 && (a.k / 64) % 4 == 0 && a.n % 4 == 0) {
    // a long contraction over few rows (fc2 of one small request): 64x64 tiles would each walk all of k and
    // re-read both operands from L2 twice as often; 128x128 tiles over a quarter of k each give as many
    // workgroups with a quarter of the iterations.  The slices are added to C in a fixed order afterwards.
    GemmArgs g = a;
    g.epi = EPI_PARTIAL; g.ksplit = 4;
    const hipError_t e = launch_cfg<128, 128, 2, 2, 64, 2, 2>(g, s);
    if (e != hipSuccess) return e;
    const int64_t n4 = (int64_t)a.m * (a.n / 4);
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, s,
                       reinterpret_cast<float*>(a.c), a.ldc, a.partial, a.bias, a.m, a.n, 4);
    return hipGetLastError();
  }
  if (mid_tiles < 200) return launch_cfg<64, 64, 1, 2, 64, 2, 4>(a, s);
  return launch_cfg<128, 128, 2, 2, 64, 2, 2>(a, s);
}

}  // namespace tcmv
