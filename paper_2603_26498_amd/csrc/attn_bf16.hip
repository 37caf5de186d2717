// Bidirectional block-diagonal attention on bf16 MFMA (gfx950), flash style:
// scores are never written to memory.  Two copies of one kernel: the general one
// keeps softmax statistics per query in fp32 and updates them block by block
// (online softmax); the other one handles the workgroups whose scores are
// provably small (from key and query norms) and exponentiates them directly,
// with no running maximum at all.  On this hardware the kernel is limited by the
// vector issue port (every MFMA also takes about 12 of its cycles, every exp2
// 16), so vector instructions per score are what counts.
//
// Work decomposition: one workgroup (NWV = 4 or 8 waves) = 32*NT*NWV query rows of
// one segment and one head; each wave owns NT tiles of 32 query rows.  Eight
// waves share one staged K/V tile stream per CU instead of two workgroups
// staging the same tiles twice; four waves waste less on short segments.  K and V^T
// tiles of 64 keys are staged in LDS by direct global->LDS loads (a ring of
// three stages, the loads of tile t+2 are in flight while tile t is consumed)
// and shared by the waves of the workgroup.  Every K / V^T
// fragment read from LDS feeds NT MFMAs: NT = 2 halves the LDS bytes per FLOP.
//
// The kernel computes S^T = K * Q^T (keys are the MFMA row dimension).  In the
// 32x32 accumulator layout a lane then holds ONE query column and 16 keys, so
//   * the running max / rescale factor are one scalar per lane and query tile,
//   * the exponentiated scores, packed to bf16 in place, already have the
//     register layout of the B operand of O^T += V^T * P^T (the contraction
//     index only has to be enumerated in the same order on both operands, so V^T
//     is stored in LDS in the key order the accumulator happens to have),
//   * P never goes through LDS.
// V arrives already transposed ([head_dim, keys], keys contiguous, the four
// quarters of every aligned group of 16 keys stored in the order 0,2,1,3 - see
// the V^T tile comment below) and zero in the padding columns.  The online
// softmax advances in blocks of 32 keys (one accumulator tile per query tile),
// which keeps the live score registers at 16*NT.
//
// When head_dim is an odd multiple of 16 the V^T tile is padded to a multiple of
// 32 rows; the first padding row is filled with ones, which makes the MFMA
// produce the softmax denominator (sum of the bf16-rounded probabilities) for
// free; otherwise the denominator is accumulated on the vector ALU.
#include "tcmv_internal.h"
#include "device_utils.h"
#include <algorithm>
#include <type_traits>

namespace tcmv {

namespace {
constexpr int BKV = 64;
constexpr int kThreads4 = 256;
constexpr int kStages = 3;          // LDS ring: tile t (V still in use), tile t+1 (K in use), tile t+2 (in flight)
typedef __attribute__((address_space(1))) const void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;
}  // namespace

// One wave-wide 16-byte-per-lane load global -> LDS through a buffer descriptor over `bytes` bytes at `base` (base,
// size and `soff` are wave-uniform; `voff` is the lane's byte offset).  Lane l writes 16 bytes at lds + 16 l; bytes
// past the end of the buffer read as zero.
__device__ __forceinline__ void buffer_load_lds16(const void* base, uint32_t bytes, void* lds, uint32_t voff, uint32_t soff) {
  const uint64_t v = reinterpret_cast<uint64_t>(base);
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<void*>(((uint64_t)hi << 32) | lo), 0,
                                                                      (int)__builtin_amdgcn_readfirstlane(bytes), 0x00020000);
  __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lptr_t)lds, 16, voff, soff, 0, 0);
}

// One 16-byte-per-lane LDS read issued outside the compiler's view (inline assembly): the compiler neither moves it nor
// waits for it; the caller places the s_waitcnt itself.  addr: LDS byte address of the lane, OFF: immediate offset.
template <int OFF>
__device__ __forceinline__ void lds_read16(bf16x8& dst, uint32_t addr, std::integral_constant<int, OFF>) {
  static_assert(OFF >= 0 && OFF < 65536, "the offset field of an LDS read has 16 bits");
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFF) : "memory");
}

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
  static constexpr int KROWCH = KCH | 1;                   // chunks per K row in LDS incl. padding
  static constexpr int NW = KROWCH + DH / 8;               // wave-wide 1 KB loads per tile (K rows, then V^T rows)
};

// V^T tile in LDS: row = head-dim index (128 bytes = 64 keys).  Inside a row the
// keys are stored in the order the PV MFMA wants them: 16-byte chunk (2G + g)
// holds keys {16G + 4g + 0..3, 16G + 8 + 4g + 0..3}, i.e. exactly the 8 keys a
// lane of half-wave g contributes to k-step G.  The transposed-V buffer in
// global memory already has this key order (the producer writes key kk of a
// 16-group at position [0,2,1,3][kk/4]*4 + kk%4), so a chunk is one 16-byte
// global load.  Chunks are XOR-swizzled by (row/2)%8: the LDS serves 16 lanes x 16
// bytes per clock over 64 banks and two 128-byte rows span the banks, so 16
// consecutive rows reading the same logical chunk land on 16 different bank groups.
// PRESC: the queries already carry the factor softmax scale * log2(e) (the QKV projection
// applies it before rounding to bf16), so a score is directly the exponent of 2.
// FAST: the kernel exists twice.  Both copies evaluate the same bound per workgroup (see below);
// the FAST copy processes the workgroups whose scores are provably small without any softmax
// reference and returns at once for the others, the other copy does the opposite.  Two
// kernels instead of one branch keep the register allocation of each loop to itself.
template <int DH, int NT, int NWV, bool PRESC, bool FAST>
__global__ __launch_bounds__(NWV * 64, 8 / NWV) void attn_bf16_kernel(AttnArgs a) {
  using C = AttnCfg<DH>;
  constexpr int NTHREADS = NWV * 64;
  constexpr int NLD = (C::NW + NWV - 1) / NWV;     // tile loads per wave
  constexpr int WQ = 32 * NT;             // query rows per wave
  __shared__ __attribute__((aligned(16))) uint8_t smem[kStages * C::STAGE];

  // the key-norm block of the next layer is cleared by the first workgroup of the first kernel of this launch
  if (FAST && blockIdx.x == 0 && a.kmax_clear)
    for (int i = threadIdx.x; i < a.n_clear; i += NTHREADS) a.kmax_clear[i] = 0u;
  const int total = a.n_work * a.heads;
  const int chunk = (total + 7) >> 3;
  const int p = (int)(blockIdx.x & 7) * chunk + (int)(blockIdx.x >> 3);
  if (p >= total) return;
  const int head = p / a.n_work;
  const AttnWork w = a.work[p - head * a.n_work];

  // the reference-tracking copy runs after the other one (same stream), which has recorded whether it
  // left any workgroup behind
  if (!FAST && a.kmax2 && a.any_left && *a.any_left == 0) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  __builtin_assume(tid >= 0 && tid < NTHREADS);
  const int lr = lane & 31, lg = lane >> 5;
  const uint16_t* Q = reinterpret_cast<const uint16_t*>(a.q);
  const uint16_t* K = reinterpret_cast<const uint16_t*>(a.k);
  const uint16_t* VT = reinterpret_cast<const uint16_t*>(a.v);

  // padding rows of the V^T tiles: ones row (denominator) then zeros
  if (C::DHP > DH) {
    for (int i = tid; i < kStages * (C::DHP - DH) * (BKV / 2); i += NTHREADS) {
      const int buf = i / ((C::DHP - DH) * (BKV / 2));
      const int rem = i - buf * ((C::DHP - DH) * (BKV / 2));
      const int row = DH + rem / (BKV / 2), c2 = rem % (BKV / 2);
      const uint32_t val = (C::ONES && row == DH) ? 0x3F803F80u : 0u;
      *reinterpret_cast<uint32_t*>(smem + buf * C::STAGE + C::K_BYTES + row * (BKV * 2) + c2 * 4) = val;
    }
  }

  // query fragments (B operand of S^T = K Q^T), kept in registers for the whole kernel
  bf16x8 qf[NT][C::KS];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    int qi = wave * WQ + nt * 32 + lr;
    if (qi >= w.nq) qi = w.nq - 1;
    const uint16_t* qp = Q + (size_t)(w.q0 + qi) * a.ldqk + head * DH + lg * 8;
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks) qf[nt][ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 16);
  }
  // Does this workgroup need a running maximum at all?  |score| <= |q| * |k| (Cauchy-Schwarz);
  // with the largest key norm of the segment (computed by knorm_kernel) every exponent of its
  // queries is bounded.  If the bound is at most kSafeExp, 2^score cannot overflow or vanish in
  // fp32 / bf16, the softmax needs no reference at all (it is shift invariant), and the
  // per-element maximum, subtraction and rescaling are dropped.
  constexpr float kSafeExp = 64.0f;
  if (!a.kmax2) {            // no key norms: the caller wants every workgroup to take the reference-tracking copy
    if (FAST) return;
  } else {
    const float kmax2 = __uint_as_float(a.kmax2[((size_t)w.seg * a.heads + head) * kKmaxStride]);
    const float c2 = PRESC ? 1.0f : a.scale * a.scale;
    bool ok = true;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      float q2 = 0.f;
#pragma unroll
      for (int ks = 0; ks < C::KS; ++ks)
#pragma unroll
        for (int e = 0; e < 8; ++e) { const float v = (float)qf[nt][ks][e]; q2 = fmaf(v, v, q2); }
      q2 += __shfl_xor(q2, 32, 64);                       // the two half-waves hold the two halves of a row
      ok = ok && (q2 * kmax2 * c2 <= kSafeExp * kSafeExp);
    }
    const bool fast = __syncthreads_and(ok) != 0;
    if (FAST && !fast && a.any_left && tid == 0) atomicOr(a.any_left, 1u);
    if (fast != FAST) return;
  }

  // Tile staging: global -> LDS directly (no registers, no LDS store instructions).  One
  // wave-wide load writes 64 consecutive 16-byte chunks of LDS (base + lane*16), so each
  // lane fetches the global chunk that belongs at its LDS position: K rows are stored
  // with a padding chunk (odd chunk count per row), V^T chunks at their swizzled position.
  // The tile is C::NW wave-loads; wave w issues loads w, w+NWV, w+2*NWV, ...
  // Both operands are addressed through buffer descriptors (base and size in SGPRs): a lane keeps one 32-bit byte
  // offset per load, the tile index goes into the scalar offset, and rows past the end of the key buffer (last
  // tile of the last segment) simply read as zero instead of being clamped - their scores are masked anyway.
  uint32_t goff[NLD];             // byte offset of this lane's tile-0 chunk from K (or VT)
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
#pragma unroll
  for (int i = 0; i < NLD; ++i) {
    const int n = wave_u + NWV * i;
    const int L = n * 64 + lane;                       // K part: chunk index incl. padding chunks
    const int rowk = L / C::KROWCH;
    int cck = L - rowk * C::KROWCH;
    if (cck >= C::KCH) cck = 0;                        // padding chunk: any valid source
    const int Lv = (n - C::KROWCH) * 64 + lane;        // V^T part
    const int rowv = Lv >> 3, lc = (Lv & 7) ^ ((rowv >> 1) & 7);
    const uint32_t ko = (uint32_t)(head * DH) + (uint32_t)(w.seg_start + rowk) * (uint32_t)a.ldqk + cck * 8;
    const uint32_t vo = (uint32_t)(head * DH + rowv) * (uint32_t)a.ldv + (uint32_t)w.v0 + lc * 8;
    goff[i] = ((n < C::KROWCH) ? ko : vo) * 2u;
  }
  const uint32_t kstep = (uint32_t)BKV * (uint32_t)a.ldqk * 2u;
  const uint32_t bytes_k = (uint32_t)(((uint64_t)(a.t_total - 1) * (uint64_t)a.ldqk + (uint64_t)a.heads * DH) * 2ull);
  const uint32_t bytes_v = (uint32_t)((uint64_t)a.heads * DH * (uint64_t)a.ldv * 2ull);
  auto load_tile = [&](int t, int buf, bool) {
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int n = wave_u + NWV * i;
      if (n < C::NW) {
        const bool is_k = n < C::KROWCH;
        const uint32_t soff = is_k ? (uint32_t)t * kstep : (uint32_t)t * (BKV * 2);
        uint8_t* dst = smem + buf * C::STAGE + (is_k ? n * 1024 : C::K_BYTES + (n - C::KROWCH) * 1024);
        buffer_load_lds16(is_k ? (const void*)K : (const void*)VT, is_k ? bytes_k : bytes_v, dst, goff[i], soff);
      }
    }
  };
  auto wait_tile = [&]() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); };

  f32x16 o[C::MT][NT];
#pragma unroll
  for (int mt = 0; mt < C::MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int v = 0; v < 16; ++v) o[mt][nt][v] = 0.f;
  float m_run[NT], l_run[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) { m_run[nt] = -INFINITY; l_run[nt] = 0.f; }
  const float cs = a.scale;   // softmax scale * log2(e)

  const int n_tiles = (w.seg_len + BKV - 1) / BKV;
  const bool ragged = (w.seg_len % BKV) != 0;

  // ---- building blocks -------------------------------------------------------------
  // K fragments (A operand of the score MFMAs) of 32-key block kb of a staged tile; they are
  // requested one region before their use
  bf16x8 kf[C::KS > 6 ? C::KS : 6];      // K fragments; the pipelined region uses all six as a ring of fragments
  auto k_frags = [&](const uint8_t* sk, int kb) {
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks)
      kf[ks] = *reinterpret_cast<const bf16x8*>(sk + (kb * 32 + lr) * C::KSTR + (2 * ks + lg) * 16);
  };
  // S^T block: 32 keys x 32*NT queries from the fragments in kf
  auto score_block = [&](f32x16 (&s)[NT]) {
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int v = 0; v < 16; ++v) s[nt][v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        s[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], qf[nt][ks], s[nt], 0, 0, 0);
  };
  auto mask_block = [&](f32x16 (&s)[NT], int key0) {
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int key = key0 + 8 * (v >> 2) + 4 * lg + (v & 3);
        if (key >= w.seg_len) s[nt][v] = -INFINITY;
      }
  };
  // Statistics of a finished score block (per lane = per query column), branch-free: block
  // maximum, decision whether the softmax reference has to move, factor for what has been
  // accumulated so far.  The reference m_run only moves when the block maximum exceeds it
  // by more than kLazy (in log2 units): probabilities may then exceed 1 (by at most
  // 2^kLazy), which changes nothing mathematically because numerator and denominator share
  // the reference, and it makes the rescaling of O rare.  Returns whether this lane's
  // reference moved.
  constexpr float kLazy = 8.0f;
  auto stats_block = [&](const f32x16 (&s)[NT], float (&alpha)[NT]) -> bool {
    bool need_rescale = false;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      float mx = s[nt][0];
#pragma unroll
      for (int v = 1; v < 16; ++v) mx = fmaxf(mx, s[nt][v]);
      {   // combine the two half-waves (same query, other keys) on the vector ALU, no LDS round trip:
          // after the swap one result holds the lower half's value in every lane, the other the upper half's
        const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
        mx = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
      }
      const bool move = (mx - m_run[nt]) * cs > kLazy;     // also true for the first block (m_run = -inf)
      const float m_new = move ? mx : m_run[nt];
      alpha[nt] = move ? __builtin_amdgcn_exp2f((m_run[nt] - m_new) * cs) : 1.0f;
      m_run[nt] = m_new;
      need_rescale = need_rescale || move;
      if (!C::ONES) l_run[nt] *= alpha[nt];
    }
    return need_rescale;
  };
  auto rescale = [&](const float (&alpha)[NT]) {
#pragma unroll
    for (int mt = 0; mt < C::MT; ++mt)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[mt][nt][v] *= alpha[nt];
  };
  // One region = one 32-key block of the online softmax, one basic block of code in the
  // unmasked case: the score MFMAs of the NEXT block (fragments already in kf), the
  // exponentials of the CURRENT block, its PV MFMAs, the statistics of the next block and the
  // request of the K fragments for the region after this one.  The MFMA is asynchronous but
  // issue is in order, so the vector work (fma / exp2 / pack / max) is spread between the
  // MFMAs by the scheduler (interleaving strategy below) instead of following them in a lump.
  // The only branch, the rare rescaling of O, is taken by the caller between regions.
  auto region = [&](auto masked, f32x16 (&s_next)[NT], const f32x16 (&s_cur)[NT], const uint8_t* sv_cur, int kb_cur,
                    const uint8_t* sk_pref, int kb_pref, bool next_valid, bool next_mask, int next_key0,
                    float (&alpha)[NT]) -> bool {
    float mc[NT], psum[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) { mc[nt] = m_run[nt] * cs; psum[nt] = 0.f; }
    // probabilities of keys 16j..16j+15 of the current block, packed as the PV B operand
    auto exp_half = [&](int j, bf16x8 (&pf)[NT]) {
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        uint32_t pk[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float a0 = __builtin_amdgcn_exp2f(fmaf(s_cur[nt][8 * j + 2 * e], cs, -mc[nt]));
          const float a1 = __builtin_amdgcn_exp2f(fmaf(s_cur[nt][8 * j + 2 * e + 1], cs, -mc[nt]));
          if (!C::ONES) psum[nt] += a0 + a1;
          pk[e] = pack_bf16x2(a0, a1);
        }
        const uint4 u = make_uint4(pk[0], pk[1], pk[2], pk[3]);
        pf[nt] = __builtin_bit_cast(bf16x8, u);
      }
    };
    auto v_frags = [&](int j, bf16x8 (&vf)[C::MT]) {
#pragma unroll
      for (int mt = 0; mt < C::MT; ++mt) {
        const int row = mt * 32 + lr;
        vf[mt] = *reinterpret_cast<const bf16x8*>(sv_cur + row * (BKV * 2) + (((2 * (2 * kb_cur + j) + lg) ^ ((row >> 1) & 7)) << 4));
      }
    };
    auto pv = [&](const bf16x8 (&vf)[C::MT], const bf16x8 (&pf)[NT]) {
#pragma unroll
      for (int mt = 0; mt < C::MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
          o[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[mt], pf[nt], o[mt][nt], 0, 0, 0);
    };
    bf16x8 pf0[NT], pf1[NT], vf0[C::MT], vf1[C::MT];
    score_block(s_next);
    exp_half(0, pf0);
    v_frags(0, vf0);
    exp_half(1, pf1);
    pv(vf0, pf0);
    v_frags(1, vf1);
    pv(vf1, pf1);
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
      if (!C::ONES) l_run[nt] += psum[nt];
    k_frags(sk_pref, kb_pref);
    bool need = false;
    if constexpr (decltype(masked)::value) {
      if (next_mask) mask_block(s_next, next_key0);
      if (next_valid) need = stats_block(s_next, alpha);
    } else {
      need = stats_block(s_next, alpha);
    }
    if constexpr (decltype(masked)::value) {
      __builtin_amdgcn_iglp_opt(3);
    } else {
      constexpr int n_mfma = C::KS * NT + 2 * C::MT * NT;
      constexpr int n_valu = 16 * NT * 3 + 8 * NT + 16 * NT + 24;      // fma, exp2, max / pack / statistics and addresses
#pragma unroll
      for (int i = 0; i < n_mfma; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x402, (n_valu + n_mfma - 1) / n_mfma, 0);
      }
    }
    return need;
  };

  // The same region without a softmax reference (see `fast` above): probabilities are
  // 2^score, nothing is tracked and nothing is ever rescaled.
  auto region_fast = [&](auto masked, f32x16 (&s_next)[NT], const f32x16 (&s_cur)[NT], const uint8_t* sv_cur, int kb_cur,
                         const uint8_t* sk_pref, int kb_pref, bool next_mask, int next_key0) {
    float psum[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) psum[nt] = 0.f;
    auto exp_half = [&](int j, bf16x8 (&pf)[NT]) {
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        uint32_t pk[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float x0 = s_cur[nt][8 * j + 2 * e], x1 = s_cur[nt][8 * j + 2 * e + 1];
          const float a0 = __builtin_amdgcn_exp2f(PRESC ? x0 : x0 * cs);
          const float a1 = __builtin_amdgcn_exp2f(PRESC ? x1 : x1 * cs);
          if (!C::ONES) psum[nt] += a0 + a1;
          pk[e] = pack_bf16x2(a0, a1);
        }
        const uint4 u = make_uint4(pk[0], pk[1], pk[2], pk[3]);
        pf[nt] = __builtin_bit_cast(bf16x8, u);
      }
    };
    auto v_frags = [&](int j, bf16x8 (&vf)[C::MT]) {
#pragma unroll
      for (int mt = 0; mt < C::MT; ++mt) {
        const int row = mt * 32 + lr;
        vf[mt] = *reinterpret_cast<const bf16x8*>(sv_cur + row * (BKV * 2) + (((2 * (2 * kb_cur + j) + lg) ^ ((row >> 1) & 7)) << 4));
      }
    };
    auto pv = [&](const bf16x8 (&vf)[C::MT], const bf16x8 (&pf)[NT]) {
#pragma unroll
      for (int mt = 0; mt < C::MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
          o[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[mt], pf[nt], o[mt][nt], 0, 0, 0);
    };
    bf16x8 pf0[NT], pf1[NT], vf0[C::MT], vf1[C::MT];
    score_block(s_next);
    exp_half(0, pf0);
    v_frags(0, vf0);
    exp_half(1, pf1);
    pv(vf0, pf0);
    v_frags(1, vf1);
    pv(vf1, pf1);
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
      if (!C::ONES) l_run[nt] += psum[nt];
    k_frags(sk_pref, kb_pref);
    if constexpr (decltype(masked)::value) {
      if (next_mask) mask_block(s_next, next_key0);
      __builtin_amdgcn_iglp_opt(3);
    } else {
      constexpr int n_mfma = C::KS * NT + 2 * C::MT * NT;
      constexpr int n_valu = 16 * NT * (PRESC ? 1 : 2) + 8 * NT + (C::ONES ? 0 : 16 * NT) + 12;   // exp2 (+ scale), pack, sums, addresses
#pragma unroll
      for (int i = 0; i < n_mfma; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x402, (n_valu + n_mfma - 1) / n_mfma, 0);
      }
    }
  };

  // The same region with the LDS fragment reads under explicit control (head size 80, two query tiles per wave).
  // The 11 fragments of a region - 5 of K for the score MFMAs, 3 + 3 of V^T for the two halves of the PV product -
  // form one stream through a ring of six registers: fragment g+5 is requested right after the MFMAs of fragment g
  // have been issued (into the register of fragment g-1), so every read has about five fragments' worth of MFMAs
  // (>= 300 cycles) to arrive.  Position 11 of a region is a gap (no read), which keeps the ring positions static.
  // The reads are inline assembly: the compiler does not see them as LDS reads (left to itself it sinks every V^T read
  // to just before its MFMA and waits there), so the waits are explicit too; LDS reads return in order, and nothing
  // else in the loop uses that counter.  The vector work is placed by hand as well: two exponentials behind each of
  // the first 16 MFMAs, their conversions one step later (no wait state after v_exp), scheduling fences in between.
  // On entry kf[0..4] hold (or are about to receive) the K fragments of this region, on exit those of the next.
  // Same arithmetic in the same order as region_fast: the results are bit-identical.
  constexpr bool PIPE = FAST && DH == 80 && NT == 2;
  const uint32_t lds0 = (uint32_t)(uintptr_t)(lptr_t)smem;
  const uint32_t koff = (uint32_t)(lr * C::KSTR + lg * 16);
  uint32_t voff[2][2];
#pragma unroll
  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
    for (int j = 0; j < 2; ++j) voff[kb][j] = (uint32_t)(lr * (BKV * 2) + (((4 * kb + 2 * j + lg) ^ ((lr >> 1) & 7)) << 4));
  auto region_pipe = [&](f32x16 (&s_next)[NT], const f32x16 (&s_cur)[NT], uint32_t sv_addr, auto kbc, uint32_t sk_addr, auto kbp) {
    if constexpr (PIPE) {
    constexpr int kb_cur = decltype(kbc)::value, kb_pref = decltype(kbp)::value;
    const uint32_t va[2] = {sv_addr + voff[kb_cur][0], sv_addr + voff[kb_cur][1]};
    const uint32_t ka = sk_addr + koff;
    float ex[4];                       // exponentials of the previous step, converted in this one
    uint32_t pk[2][NT][4];             // packed probabilities: [half][query tile][4 x 2 bf16]
    bf16x8 pf[2][NT];
    static_for<11>([&](auto ic) {
      constexpr int i = decltype(ic)::value;
      constexpr int slot = i % 6;
      auto conv = [&]() {              // conversions of the exponentials of the previous step (no wait state after v_exp)
        if constexpr (i >= 1 && i <= 8) {
          constexpr int e0 = 4 * (i - 1);                 // exponentials e0 .. e0+3: half e/16, tile (e%16)/8, element e%8
          constexpr int hj = e0 / 16, nt = (e0 % 16) / 8, q = (e0 % 8) / 2;
          pk[hj][nt][q] = pack_bf16x2(ex[0], ex[1]);
          pk[hj][nt][q + 1] = pack_bf16x2(ex[2], ex[3]);
          if constexpr (q == 2) {
            const uint4 u = make_uint4(pk[hj][nt][0], pk[hj][nt][1], pk[hj][nt][2], pk[hj][nt][3]);
            pf[hj][nt] = __builtin_bit_cast(bf16x8, u);
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      };
      // one wait per three fragments (a wait costs an issue slot even when nothing is outstanding): before
      // fragments i, i+1, i+2 are used, at most the two reads behind them may be outstanding (i+3 and i+4; position
      // 11 is the gap, so behind 9 and 10 come the first two of the next region)
      auto waitf = [&]() {
        if constexpr (i % 3 == 0) {
          if constexpr (i < 9)
            asm volatile("s_waitcnt lgkmcnt(2)" : "+v"(kf[slot]), "+v"(kf[(i + 1) % 6]), "+v"(kf[(i + 2) % 6]));
          else
            asm volatile("s_waitcnt lgkmcnt(2)" : "+v"(kf[slot]), "+v"(kf[(i + 1) % 6]));
        }
        __builtin_amdgcn_sched_barrier(0);
      };
      auto mfma = [&](auto ntc) {
        constexpr int nt = decltype(ntc)::value;
        if constexpr (i < 5) {
          if constexpr (i == 0) {
#pragma unroll
            for (int v = 0; v < 16; ++v) s_next[nt][v] = 0.f;
          }
          s_next[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[slot], qf[nt][i], s_next[nt], 0, 0, 0);
        } else {
          constexpr int hj = (i - 5) / 3, mt = (i - 5) % 3;
          o[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[slot], pf[hj][nt], o[mt][nt], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
      };
      auto exps = [&](auto ntc) {      // two exponentials behind each of the first 16 MFMAs
        constexpr int nt = decltype(ntc)::value;
        if constexpr (i < 8) {
          constexpr int e0 = 4 * i + 2 * nt;
          constexpr int hj = e0 / 16, ent = (e0 % 16) / 8, el = e0 % 8;
          const float x0 = s_cur[ent][8 * hj + el], x1 = s_cur[ent][8 * hj + el + 1];
          ex[2 * nt] = __builtin_amdgcn_exp2f(PRESC ? x0 : x0 * cs);
          ex[2 * nt + 1] = __builtin_amdgcn_exp2f(PRESC ? x1 : x1 * cs);
        }
        __builtin_amdgcn_sched_barrier(0);
      };
      auto readf = [&]() {             // request fragment i+5 into the register of fragment i-1
        constexpr int nslot = (i + 5) % 6;
        if constexpr (i <= 2)
          lds_read16(kf[nslot], va[0], std::integral_constant<int, i * 32 * BKV * 2>{});
        else if constexpr (i <= 5)
          lds_read16(kf[nslot], va[1], std::integral_constant<int, (i - 3) * 32 * BKV * 2>{});
        else if constexpr (i >= 7)
          lds_read16(kf[nslot], ka, std::integral_constant<int, kb_pref * 32 * C::KSTR + (i - 7) * 32>{});
        __builtin_amdgcn_sched_barrier(0);
      };
      constexpr std::integral_constant<int, 0> n0{};
      constexpr std::integral_constant<int, 1> n1{};
      // order inside a step (measured: requesting the next fragment between the second MFMA and its exponentials, and
      // converting behind the first MFMA, is the fastest of ten orders tried; the spread is 3 %)
      waitf(); mfma(n0); conv(); exps(n0); mfma(n1); readf(); exps(n1);
    });
    // position 11 is the gap; the fifth K fragment of the next region goes into ring position 16 % 6 = 4
    lds_read16(kf[4], ka, std::integral_constant<int, kb_pref * 32 * C::KSTR + 4 * 32>{});
    __builtin_amdgcn_sched_barrier(0);
    }
  };

  // ---- pipeline ---------------------------------------------------------------------
  // LDS ring of three stages.  At the barrier that opens iteration t, tile t+1 has landed (its
  // loads were issued one iteration earlier) and every wave is done with tile t-1, so tile
  // t+2 can be requested into that stage; nothing else synchronises the waves.
  load_tile(0, 0, ragged && n_tiles == 1);
  if (n_tiles > 1) load_tile(1, 1, ragged && n_tiles == 2);
  // tile 0 (the older one) has landed once at most a tile's worth of loads is outstanding; waves
  // issue NW/NWV or NW/NWV+1 loads per tile, so the smaller count is the safe threshold for all
  if (n_tiles > 1) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(C::NW / NWV) : "memory");
  else wait_tile();
  __syncthreads();
  f32x16 s0[NT], s1[NT];
  {
    float alpha[NT];
    k_frags(smem, 0);
    score_block(s0);
    k_frags(smem, 1);
    if (ragged && n_tiles == 1) mask_block(s0, 0);
    if (!FAST) (void)stats_block(s0, alpha);      // O is still zero: nothing to rescale
  }
  int st = 0;                                     // stage of tile t
  // iteration t: block 0 of tile t (scores in s0) and block 1 (scored in the first region);
  // the second region already scores block 0 of tile t+1.  For the last tile that extra block
  // comes from a stale stage and is ignored.
  auto iteration = [&](auto masked, int t) {
    const int j0 = t * BKV;
    const int st1 = (st + 1 == kStages) ? 0 : st + 1;
    const int st2 = (st1 + 1 == kStages) ? 0 : st1 + 1;
    const uint8_t* sv = smem + st * C::STAGE + C::K_BYTES;
    const uint8_t* sk1 = smem + st1 * C::STAGE;
    wait_tile();
    // The barrier orders two things: every wave's tile loads have landed (the wait above) and every wave is done
    // reading tile t-1 (each wave has waited for those fragments before it used them).  The pipelined regions keep
    // LDS reads of tile t+1 in flight across it, so they take the bare barrier, not one that first drains the LDS
    // counter.
    if constexpr (FAST && PIPE && !decltype(masked)::value) __builtin_amdgcn_s_barrier();
    else __syncthreads();
    if (t + 2 < n_tiles) load_tile(t + 2, st2, ragged && (t + 3 == n_tiles));
    if constexpr (FAST && PIPE && !decltype(masked)::value) {
      const uint32_t sva = lds0 + (uint32_t)(st * C::STAGE + C::K_BYTES), ska = lds0 + (uint32_t)(st1 * C::STAGE);
      region_pipe(s1, s0, sva, std::integral_constant<int, 0>{}, ska, std::integral_constant<int, 0>{});
      region_pipe(s0, s1, sva, std::integral_constant<int, 1>{}, ska, std::integral_constant<int, 1>{});
    } else if constexpr (FAST) {
      region_fast(masked, s1, s0, sv, 0, sk1, 0, ragged && t + 1 == n_tiles, j0 + 32);
      region_fast(masked, s0, s1, sv, 1, sk1, 1, ragged && t + 2 == n_tiles, j0 + BKV);
    } else {
      float alpha[NT];
      bool need = region(masked, s1, s0, sv, 0, sk1, 0, true, ragged && t + 1 == n_tiles, j0 + 32, alpha);
      if (__builtin_expect(__any(need), 0)) rescale(alpha);
      need = region(masked, s0, s1, sv, 1, sk1, 1, t + 1 < n_tiles, ragged && t + 2 == n_tiles, j0 + BKV, alpha);
      if (__builtin_expect(__any(need), 0)) rescale(alpha);
    }
    st = st1;
  };
  // only the last two iterations can meet masked blocks (ragged tail) or the ignored extra block
  int t = 0;
  if constexpr (PIPE) {
    // The K fragments read above were the compiler's own loads: make it finish them here (it waits before the first
    // use it sees), so that no wait of its own for them ends up inside the loop, where it would also wait for the
    // ring's reads.
    asm volatile("" : "+v"(kf[0]), "+v"(kf[1]), "+v"(kf[2]), "+v"(kf[3]), "+v"(kf[4]));
  }
  // A segment that fills its last tile needs no masks at all: its last two tiles run through the mask-free body
  // too (the extra block that the last region scores comes from a stale stage, stays inside LDS and is ignored).
  const int n_plain = (PIPE && !ragged) ? n_tiles : n_tiles - 2;
  for (; t < n_plain; ++t) iteration(std::false_type{}, t);
  if constexpr (PIPE) {                // the ring's reads were issued outside the compiler's view: let them land
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(kf[0]), "+v"(kf[1]), "+v"(kf[2]), "+v"(kf[3]), "+v"(kf[4]));
  }
  for (; t < n_tiles; ++t) iteration(std::true_type{}, t);

  // ---- normalise and store: lane holds query (lane & 31), head-dim rows 8*(v/4) + 4*lg + v%4
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    float l;
    if (C::ONES) {
      constexpr int r = DH % 32;                          // row of the ones line inside its tile (16)
      l = __shfl(o[DH / 32][nt][4 * (r / 8)], lr, 64);    // held by the lanes of the lower half-wave
    } else {
      l = l_run[nt] + __shfl_xor(l_run[nt], 32, 64);
    }
    const float inv = 1.0f / l;
    const int qi = wave * WQ + nt * 32 + lr;
    if (qi < w.nq) {
      uint16_t* op = reinterpret_cast<uint16_t*>(a.out) + (size_t)(w.q0 + qi) * a.ldo + head * DH;
#pragma unroll
      for (int mt = 0; mt < C::MT; ++mt)
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) {
          const int dh0 = mt * 32 + 8 * vq + 4 * lg;
          if (dh0 < DH) {
            uint2 pk;
            pk.x = pack_bf16x2(o[mt][nt][4 * vq] * inv, o[mt][nt][4 * vq + 1] * inv);
            pk.y = pack_bf16x2(o[mt][nt][4 * vq + 2] * inv, o[mt][nt][4 * vq + 3] * inv);
            *reinterpret_cast<uint2*>(op + dh0) = pk;
          }
        }
    }
  }
}

template <bool PRESC, bool FAST>
static hipError_t launch_attn_t(const AttnArgs& a, unsigned grid, hipStream_t s) {
#define TCMV_ATTN_CASE(D)                                                                                     \
  case D:                                                                                                     \
    if (a.bq == 512) hipLaunchKernelGGL((attn_bf16_kernel<D, 2, 8, PRESC, FAST>), dim3(grid), dim3(512), 0, s, a);  \
    else if (a.bq == 256) hipLaunchKernelGGL((attn_bf16_kernel<D, 2, 4, PRESC, FAST>), dim3(grid), dim3(kThreads4), 0, s, a); \
    else hipLaunchKernelGGL((attn_bf16_kernel<D, 1, 4, PRESC, FAST>), dim3(grid), dim3(kThreads4), 0, s, a);  \
    break;
  switch (a.dh) {
    TCMV_ATTN_CASE(32) TCMV_ATTN_CASE(64) TCMV_ATTN_CASE(80)
    case 96:   // the register file holds one query tile per wave only
      if (a.bq != 128) return hipErrorInvalidValue;
      hipLaunchKernelGGL((attn_bf16_kernel<96, 1, 4, PRESC, FAST>), dim3(grid), dim3(kThreads4), 0, s, a);
      break;
    default: return hipErrorInvalidValue;
  }
#undef TCMV_ATTN_CASE
  return hipGetLastError();
}

hipError_t launch_attn_bf16(const AttnArgs& a, hipStream_t s) {
  if (a.n_work == 0 || a.heads == 0) return hipSuccess;
  const int64_t total = (int64_t)a.n_work * a.heads;
  if (total > (1 << 30)) return hipErrorInvalidValue;
  if (a.ldqk % 8 || a.ldv % 8 || a.ldo % 4) return hipErrorInvalidValue;
  if (a.bq != 128 && a.bq != 256 && a.bq != 512) return hipErrorInvalidValue;
  // operands are addressed in bytes, 32 bits
  if ((double)a.t_total * (double)a.ldqk * 2.0 >= 4294967296.0 || (double)a.heads * a.dh * (double)a.ldv * 2.0 >= 4294967296.0) return hipErrorInvalidValue;
  const unsigned grid = (unsigned)(((total + 7) / 8) * 8);
  // with key norms both copies visit every work item and each item is processed by exactly one of them;
  // without, only the reference-tracking copy runs
  if (a.kmax2) {
    const hipError_t e = a.prescaled ? launch_attn_t<true, true>(a, grid, s) : launch_attn_t<false, true>(a, grid, s);
    if (e != hipSuccess) return e;
  }
  return a.prescaled ? launch_attn_t<true, false>(a, grid, s) : launch_attn_t<false, false>(a, grid, s);
}

// Largest squared key norm per (segment, head), the input of the attention kernel's decision
// whether a running maximum is needed.  A workgroup takes 32 rows: every thread squares and
// sums 16-byte chunks (coalesced along the row), the chunks of a head are added up through
// LDS, then one thread per head walks the 32 rows and issues one atomic max per run of rows
// of the same segment (norms are >= 0, so their float bits order like unsigned integers).
__global__ __launch_bounds__(256) void knorm_kernel(const uint16_t* k, int64_t ldk, int64_t rows, int heads, int cph,
                                                    const int32_t* row_seg, uint32_t* kmax2) {
  constexpr int R = 32;
  extern __shared__ float part[];                    // [R][heads * cph] chunk sums, then [R][heads] norms
  const int cpr = heads * cph;                       // 16-byte chunks per row
  const int64_t r0 = (int64_t)blockIdx.x * R;
  const int nr = (int)min((int64_t)R, rows - r0);
  for (int i = threadIdx.x; i < nr * cpr; i += 256) {
    const int r = i / cpr, c = i - r * cpr;
    const uint4 u = *reinterpret_cast<const uint4*>(k + (r0 + r) * ldk + c * 8);
    const uint32_t wds[4] = {u.x, u.y, u.z, u.w};
    float sq = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float lo = __uint_as_float(wds[j] << 16), hi = __uint_as_float(wds[j] & 0xFFFF0000u);
      sq = fmaf(lo, lo, sq);
      sq = fmaf(hi, hi, sq);
    }
    part[i] = sq;
  }
  __syncthreads();
  float* norm = part + R * cpr;
  for (int i = threadIdx.x; i < nr * heads; i += 256) {
    const int r = i / heads, h = i - r * heads;
    float sq = 0.f;
    for (int c = 0; c < cph; ++c) sq += part[r * cpr + h * cph + c];
    norm[i] = sq;
  }
  __syncthreads();
  if ((int)threadIdx.x < heads) {
    const int h = threadIdx.x;
    int seg = row_seg[r0];
    float mx = 0.f;
    for (int r = 0; r < nr; ++r) {
      const int sg = row_seg[r0 + r];
      if (sg != seg) {
        atomicMax(kmax2 + ((size_t)seg * heads + h) * kKmaxStride, __float_as_uint(mx));
        seg = sg;
        mx = 0.f;
      }
      mx = fmaxf(mx, norm[r * heads + h]);
    }
    atomicMax(kmax2 + ((size_t)seg * heads + h) * kKmaxStride, __float_as_uint(mx));
  }
}

hipError_t launch_knorm(const void* k, int64_t ldk, int64_t rows, int heads, int dh, const int32_t* row_seg,
                        uint32_t* kmax2, hipStream_t s) {
  if (rows == 0) return hipSuccess;
  if (dh % 8 || heads <= 0 || heads > 256 || ldk % 8) return hipErrorInvalidValue;
  const int cph = dh / 8;
  const size_t lds = (size_t)32 * heads * (cph + 1) * sizeof(float);
  if (lds > 64 * 1024) return hipErrorInvalidValue;
  hipLaunchKernelGGL(knorm_kernel, dim3((unsigned)((rows + 31) / 32)), dim3(256), lds, s,
                     reinterpret_cast<const uint16_t*>(k), ldk, rows, heads, cph, row_seg, kmax2);
  return hipGetLastError();
}

// Start of an encode: zero the padding columns of the transposed-V buffer (block x = padding run, block y walks the
// rows) and a block of 32-bit words (the key-norm tables).
__global__ __launch_bounds__(256) void attn_prepare_kernel(uint16_t* vt, int64_t ldvt, int rows, const int32_t* pads, int n_pads,
                                                           uint32_t* words, int n_words) {
  if (blockIdx.x == 0 && blockIdx.y == 0)
    for (int i = threadIdx.x; i < n_words; i += 256) words[i] = 0u;
  if ((int)blockIdx.x >= n_pads) return;
  const int c0 = pads[2 * blockIdx.x], c1 = pads[2 * blockIdx.x + 1];
  const int w = c1 - c0;                             // at most 63 columns
  for (int64_t i = (int64_t)blockIdx.y * 256 + threadIdx.x; i < (int64_t)rows * w; i += (int64_t)gridDim.y * 256) {
    const int64_t r = i / w;
    vt[r * ldvt + c0 + (int)(i - r * w)] = 0;
  }
}

hipError_t launch_attn_prepare(void* vt, int64_t ldvt, int rows, const int32_t* pads, int n_pads, uint32_t* words,
                               int n_words, hipStream_t s) {
  if (n_pads < 0 || n_words < 0 || n_pads > 65535 * 256) return hipErrorInvalidValue;
  if (n_pads == 0 && n_words == 0) return hipSuccess;
  const dim3 grid((unsigned)std::max(n_pads, 1), n_pads ? 8 : 1);
  hipLaunchKernelGGL(attn_prepare_kernel, grid, dim3(256), 0, s, reinterpret_cast<uint16_t*>(vt), ldvt, rows, pads, n_pads,
                     words, n_words);
  return hipGetLastError();
}

// zero fill (16-byte stores); n16 = number of 16-byte units
__global__ __launch_bounds__(256) void fill_zero_kernel(uint4* p, size_t n16) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) p[i] = make_uint4(0, 0, 0, 0);
}

hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s) {
  if (bytes == 0) return hipSuccess;
  if (bytes % 16 || reinterpret_cast<uintptr_t>(p) % 16) return hipErrorInvalidValue;
  const size_t n16 = bytes / 16;
  const unsigned grid = (unsigned)std::min<size_t>((n16 + 255) / 256, 256 * 16);
  hipLaunchKernelGGL(fill_zero_kernel, dim3(grid), dim3(256), 0, s, reinterpret_cast<uint4*>(p), n16);
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
