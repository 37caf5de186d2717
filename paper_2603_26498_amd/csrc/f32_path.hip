// fp32 kernels: a plain LDS-tiled SGEMM with the same epilogues as the bf16
// GEMM, and a straightforward attention kernel (one thread per query row, keys
// and values staged in LDS, online softmax in fp32).  This path exists for
// fp32 models, where exactness matters and speed does not.
#include "tcmv_internal.h"
#include "device_utils.h"

namespace tcmv {

// ---------------------------------------------------------------------------
// SGEMM: 64x64 tile, 16-deep k slices, 256 threads, 4x4 outputs per thread.
// ---------------------------------------------------------------------------
template <int EPI>
__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmArgs g) {
  constexpr int BM = 64, BN = 64, BK = 16;
  __shared__ float sa[BK][BM + 4];
  __shared__ float sb[BK][BN + 4];
  const float* A = reinterpret_cast<const float*>(g.a);
  const float* W = reinterpret_cast<const float*>(g.w);
  const int64_t m0 = (int64_t)blockIdx.y * BM;
  const int n0 = blockIdx.x * BN;
  const int tid = threadIdx.x;
  const int tx = tid & 15, ty = tid >> 4;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

  for (int k0 = 0; k0 < g.k; k0 += BK) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = tid + i * 256;           // 1024 elements per operand tile
      const int r = e >> 4, kk = e & 15;
      const int64_t gr = m0 + r;
      sa[kk][r] = (gr < g.m && k0 + kk < g.k) ? A[(size_t)gr * g.lda + k0 + kk] : 0.f;
      const int gn = n0 + r;
      sb[kk][r] = (gn < g.n && k0 + kk < g.k) ? W[(size_t)gn * g.k + k0 + kk] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < BK; ++kk) {
      float av[4], bv[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) av[i] = sa[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) bv[j] = sb[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int64_t row = m0 + ty * 4 + i;
    if (row >= g.m) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int col = n0 + tx * 4 + j;
      if (col >= g.n) continue;
      float val = acc[i][j] + (g.bias ? g.bias[col] : 0.f);
      float* C = reinterpret_cast<float*>(g.c);
      if (EPI == EPI_STORE || EPI == EPI_QKV) {
        C[(size_t)row * g.ldc + col] = val;
      } else if (EPI == EPI_GELU) {
        C[(size_t)row * g.ldc + col] = gelu_erf(val);
      } else if (EPI == EPI_RESID) {
        C[(size_t)row * g.ldc + col] += val;
      } else if (EPI == EPI_EMBED) {
        const int pi = g.pos_idx ? g.pos_idx[row] : 0;
        if (g.pos_kind == 1) {
          val += g.pos0[(size_t)pi * g.n + col];
        } else if (g.pos_kind == 2) {
          val += g.pos0[(size_t)(pi & 0xFFFF) * g.n + col] + g.pos1[(size_t)(pi >> 16) * g.n + col];
        }
        const int64_t dst = g.dst_row ? (int64_t)g.dst_row[row] : row;
        C[(size_t)dst * g.ldc + col] = val;
      }
    }
  }
}

hipError_t launch_gemm_f32(const GemmArgs& a, hipStream_t s) {
  if (a.m == 0 || a.n == 0) return hipSuccess;
  if (a.k <= 0) return hipErrorInvalidValue;
  const int64_t gy = (a.m + 63) / 64;
  if (gy > 65535) return hipErrorInvalidValue;
  dim3 grid((unsigned)((a.n + 63) / 64), (unsigned)gy), block(256);
  switch (a.epi) {
    case EPI_STORE: hipLaunchKernelGGL((gemm_f32_kernel<EPI_STORE>), grid, block, 0, s, a); break;
    case EPI_GELU: hipLaunchKernelGGL((gemm_f32_kernel<EPI_GELU>), grid, block, 0, s, a); break;
    case EPI_RESID: hipLaunchKernelGGL((gemm_f32_kernel<EPI_RESID>), grid, block, 0, s, a); break;
    case EPI_EMBED: hipLaunchKernelGGL((gemm_f32_kernel<EPI_EMBED>), grid, block, 0, s, a); break;
    case EPI_QKV: hipLaunchKernelGGL((gemm_f32_kernel<EPI_QKV>), grid, block, 0, s, a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Attention, fp32: a workgroup of 64 threads handles 64 query rows of one
// segment and one head; tiles of 32 keys (K and V rows) are staged in LDS and
// read by all threads at the same address (broadcast).
// ---------------------------------------------------------------------------
template <int DH>
__global__ __launch_bounds__(64) void attn_f32_kernel(AttnArgs a) {
  constexpr int BK = 32;
  __shared__ float sk[BK][DH];
  __shared__ float sv[BK][DH];
  const int head = blockIdx.y;
  const AttnWork w = a.work[blockIdx.x];
  const float* Q = reinterpret_cast<const float*>(a.q);
  const float* K = reinterpret_cast<const float*>(a.k);
  const float* V = reinterpret_cast<const float*>(a.v);
  const int tid = threadIdx.x;
  int qi = tid < w.nq ? tid : w.nq - 1;
  float q[DH], o[DH];
  const float* qp = Q + (size_t)(w.q0 + qi) * a.ldqk + head * DH;
#pragma unroll
  for (int c = 0; c < DH; ++c) { q[c] = qp[c] * a.scale; o[c] = 0.f; }
  float m = -INFINITY, l = 0.f;
  for (int j0 = 0; j0 < w.seg_len; j0 += BK) {
    const int nk = min(BK, w.seg_len - j0);
    __syncthreads();
    for (int e = tid; e < BK * DH; e += 64) {
      const int r = e / DH, c = e - r * DH;
      if (r < nk) {
        const size_t gr = (size_t)(w.seg_start + j0 + r);
        sk[r][c] = K[gr * a.ldqk + head * DH + c];
        sv[r][c] = V[gr * a.ldv + head * DH + c];
      }
    }
    __syncthreads();
    for (int r = 0; r < nk; ++r) {
      float s = 0.f;
#pragma unroll
      for (int c = 0; c < DH; ++c) s = fmaf(q[c], sk[r][c], s);
      const float mn = fmaxf(m, s);
      const float al = expf(m - mn);
      const float pr = expf(s - mn);
      l = l * al + pr;
#pragma unroll
      for (int c = 0; c < DH; ++c) o[c] = fmaf(pr, sv[r][c], o[c] * al);
      m = mn;
    }
  }
  if (tid < w.nq) {
    float* op = reinterpret_cast<float*>(a.out) + (size_t)(w.q0 + tid) * a.ldo + head * DH;
    const float inv = 1.0f / l;
#pragma unroll
    for (int c = 0; c < DH; ++c) op[c] = o[c] * inv;
  }
}

hipError_t launch_attn_f32(const AttnArgs& a, hipStream_t s) {
  if (a.n_work == 0 || a.heads == 0) return hipSuccess;
  dim3 grid((unsigned)a.n_work, (unsigned)a.heads), block(64);
#define TCMV_ATTN32_CASE(D)                                                  \
  case D:                                                                    \
    hipLaunchKernelGGL((attn_f32_kernel<D>), grid, block, 0, s, a);          \
    break;
  switch (a.dh) {
    TCMV_ATTN32_CASE(16) TCMV_ATTN32_CASE(32) TCMV_ATTN32_CASE(48) TCMV_ATTN32_CASE(64)
    TCMV_ATTN32_CASE(80) TCMV_ATTN32_CASE(96) TCMV_ATTN32_CASE(112) TCMV_ATTN32_CASE(128)
    default: return hipErrorInvalidValue;
  }
#undef TCMV_ATTN32_CASE
  return hipGetLastError();
}

// hidden[cls_rows[i]][:] = cls + pos0[0]
__global__ void cls_rows_kernel(float* hidden, const int32_t* cls_rows, int n, const float* cls, const float* pos0,
                                int d) {
  const int i = blockIdx.x;
  float* dst = hidden + (size_t)cls_rows[i] * d;
  for (int c = threadIdx.x; c < d; c += blockDim.x) dst[c] = cls[c] + (pos0 ? pos0[c] : 0.f);
}

hipError_t launch_cls_rows(float* hidden, const int32_t* cls_rows, int n, const float* cls, const float* pos0, int d,
                           hipStream_t s) {
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(cls_rows_kernel, dim3((unsigned)n), dim3(256), 0, s, hidden, cls_rows, n, cls, pos0, d);
  return hipGetLastError();
}

}  // namespace tcmv
