// Grouped GEMM, plain fp32 FMA version: any M, N, K, any activation type.
// This is the fp32 path (fp32 configurations need true fp32 products, which the bf16 matrix
// cores cannot give) and the shape-agnostic reference the MFMA kernel is checked against.
#pragma once

#include "common.h"

namespace armt {

constexpr int GG_BM = 64, GG_BN = 64, GG_BK = 16;

template <typename T>
__device__ __forceinline__ const T* weight_row(const GemmGroup& g, const GemmShape& s, int n) {
  if (n < s.n0) return (const T*)g.B0 + (size_t)n * s.ldb;
  n -= s.n0;
  if (n < s.n1) return (const T*)g.B1 + (size_t)n * s.ldb;
  return (const T*)g.B2 + (size_t)(n - s.n1) * s.ldb;
}

// grid: (ceil(N / 64), ceil(M / 64), g); block: 256 threads, each owns a 4 x 4 patch of the tile.
template <typename T>
__global__ __launch_bounds__(256) void gemm_generic_kernel(const GemmGroup* __restrict__ table, int first,
                                                           GemmShape s) {
  const GemmGroup g = table[first + blockIdx.z];
  const bool swiglu = (s.epi == EPI_SWIGLU);
  __shared__ float As[GG_BK][GG_BM + 4];
  __shared__ float Bs[GG_BK][GG_BN + 4];
  __shared__ float Bu[GG_BK][GG_BN + 4];   // second weight of the SwiGLU pair

  const int tid = threadIdx.x;
  const int m0 = blockIdx.y * GG_BM, n0 = blockIdx.x * GG_BN;
  const int lr = tid >> 2, lk = (tid & 3) * 4;   // tile row and first k this thread loads
  const int ty = tid >> 4, tx = tid & 15;

  float acc[4][4] = {}, acu[4][4] = {};
  const T* arow = (m0 + lr < s.M) ? (const T*)g.A + (size_t)(m0 + lr) * s.lda : nullptr;
  const T* brow = nullptr;
  const T* urow = nullptr;
  if (n0 + lr < s.N) {
    if (swiglu) {
      brow = (const T*)g.B0 + (size_t)(n0 + lr) * s.ldb;
      urow = (const T*)g.B1 + (size_t)(n0 + lr) * s.ldb;
    } else {
      brow = weight_row<T>(g, s, n0 + lr);
    }
  }

  for (int k0 = 0; k0 < s.K; k0 += GG_BK) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int k = k0 + lk + i;
      const bool kin = k < s.K;
      As[lk + i][lr] = (arow && kin) ? to_f32(arow[k]) : 0.f;
      Bs[lk + i][lr] = (brow && kin) ? to_f32(brow[k]) : 0.f;
      if (swiglu) Bu[lk + i][lr] = (urow && kin) ? to_f32(urow[k]) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < GG_BK; ++k) {
      float a[4], b[4], u[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[k][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[k][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
      if (swiglu) {
#pragma unroll
        for (int j = 0; j < 4; ++j) u[j] = Bu[k][tx * 4 + j];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) acu[i][j] = fmaf(a[i], u[j], acu[i][j]);
      }
    }
    __syncthreads();
  }

#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m >= s.M) continue;
    const float rs = g.rowscale ? g.rowscale[m] : 1.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n >= s.N) continue;
      const float v = acc[i][j];
      switch (s.epi) {
        case EPI_STORE_ACT: ((T*)g.C)[(size_t)m * s.ldc + n] = from_f32<T>(v * rs); break;
        case EPI_STORE_F32: ((float*)g.C)[(size_t)m * s.ldc + n] = v * rs; break;
        case EPI_RESID_F32: {
          const float r = (g.R ? g.R[(size_t)m * s.ldr + n] : 0.f) + v * rs;
          ((float*)g.C)[(size_t)m * s.ldc + n] = r;
          if (g.C2) ((T*)g.C2)[(size_t)m * s.ldc2 + n] = from_f32<T>(g.gain ? r * to_f32(((const T*)g.gain)[n]) : r);
        } break;
        case EPI_SWIGLU: {
          const float gv = v * rs, sg = gv / (1.f + expf(-gv));
          ((T*)g.C)[(size_t)m * s.ldc + n] = from_f32<T>(sg * (acu[i][j] * rs));
        } break;
      }
    }
  }
}

template <typename T>
inline hipError_t launch_gemm_generic(const GemmGroup* table, int first, int g, const GemmShape& s,
                                      hipStream_t st) {
  if (g <= 0 || s.M <= 0 || s.N <= 0) return hipSuccess;
  dim3 grid((s.N + GG_BN - 1) / GG_BN, (s.M + GG_BM - 1) / GG_BM, g);
  gemm_generic_kernel<T><<<grid, 256, 0, st>>>(table, first, s);
  return hipGetLastError();
}

}  // namespace armt
