// Token-level ends of Algorithm 1: the embedding gather in front of the cells and the final RMSNorm
// behind them (the linear head itself is a grouped GEMM with the 1 / rms row scale in its epilogue).
#pragma once

#include "common.h"

namespace armt {

// out[i][:] = table[clamp(ids[i], 0, vocab - 1)][:], rows of `row_bytes` bytes (a multiple of 16).
// grid: n_tokens, block: 256.
__global__ __launch_bounds__(256) void embed_rows_kernel(const unsigned char* __restrict__ table,
                                                         const int32_t* __restrict__ ids, int vocab, int row_bytes,
                                                         unsigned char* __restrict__ out) {
  const size_t i = blockIdx.x;
  const int id = min(max(ids[i], 0), vocab - 1);
  const uint4* src = (const uint4*)(table + (size_t)id * row_bytes);
  uint4* dst = (uint4*)(out + i * row_bytes);
  for (int c = threadIdx.x; c < row_bytes / 16; c += blockDim.x) dst[c] = src[c];
}

// Final RMSNorm, split the way the GEMM wants it: out = (T)(h * gain) (the un-normalised operand) and
// rstd[row] = 1 / sqrt(mean(h^2) + eps), which the head GEMM applies to its result rows.
// grid: n_rows, block: 256.
template <typename T>
__global__ __launch_bounds__(256) void final_norm_kernel(const T* __restrict__ h, const T* __restrict__ gain, int d,
                                                         float eps, T* __restrict__ out, float* __restrict__ rstd) {
  __shared__ float red[17];
  const size_t row = blockIdx.x;
  const T* x = h + row * d;
  float ss = 0.f;
  for (int c = threadIdx.x; c < d; c += blockDim.x) {
    const float v = to_f32(x[c]);
    ss = fmaf(v, v, ss);
    out[row * d + c] = from_f32<T>(v * to_f32(gain[c]));
  }
  ss = block_sum(ss, red);
  if (threadIdx.x == 0) rstd[row] = 1.0f / sqrtf(ss / (float)d + eps);
}

}  // namespace armt
