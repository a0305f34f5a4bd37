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

// ---- backward of the token-level ends
// Final RMSNorm as the head's backward needs it: n = h * rstd * gain (the operand of dW = dL^T n) and rstd.
// grid: n_rows, block: 256.
template <typename T>
__global__ __launch_bounds__(256) void final_norm_train_kernel(const T* __restrict__ h, const T* __restrict__ gain, int d,
                                                               float eps, T* __restrict__ n, float* __restrict__ rstd) {
  __shared__ float red[17];
  const size_t row = blockIdx.x;
  const T* x = h + row * d;
  float ss = 0.f;
  for (int c = threadIdx.x; c < d; c += blockDim.x) ss = fmaf(to_f32(x[c]), to_f32(x[c]), ss);
  ss = block_sum(ss, red);
  const float r = 1.0f / sqrtf(ss / (float)d + eps);
  for (int c = threadIdx.x; c < d; c += blockDim.x) n[row * d + c] = from_f32<T>(to_f32(x[c]) * r * to_f32(gain[c]));
  if (threadIdx.x == 0) rstd[row] = r;
}

// dst[i][0:V] = (T)src[i][0:V], dst[i][V:Vp] = 0: the upstream gradient of the logits as a GEMM operand whose
// reduction dimension is padded to the k-tile.  grid: n_rows, block: 256.
template <typename T>
__global__ __launch_bounds__(256) void pad_convert_rows_kernel(const float* __restrict__ src, int V, T* __restrict__ dst, int Vp) {
  const size_t row = blockIdx.x;
  for (int c = threadIdx.x; c < Vp; c += blockDim.x) dst[row * Vp + c] = from_f32<T>(c < V ? src[row * V + c] : 0.f);
}

// With u = dL W (gradient of the normalised row): dh = rstd (g u - h rstd^2 mean(g u h)).  grid: n_rows, block: 256.
template <typename T>
__global__ __launch_bounds__(256) void final_norm_bwd_kernel(const float* __restrict__ u, const T* __restrict__ h,
                                                             const T* __restrict__ gain, const float* __restrict__ rstd, int d,
                                                             float* __restrict__ dh) {
  __shared__ float red[17];
  const size_t row = blockIdx.x;
  const float r = rstd[row];
  float s = 0.f;
  for (int c = threadIdx.x; c < d; c += blockDim.x) s = fmaf(to_f32(gain[c]) * u[row * d + c], to_f32(h[row * d + c]), s);
  s = block_sum(s, red) / (float)d;
  const float k = r * r * s;
  for (int c = threadIdx.x; c < d; c += blockDim.x)
    dh[row * d + c] = r * (to_f32(gain[c]) * u[row * d + c] - to_f32(h[row * d + c]) * k);
}

// Backward of the gather: dtable[ids[i]] += dx[i].  Rows that share an id are added with atomics, so the order of the
// additions (and the last bits of such rows) can differ from run to run.  grid: n_tokens, block: 256.
__global__ __launch_bounds__(256) void embed_bwd_kernel(const float* __restrict__ dx, const int32_t* __restrict__ ids, int vocab,
                                                        int d, float* __restrict__ dtable) {
  const size_t i = blockIdx.x;
  const int id = min(max(ids[i], 0), vocab - 1);
  for (int c = threadIdx.x; c < d; c += blockDim.x) atomicAdd(dtable + (size_t)id * d + c, dx[i * d + c]);
}

}  // namespace armt
