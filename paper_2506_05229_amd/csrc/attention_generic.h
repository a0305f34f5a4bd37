// Causal grouped-query attention over the T rows of each cell, plain fp32 version (any head_dim,
// any T).  Used by fp32 configurations; the bf16 path uses the MFMA kernel in attention_mfma.h.
#pragma once

#include "common.h"

namespace armt {

// QKV: [L][T][(H + 2 Hkv) dh], rows laid out [q heads | k heads | v heads], q and k already rotated.
// Out: [L][T][H dh].  grid: (T, H, g), block: 64 (one wave per query row and head).
template <typename T>
__global__ __launch_bounds__(64) void attention_generic_kernel(const T* __restrict__ QKV, T* __restrict__ Out,
                                                               int first, int Trows, int H, int Hkv, int dh,
                                                               float scale) {
  extern __shared__ float sm[];      // q: dh floats, p: Trows floats
  float* q = sm;
  float* p = sm + dh;
  const int i = blockIdx.x, h = blockIdx.y, l = first + blockIdx.z, lane = threadIdx.x;
  const int ldq = (H + 2 * Hkv) * dh, kvh = h / (H / Hkv);
  const T* base = QKV + (size_t)l * Trows * ldq;
  const T* kbase = base + H * dh + kvh * dh;
  const T* vbase = base + (H + Hkv) * dh + kvh * dh;
  for (int c = lane; c < dh; c += 64) q[c] = to_f32(base[(size_t)i * ldq + h * dh + c]);
  __syncthreads();
  float mx = -INFINITY;
  for (int j = lane; j <= i; j += 64) {
    const T* kr = kbase + (size_t)j * ldq;
    float s = 0.f;
    for (int c = 0; c < dh; ++c) s = fmaf(q[c], to_f32(kr[c]), s);
    s *= scale;
    p[j] = s;
    mx = fmaxf(mx, s);
  }
  mx = wave_max(mx);
  float sum = 0.f;
  for (int j = lane; j <= i; j += 64) {
    const float e = expf(p[j] - mx);
    p[j] = e;
    sum += e;
  }
  sum = wave_sum(sum);
  __syncthreads();
  const float inv = 1.0f / sum;
  for (int c = lane; c < dh; c += 64) {
    float o = 0.f;
    for (int j = 0; j <= i; ++j) o = fmaf(p[j], to_f32(vbase[(size_t)j * ldq + c]), o);
    Out[((size_t)l * Trows + i) * (H * dh) + h * dh + c] = from_f32<T>(o * inv);
  }
}

}  // namespace armt
