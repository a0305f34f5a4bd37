// Row-wise kernels of one ARMT step: segment packing, RMSNorm with per-layer gain, rotary
// embedding, DPFP feature map with the read denominator, and the delta-rule memory update.
// All of them are bound by HBM traffic: one block (or wave) per row, coalesced row accesses.
#pragma once

#include "common.h"

namespace armt {

// Per-layer pointers that are not GEMM operands (device table, one entry per layer).
struct LayerAux {
  const void* rms1;     // [d] gain of the first norm
  const void* rms2;     // [d] gain of the second norm
  const void* wm_b;     // [d] W_beta
  float* A;             // [d, Phi] associative matrix of the layer (fp32, updated in place)
  float* z;             // [Phi]
  bf16* A16;            // [d, Phi] bf16 shadow of A, operand of the read GEMM (bf16 configs; else null)
};

// ------------------------------------------------------------------------------------------------
// Cell input of a new segment at layer 0: seg_len embedding rows followed by the n_mem memory-token
// embeddings (Eq. 2, "[H, M]"; Algorithm 1, Segment).  grid: (T), block: 256.
template <typename T>
__global__ __launch_bounds__(256) void pack_segment_kernel(const T* __restrict__ x_seg,
                                                           const T* __restrict__ mem_emb, int S, int d,
                                                           float* __restrict__ X0, T* __restrict__ Xb0) {
  const int r = blockIdx.x;
  const T* src = (r < S) ? x_seg + (size_t)r * d : mem_emb + (size_t)(r - S) * d;
  for (int c = threadIdx.x; c < d; c += blockDim.x) {
    const T v = src[c];
    X0[(size_t)r * d + c] = to_f32(v);
    if (Xb0) Xb0[(size_t)r * d + c] = v;
  }
}

// Output of the last layer at the token rows of a segment -> hidden_out.  grid: (S), block: 256.
template <typename T>
__global__ __launch_bounds__(256) void store_hidden_kernel(const float* __restrict__ XL, int d,
                                                           T* __restrict__ out) {
  const size_t r = blockIdx.x;
  for (int c = threadIdx.x; c < d; c += blockDim.x) out[r * d + c] = from_f32<T>(XL[r * d + c]);
}

__global__ void fill_f32_kernel(float* __restrict__ p, size_t n, float v) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}

__global__ void copy_f32_kernel(float* __restrict__ dst, const float* __restrict__ src, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
    dst[i] = src[i];
}

__global__ void f32_to_bf16_kernel(bf16* __restrict__ dst, const float* __restrict__ src, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
    dst[i] = (bf16)src[i];
}

// ------------------------------------------------------------------------------------------------
// RMSNorm with the gain of the cell's own layer (Section 3.3 item 2: per-layer norm weights).
// X: [L+1][T][d] fp32 slots (or Hres [L][T][d]); out: [L][T][d].  grid: (T, g), block: 256.
// With rstd_out the row is written as x * gain only and 1 / rms goes to rstd_out [L][T]: the following GEMM
// applies it as a per-row scale of its result, (x * gain * rstd) W^T = rstd * ((x * gain) W^T).
template <typename T>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const float* __restrict__ X, const LayerAux* __restrict__ aux,
                                                      int first, int which, int Trows, int d, float eps,
                                                      T* __restrict__ out, float* __restrict__ rstd_out) {
  __shared__ float red[17];
  const int l = first + blockIdx.y;
  const size_t row = ((size_t)l * Trows + blockIdx.x) * d;
  const T* gain = (const T*)(which == 0 ? aux[l].rms1 : aux[l].rms2);
  float ss = 0.f;
  for (int c = threadIdx.x; c < d; c += blockDim.x) {
    const float v = X[row + c];
    ss = fmaf(v, v, ss);
  }
  ss = block_sum(ss, red);
  const float rstd = 1.0f / sqrtf(ss / (float)d + eps);
  const float f = rstd_out ? 1.0f : rstd;
  for (int c = threadIdx.x; c < d; c += blockDim.x) out[row + c] = from_f32<T>(X[row + c] * f * to_f32(gain[c]));
  if (rstd_out && threadIdx.x == 0) rstd_out[(size_t)l * Trows + blockIdx.x] = rstd;
}

// 1 / rms of every row from the per-tile sums of squares a GEMM epilogue left behind.
// ssq: [L][T][parts]; rstd: [L][T].  grid: (ceil(T / 256), g), block: 256.
__global__ __launch_bounds__(256) void rstd_kernel(const float* __restrict__ ssq, int first, int Trows, int parts,
                                                   int d, float eps, float* __restrict__ rstd) {
  const int l = first + blockIdx.y, r = blockIdx.x * 256 + threadIdx.x;
  if (r >= Trows) return;
  const float* p = ssq + ((size_t)l * Trows + r) * parts;
  float s = 0.f;
  for (int i = 0; i < parts; ++i) s += p[i];
  rstd[(size_t)l * Trows + r] = 1.0f / sqrtf(s / (float)d + eps);
}

// ------------------------------------------------------------------------------------------------
// cos / sin of p * theta^(-2j/dh), p = 0..T-1, j = 0..dh/2-1, computed in double once per call.
__global__ void rope_table_kernel(float* __restrict__ cs, int Trows, int half, double theta) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= Trows * half) return;
  const int p = i / half, j = i % half;
  const double ang = (double)p * pow(theta, -(double)j / (double)half);
  cs[2 * i] = (float)cos(ang);
  cs[2 * i + 1] = (float)sin(ang);
}

// Rotary embedding of q and k in place, rotate-half pairing (j, j + dh/2), position = row in the cell.
// QKV: [L][T][(H + 2 Hkv) dh].  grid: (T, g), block: 256.
template <typename T>
__global__ __launch_bounds__(256) void rope_kernel(T* __restrict__ QKV, const float* __restrict__ cs, int first,
                                                   int Trows, int n_rot_heads, int dh, int ldq) {
  const int l = first + blockIdx.y, p = blockIdx.x, half = dh >> 1;
  T* row = QKV + ((size_t)l * Trows + p) * ldq;
  for (int i = threadIdx.x; i < n_rot_heads * half; i += blockDim.x) {
    const int h = i / half, j = i % half;
    const float c = cs[2 * (p * half + j)], s = cs[2 * (p * half + j) + 1];
    const float a = to_f32(row[h * dh + j]), b = to_f32(row[h * dh + j + half]);
    row[h * dh + j] = from_f32<T>(a * c - b * s);
    row[h * dh + j + half] = from_f32<T>(b * c + a * s);
  }
}

// ------------------------------------------------------------------------------------------------
// DPFP-nu feature map (the nonlinearity phi of Section 2.1, after Schlag et al. 2021):
// r = [relu(k), relu(-k)], phi[(j-1) 2dm + i] = r[i] r[(i-j) mod 2dm], j = 1..nu.
__device__ __forceinline__ float dpfp_r(const float* k, int dm, int i) {
  return i < dm ? fmaxf(k[i], 0.f) : fmaxf(-k[i - dm], 0.f);
}
__device__ __forceinline__ float dpfp_at(const float* k, int dm, int idx) {
  const int n = 2 * dm, j = idx / n + 1, i = idx % n;
  int i2 = i - j;
  if (i2 < 0) i2 += n;
  return dpfp_r(k, dm, i) * dpfp_r(k, dm, i2);
}

// Read side (Eq. 6): f = phi(W_Q x) for every row of the cell, 1 / (z.f + eps) for the read GEMM's
// epilogue.  Qm: [L][T][dm] fp32; Fphi: [L][T][Phi]; RDen: [L][T].  grid: (T, g), block: 128.
template <typename T>
__global__ __launch_bounds__(128) void dpfp_read_kernel(const float* __restrict__ Qm, const LayerAux* __restrict__ aux,
                                                        int first, int Trows, int dm, int nu, float eps,
                                                        T* __restrict__ Fphi, float* __restrict__ RDen) {
  extern __shared__ float sm[];          // dm floats + 17
  float* k = sm;
  float* red = sm + dm;
  const int l = first + blockIdx.y;
  const size_t r = (size_t)l * Trows + blockIdx.x;
  const int Phi = 2 * nu * dm;
  for (int c = threadIdx.x; c < dm; c += blockDim.x) k[c] = Qm[r * dm + c];
  __syncthreads();
  const float* z = aux[l].z;
  float den = 0.f;
  for (int c = threadIdx.x; c < Phi; c += blockDim.x) {
    const float f = dpfp_at(k, dm, c);
    den = fmaf(f, z[c], den);
    Fphi[r * Phi + c] = from_f32<T>(f);
  }
  den = block_sum(den, red);
  if (threadIdx.x == 0) RDen[r] = 1.0f / (den + eps);
}

// Write side (Eq. 3-4) for the m memory rows of each cell: f_i = phi(k_i), beta_i = sigmoid(W_beta y_i),
// gamma_i = 1 - z.f_i / (|f_i|^2 + eps), and 1 / (z.f_i + eps) (0 for the cells [empty_lo, empty_hi), whose
// memory is still empty: v_bar = 0).
// KV: [L][m][dm + d] fp32 (k then v); Y0 + l * y_stride: the m memory rows [m][d] of layer l's output.
// Fm: [L][m][Phi] fp32; Coef: [L][m][4] = {beta, gamma, 1/den, z.f}.  grid: (m, g), block: 128.
template <typename T>
__global__ __launch_bounds__(128) void memupd_prep_kernel(const float* __restrict__ KV, const T* __restrict__ Y0,
                                                          size_t y_stride, const LayerAux* __restrict__ aux, int first,
                                                          int empty_lo, int empty_hi, int m, int d, int dm, int nu,
                                                          float eps,
                                                          float* __restrict__ Fm, float* __restrict__ Coef) {
  extern __shared__ float sm[];
  float* k = sm;
  float* red = sm + dm;
  const int l = first + blockIdx.y, i = blockIdx.x;
  const int Phi = 2 * nu * dm;
  const size_t mi = (size_t)l * m + i;
  // the kernel is a chain of memory latencies, not of arithmetic: request everything up front (the W_beta dot
  // product in four independent partial sums so that its loads are all in flight together) and reduce the three
  // sums with one pass through LDS
  for (int c = threadIdx.x; c < dm; c += blockDim.x) k[c] = KV[mi * (dm + d) + c];
  const T* y = Y0 + (size_t)l * y_stride + (size_t)i * d;
  const T* wb = (const T*)aux[l].wm_b;
  float b0 = 0.f, b1 = 0.f, b2 = 0.f, b3 = 0.f;
  int c = threadIdx.x;
  const int step = blockDim.x;
  for (; c + 3 * step < d; c += 4 * step) {
    const float y0 = to_f32(y[c]), y1 = to_f32(y[c + step]), y2 = to_f32(y[c + 2 * step]), y3 = to_f32(y[c + 3 * step]);
    const float w0 = to_f32(wb[c]), w1 = to_f32(wb[c + step]), w2 = to_f32(wb[c + 2 * step]), w3 = to_f32(wb[c + 3 * step]);
    b0 = fmaf(y0, w0, b0); b1 = fmaf(y1, w1, b1); b2 = fmaf(y2, w2, b2); b3 = fmaf(y3, w3, b3);
  }
  for (; c < d; c += step) b0 = fmaf(to_f32(y[c]), to_f32(wb[c]), b0);
  float bl = (b0 + b1) + (b2 + b3);
  __syncthreads();
  const float* z = aux[l].z;
  float zf = 0.f, ff = 0.f;
  for (int cc = threadIdx.x; cc < Phi; cc += blockDim.x) {
    const float f = dpfp_at(k, dm, cc);
    zf = fmaf(f, z[cc], zf);
    ff = fmaf(f, f, ff);
    Fm[mi * Phi + cc] = f;
  }
  zf = wave_sum(zf);
  ff = wave_sum(ff);
  bl = wave_sum(bl);
  const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;      // nw <= 5: red holds 17 floats
  if ((threadIdx.x & 63) == 0) { red[3 * w] = zf; red[3 * w + 1] = ff; red[3 * w + 2] = bl; }
  __syncthreads();
  if (threadIdx.x == 0) {
    zf = ff = bl = 0.f;
    for (int j = 0; j < nw; ++j) { zf += red[3 * j]; ff += red[3 * j + 1]; bl += red[3 * j + 2]; }
    Coef[mi * 4 + 0] = 1.0f / (1.0f + expf(-bl));
    Coef[mi * 4 + 1] = 1.0f - zf / (ff + eps);
    Coef[mi * 4 + 2] = (l >= empty_lo && l < empty_hi) ? 0.f : 1.0f / (zf + eps);
    Coef[mi * 4 + 3] = zf;
  }
}

// Delta rule (Eq. 5), one pass over A: row r of A needs only A[r, :], v_i[r] and the shared f_i, so
// each wave owns DR_ROWS rows, keeps them in registers, computes v_bar_i[r] = A[r,:].f_i / den_i for all i
// from the OLD rows, accumulates sum_i beta_i (v_i[r] - v_bar_i[r]) f_i and writes each row back once (plus its
// bf16 shadow).  The f_i pass through LDS in chunks of DR_CHUNK memory tokens, so any n_mem fits.
// The block with blockIdx.x == 0 also updates z += sum_i gamma_i f_i (z is not read here).
// grid: (ceil(d / (4 * DR_ROWS)), g), block: 256 (4 waves).  Phi <= 64 * NPL.
// dynamic LDS: min(m, DR_CHUNK) * (Phi + 4) floats.
constexpr int DR_ROWS = 4, DR_CHUNK = 32;
template <int NPL>
__global__ __launch_bounds__(256) void delta_rule_kernel(const float* __restrict__ KV, const float* __restrict__ Fm,
                                                         const float* __restrict__ Coef,
                                                         const LayerAux* __restrict__ aux, int first, int m, int d,
                                                         int dm, int Phi) {
  extern __shared__ float sm[];          // F: chunk * Phi, then coef: chunk * 4
  const int chunk = min(m, DR_CHUNK);
  float* F = sm;
  float* cf = sm + (size_t)chunk * Phi;
  const int l = first + blockIdx.y;
  const float* Fl = Fm + (size_t)l * m * Phi;
  float* A = aux[l].A;
  bf16* A16 = aux[l].A16;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int r0 = blockIdx.x * (4 * DR_ROWS) + w * DR_ROWS;      // this wave's rows r0 .. r0 + DR_ROWS - 1
  const float* V = KV + (size_t)l * m * (dm + d) + dm;          // v_i[r] = V[i * (dm + d) + r]
  float a[DR_ROWS][NPL], upd[DR_ROWS][NPL];
#pragma unroll
  for (int q = 0; q < DR_ROWS; ++q)
#pragma unroll
    for (int k = 0; k < NPL; ++k) {
      const int c = lane + 64 * k;
      a[q][k] = (r0 + q < d && c < Phi) ? A[(size_t)(r0 + q) * Phi + c] : 0.f;
      upd[q][k] = 0.f;
    }
  float zs[2] = {0.f, 0.f};              // z columns threadIdx.x and threadIdx.x + 256 (Phi <= 512)
  for (int i0 = 0; i0 < m; i0 += chunk) {
    const int n = min(chunk, m - i0);
    __syncthreads();                     // the previous chunk is no longer read
    for (int c = threadIdx.x; c < n * Phi; c += blockDim.x) F[c] = Fl[(size_t)i0 * Phi + c];
    for (int c = threadIdx.x; c < n * 4; c += blockDim.x) cf[c] = Coef[((size_t)l * m + i0) * 4 + c];
    __syncthreads();
#pragma unroll
    for (int q = 0; q < DR_ROWS; ++q) {
      const int r = r0 + q;
      if (r >= d) break;                 // wave-uniform
      for (int i = 0; i < n; ++i) {
        float dot = 0.f;
#pragma unroll
        for (int k = 0; k < NPL; ++k) {
          const int c = lane + 64 * k;
          if (c < Phi) dot = fmaf(a[q][k], F[i * Phi + c], dot);
        }
        dot = wave_sum(dot);
        const float coef = cf[i * 4 + 0] * (V[(size_t)(i0 + i) * (dm + d) + r] - dot * cf[i * 4 + 2]);
#pragma unroll
        for (int k = 0; k < NPL; ++k) {
          const int c = lane + 64 * k;
          if (c < Phi) upd[q][k] = fmaf(coef, F[i * Phi + c], upd[q][k]);
        }
      }
    }
    if (blockIdx.x == 0) {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int c = threadIdx.x + 256 * h;
        if (c < Phi)
          for (int i = 0; i < n; ++i) zs[h] = fmaf(cf[i * 4 + 1], F[i * Phi + c], zs[h]);
      }
    }
  }
#pragma unroll
  for (int q = 0; q < DR_ROWS; ++q)
#pragma unroll
    for (int k = 0; k < NPL; ++k) {
      const int c = lane + 64 * k;
      if (r0 + q < d && c < Phi) {
        const float v = a[q][k] + upd[q][k];
        A[(size_t)(r0 + q) * Phi + c] = v;
        if (A16) A16[(size_t)(r0 + q) * Phi + c] = (bf16)v;
      }
    }
  if (blockIdx.x == 0) {
    float* z = aux[l].z;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int c = threadIdx.x + 256 * h;
      if (c < Phi) z[c] += zs[h];
    }
  }
}

// Lanes < 32 get a + (a of lane + 32), lanes >= 32 get b + (b of lane - 32): the level "lane ^ 32" of a transposing
// butterfly in one swap.  dr_swap_add16: the same for "lane ^ 16" (lanes with bit 4 clear get the sum of a).
__device__ __forceinline__ float dr_swap_add32(float a, float b) {
  typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
  const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(a), __float_as_uint(b), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float dr_swap_add16(float a, float b) {
  typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
  const u32x2 r = __builtin_amdgcn_permlane16_swap(__float_as_uint(a), __float_as_uint(b), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
// value of another lane of the same row of 16 (CTRL 0x128: lane ^ 8 as a rotation by 8, 0x4E: lane ^ 2, 0xB1: lane ^ 1)
template <int CTRL>
__device__ __forceinline__ float dr_dpp(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}

// Fast path of the delta rule for n_mem = 16 and Phi = 64 * NPL: phi(k_i) lives in registers (lane owns columns
// lane + 64 k), the 16 dot products of a row are reduced with a transposing butterfly (17 exchanges instead of
// 16 full wave reductions; afterwards lane L holds the complete dot product for i = (L >> 2) & 15), and the 16
// coefficients are broadcast through scalar registers.  grid: (ceil(d / rows_per_block), g), block: 256.
template <int NPL>
__global__ __launch_bounds__(256) void delta_rule16_kernel(const float* __restrict__ KV, const float* __restrict__ Fm,
                                                           const float* __restrict__ Coef,
                                                           const LayerAux* __restrict__ aux, int first, int d, int dm,
                                                           int rows_per_block) {
  constexpr int M = 16, Phi = 64 * NPL;
  const int l = first + blockIdx.y;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const float* Fl = Fm + (size_t)l * M * Phi;
  const float* cf = Coef + (size_t)l * M * 4;
  float f[M][NPL];
#pragma unroll
  for (int i = 0; i < M; ++i)
#pragma unroll
    for (int k = 0; k < NPL; ++k) f[i][k] = Fl[i * Phi + lane + 64 * k];
  const int mi = (lane >> 2) & 15;                 // the memory token whose dot product this lane ends up with
  const float beta = cf[mi * 4 + 0], rden = cf[mi * 4 + 2];
  const float* Vmi = KV + (size_t)l * M * (dm + d) + (size_t)mi * (dm + d) + dm;
  float* A = aux[l].A;
  bf16* A16 = aux[l].A16;
  const bool b3 = lane & 8, b2 = lane & 4;
  const int r0 = blockIdx.x * rows_per_block, r1 = min(d, r0 + rows_per_block);
  // the wave's next row is requested before the current one is worked on: with one row of 4 * Phi bytes in flight
  // per wave the pass ran at the latency of HBM, not at its rate
  float an[NPL], vn = 0.f;
  if (r0 + w < r1) {
#pragma unroll
    for (int k = 0; k < NPL; ++k) an[k] = A[(size_t)(r0 + w) * Phi + lane + 64 * k];
    vn = Vmi[r0 + w];
  }
  for (int r = r0 + w; r < r1; r += 4) {
    float a[NPL];
#pragma unroll
    for (int k = 0; k < NPL; ++k) a[k] = an[k];
    const float vr = vn;
    if (r + 4 < r1) {
#pragma unroll
      for (int k = 0; k < NPL; ++k) an[k] = A[(size_t)(r + 4) * Phi + lane + 64 * k];
      vn = Vmi[r + 4];
    }
    float p[M];
#pragma unroll
    for (int i = 0; i < M; ++i) {
      float t = 0.f;
#pragma unroll
      for (int k = 0; k < NPL; ++k) t = fmaf(a[k], f[i][k], t);
      p[i] = t;
    }
    // transposing butterfly: the first two levels are lane-half / lane-row swaps (one instruction exchanges what the two
    // sides of a level send each other), the others data-parallel moves inside a row; sums as in the plain exchange
    float q8[8], q4[4], q2[2];
#pragma unroll
    for (int j = 0; j < 8; ++j) q8[j] = dr_swap_add32(p[j], p[j + 8]);
#pragma unroll
    for (int j = 0; j < 4; ++j) q4[j] = dr_swap_add16(q8[j], q8[j + 4]);
#pragma unroll
    for (int j = 0; j < 2; ++j) q2[j] = (b3 ? q4[j + 2] : q4[j]) + dr_dpp<0x128>(b3 ? q4[j] : q4[j + 2]);   // lane ^ 8
    float dot = (b2 ? q2[1] : q2[0]) + __shfl_xor(b2 ? q2[0] : q2[1], 4, kWave);
    dot += dr_dpp<0x4E>(dot);      // lane ^ 2
    dot += dr_dpp<0xB1>(dot);      // lane ^ 1
    const float coef = beta * (vr - dot * rden);      // beta_i (v_i[r] - v_bar_i[r])
    float upd[NPL] = {};
#pragma unroll
    for (int i = 0; i < M; ++i) {
      const float ci = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, coef), i * 4));
#pragma unroll
      for (int k = 0; k < NPL; ++k) upd[k] = fmaf(ci, f[i][k], upd[k]);
    }
#pragma unroll
    for (int k = 0; k < NPL; ++k) {
      const float v = a[k] + upd[k];
      A[(size_t)r * Phi + lane + 64 * k] = v;
      if (A16) A16[(size_t)r * Phi + lane + 64 * k] = (bf16)v;
    }
  }
  if (blockIdx.x == 0 && w == 0) {
    float* z = aux[l].z;
#pragma unroll
    for (int k = 0; k < NPL; ++k) {
      float s = 0.f;
#pragma unroll
      for (int i = 0; i < M; ++i) s = fmaf(cf[i * 4 + 1], f[i][k], s);
      z[lane + 64 * k] += s;
    }
  }
}

// The same for n_mem = 16 * C (the paper's tables use 128 memory tokens): the tokens are taken 16 at a time as above.
// All of them see the OLD row (Eq. 4 is written with A_{s-1}), so a wave keeps the running update of its DRC_ROWS rows
// in registers over the chunks, re-reads the old rows for every chunk (they stay in the L2) and writes each row once
// at the end.  grid: (ceil(d / (4 * DRC_ROWS)), g), block: 256.
constexpr int DRC_ROWS = 8;
template <int NPL>
__global__ __launch_bounds__(256) void delta_rule16c_kernel(const float* __restrict__ KV, const float* __restrict__ Fm,
                                                            const float* __restrict__ Coef,
                                                            const LayerAux* __restrict__ aux, int first, int m, int d,
                                                            int dm) {
  constexpr int Phi = 64 * NPL;
  const int l = first + blockIdx.y;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const float* Fl = Fm + (size_t)l * m * Phi;
  const float* cf = Coef + (size_t)l * m * 4;
  float* A = aux[l].A;
  bf16* A16 = aux[l].A16;
  const int mi = (lane >> 2) & 15;                 // the token of the chunk whose dot product this lane ends up with
  const bool b5 = lane & 32, b4 = lane & 16, b3 = lane & 8, b2 = lane & 4;
  const int r0 = blockIdx.x * (4 * DRC_ROWS) + w;  // this wave's rows: r0 + 4 q
  const bool zwave = blockIdx.x == 0 && w == 0;    // also updates z += sum_i gamma_i f_i
  float upd[DRC_ROWS][NPL], zs[NPL];
#pragma unroll
  for (int k = 0; k < NPL; ++k) {
    zs[k] = 0.f;
#pragma unroll
    for (int q = 0; q < DRC_ROWS; ++q) upd[q][k] = 0.f;
  }
  for (int i0 = 0; i0 < m; i0 += 16) {
    float f[16][NPL];
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
      for (int k = 0; k < NPL; ++k) f[i][k] = Fl[(size_t)(i0 + i) * Phi + lane + 64 * k];
    const float beta = cf[(i0 + mi) * 4 + 0], rden = cf[(i0 + mi) * 4 + 2];
    const float* Vmi = KV + ((size_t)l * m + i0 + mi) * (dm + d) + dm;
#pragma unroll
    for (int q = 0; q < DRC_ROWS; ++q) {
      const int r = r0 + 4 * q;
      if (r >= d) continue;                        // wave-uniform
      float a[NPL];
#pragma unroll
      for (int k = 0; k < NPL; ++k) a[k] = A[(size_t)r * Phi + lane + 64 * k];
      const float vr = Vmi[r];
      float p[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        float t = 0.f;
#pragma unroll
        for (int k = 0; k < NPL; ++k) t = fmaf(a[k], f[i][k], t);
        p[i] = t;
      }
      float q8[8], q4[4], q2[2];
#pragma unroll
      for (int j = 0; j < 8; ++j) q8[j] = (b5 ? p[j + 8] : p[j]) + __shfl_xor(b5 ? p[j] : p[j + 8], 32, kWave);
#pragma unroll
      for (int j = 0; j < 4; ++j) q4[j] = (b4 ? q8[j + 4] : q8[j]) + __shfl_xor(b4 ? q8[j] : q8[j + 4], 16, kWave);
#pragma unroll
      for (int j = 0; j < 2; ++j) q2[j] = (b3 ? q4[j + 2] : q4[j]) + __shfl_xor(b3 ? q4[j] : q4[j + 2], 8, kWave);
      float dot = (b2 ? q2[1] : q2[0]) + __shfl_xor(b2 ? q2[0] : q2[1], 4, kWave);
      dot += __shfl_xor(dot, 2, kWave);
      dot += __shfl_xor(dot, 1, kWave);
      const float coef = beta * (vr - dot * rden);      // beta_i (v_i[r] - v_bar_i[r])
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const float ci = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, coef), i * 4));
#pragma unroll
        for (int k = 0; k < NPL; ++k) upd[q][k] = fmaf(ci, f[i][k], upd[q][k]);
      }
    }
    if (zwave) {
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const float gi = cf[(i0 + i) * 4 + 1];
#pragma unroll
        for (int k = 0; k < NPL; ++k) zs[k] = fmaf(gi, f[i][k], zs[k]);
      }
    }
  }
#pragma unroll
  for (int q = 0; q < DRC_ROWS; ++q) {
    const int r = r0 + 4 * q;
    if (r >= d) continue;
#pragma unroll
    for (int k = 0; k < NPL; ++k) {
      const size_t at = (size_t)r * Phi + lane + 64 * k;
      const float v = A[at] + upd[q][k];
      A[at] = v;
      if (A16) A16[at] = (bf16)v;
    }
  }
  if (zwave) {
    float* z = aux[l].z;
#pragma unroll
    for (int k = 0; k < NPL; ++k) z[lane + 64 * k] += zs[k];
  }
}

}  // namespace armt
