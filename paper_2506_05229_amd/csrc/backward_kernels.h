// Kernels of the ARMT backward pass (the paper's appendix states that a backward pass of the diagonal
// schedule exists; what it computes is the gradient of the forward of Section 2.1, Eq. 2-6).
// Everything that is a contraction goes through the grouped GEMM (with transposed operand copies made
// by transpose_kernel); this file holds the element-wise, row-wise and reduction parts, the
// attention backward and the backward of the delta rule.  Plain fp32 arithmetic throughout.
#pragma once

#include "common.h"
#include "rowwise_kernels.h"

namespace armt {

// dst[c * ldd + r] = src[r * lds + c] for r < R, c < C, per cell (cell strides in elements).
// Columns [R, ldd) of dst are never written: callers keep them zero (they pad the reduction dimension
// of the following GEMM).  grid: (ceil(C / 32), ceil(R / 32), g), block: (32, 8).
template <typename Tin, typename Tout>
__global__ __launch_bounds__(256) void transpose_kernel(const Tin* __restrict__ src, size_t src_cell, int lds,
                                                        Tout* __restrict__ dst, size_t dst_cell, int ldd, int R, int C) {
  __shared__ float tile[32][33];
  const Tin* s = src + (size_t)blockIdx.z * src_cell;
  Tout* o = dst + (size_t)blockIdx.z * dst_cell;
  const int c0 = blockIdx.x * 32, r0 = blockIdx.y * 32;
  for (int j = threadIdx.y; j < 32; j += 8) {
    const int r = r0 + j, c = c0 + threadIdx.x;
    tile[j][threadIdx.x] = (r < R && c < C) ? to_f32(s[(size_t)r * lds + c]) : 0.f;
  }
  __syncthreads();
  for (int j = threadIdx.y; j < 32; j += 8) {
    const int c = c0 + j, r = r0 + threadIdx.x;
    if (c < C && r < R) o[(size_t)c * ldd + r] = from_f32<Tout>(tile[threadIdx.x][j]);
  }
}

// The same for bf16 -> bf16 with 16-byte accesses on both sides: 64 x 64 tiles through LDS (row stride 66 keeps the
// column reads of the second phase on distinct banks).  Needs C, lds, ldd multiples of 8 and 16-byte aligned bases;
// rows [R, ldd) of a tile are written as zeros, which is what the padding columns of dst must hold anyway.
// grid: (ceil(C / 64), ceil(R / 64), g), block: 256.
__global__ __launch_bounds__(256) void transpose_bf16_kernel(const bf16* __restrict__ src, size_t src_cell, int lds,
                                                             bf16* __restrict__ dst, size_t dst_cell, int ldd, int R, int C) {
  __shared__ unsigned int tile[64 * 33];
  const bf16* s = src + (size_t)blockIdx.z * src_cell;
  bf16* o = dst + (size_t)blockIdx.z * dst_cell;
  const int c0 = blockIdx.x * 64, r0 = blockIdx.y * 64;
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const int idx = threadIdx.x + 256 * k, r = idx >> 3, ch = idx & 7;
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (r0 + r < R && c0 + 8 * ch < C) v = *(const uint4*)(s + (size_t)(r0 + r) * lds + c0 + 8 * ch);
    unsigned int* t = tile + r * 33 + 4 * ch;
    t[0] = v.x; t[1] = v.y; t[2] = v.z; t[3] = v.w;
  }
  __syncthreads();
  const unsigned short* th = (const unsigned short*)tile;
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const int idx = threadIdx.x + 256 * k, c = idx >> 3, rch = idx & 7;
    if (c0 + c >= C || r0 + 8 * rch + 7 >= ldd) continue;
    unsigned int w[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const unsigned int lo = th[(8 * rch + 2 * e) * 66 + c], hi = th[(8 * rch + 2 * e + 1) * 66 + c];
      w[e] = lo | (hi << 16);
    }
    *(uint4*)(o + (size_t)(c0 + c) * ldd + r0 + 8 * rch) = make_uint4(w[0], w[1], w[2], w[3]);
  }
}

// Zero `col_bytes` bytes (a multiple of 4) at the start of each of gridDim.x rows that are `row_bytes` apart.
__global__ __launch_bounds__(256) void zero_columns_kernel(char* __restrict__ base, size_t row_bytes, size_t col_bytes) {
  unsigned int* p = (unsigned int*)(base + (size_t)blockIdx.x * row_bytes);
  for (size_t i = threadIdx.x; i < col_bytes / 4; i += blockDim.x) p[i] = 0u;
}

template <typename Tin, typename Tout>
__global__ void convert_kernel(const Tin* __restrict__ src, Tout* __restrict__ dst, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
    dst[i] = from_f32<Tout>(to_f32(src[i]));
}

// RMSNorm that keeps 1 / rms for the backward pass: out = x * rstd * gain.  grid: (T, g), block: 256.
template <typename T>
__global__ __launch_bounds__(256) void rmsnorm_train_kernel(const float* __restrict__ X, size_t x_cell,
                                                            const LayerAux* __restrict__ aux, int first, int which,
                                                            int Trows, int d, float eps, T* __restrict__ out,
                                                            float* __restrict__ rstd_out) {
  __shared__ float red[17];
  const int l = first + blockIdx.y;
  const float* x = X + (size_t)l * x_cell + (size_t)blockIdx.x * d;
  const size_t row = ((size_t)l * Trows + blockIdx.x) * d;
  const T* gain = (const T*)(which == 0 ? aux[l].rms1 : aux[l].rms2);
  float ss = 0.f;
  for (int c = threadIdx.x; c < d; c += blockDim.x) ss = fmaf(x[c], x[c], ss);
  ss = block_sum(ss, red);
  const float rstd = 1.0f / sqrtf(ss / (float)d + eps);
  for (int c = threadIdx.x; c < d; c += blockDim.x) out[row + c] = from_f32<T>(x[c] * rstd * to_f32(gain[c]));
  if (threadIdx.x == 0) rstd_out[(size_t)l * Trows + blockIdx.x] = rstd;
}

// Backward of n = x * rstd * gain for one row: dx = din + rstd * (g dn - x rstd^2 mean(g dn x)).
// dN, X, din, dout are [cells][T][d] with their own cell strides (din / dout may be slots of the gradient
// stream); doutb (optional) is an activation-typed copy of dout.  grid: (T, g), block: 256.
template <typename T>
__global__ __launch_bounds__(256) void rmsnorm_bwd_kernel(const T* __restrict__ dN, const float* __restrict__ X,
                                                          size_t x_cell, const LayerAux* __restrict__ aux, int first,
                                                          int which, const float* __restrict__ rstd_all,
                                                          const float* __restrict__ din, size_t din_cell,
                                                          float* __restrict__ dout, size_t dout_cell,
                                                          T* __restrict__ doutb, int Trows, int d) {
  __shared__ float red[17];
  const int l = first + blockIdx.y, i = blockIdx.x;
  const T* dn = dN + ((size_t)l * Trows + i) * d;
  const float* x = X + (size_t)l * x_cell + (size_t)i * d;
  const float* di = din + (size_t)l * din_cell + (size_t)i * d;
  float* dout_r = dout + (size_t)l * dout_cell + (size_t)i * d;
  const T* gain = (const T*)(which == 0 ? aux[l].rms1 : aux[l].rms2);
  const float rstd = rstd_all[(size_t)l * Trows + i];
  float s = 0.f;
  for (int c = threadIdx.x; c < d; c += blockDim.x) s = fmaf(to_f32(gain[c]) * to_f32(dn[c]), x[c], s);
  s = block_sum(s, red) / (float)d;
  const float k = rstd * rstd * s;
  for (int c = threadIdx.x; c < d; c += blockDim.x) {
    const float v = di[c] + rstd * (to_f32(gain[c]) * to_f32(dn[c]) - x[c] * k);
    dout_r[c] = v;
    if (doutb) doutb[((size_t)l * Trows + i) * d + c] = from_f32<T>(v);
  }
}

// Column sums over the T rows of a cell, in two deterministic stages.  Stage 1: the rows are cut into gridDim.z
// chunks; a thread owns a column and adds its chunk's rows in order:
//   part[cell][chunk][c] = sum_{i in chunk} w[i] a[i, c] (b ? b[i, c] : 1).
// Stage 2 (colsum_finish_kernel) adds the chunks in order into the destination.
// a: [cells][T][C] activation type; b: fp32 with its own cell stride (or null); w: [cells][T].
// grid: (ceil(C / 256), g, chunks), block: 256.
constexpr int CS_CHUNKS = 16;
template <typename T>
__global__ __launch_bounds__(256) void colsum_partial_kernel(const T* __restrict__ a, const float* __restrict__ b, size_t b_cell,
                                                             const float* __restrict__ w, float* __restrict__ part, int first,
                                                             int Trows, int C) {
  const int l = first + blockIdx.y, c = blockIdx.x * 256 + threadIdx.x;
  if (c >= C) return;
  const int per = (Trows + gridDim.z - 1) / gridDim.z;
  const int i0 = blockIdx.z * per, i1 = min(Trows, i0 + per);
  const T* ap = a + (size_t)l * Trows * C;
  const float* bp = b ? b + (size_t)l * b_cell : nullptr;
  const float* wp = w + (size_t)l * Trows;
  float s = 0.f;
  for (int i = i0; i < i1; ++i) {
    const float v = to_f32(ap[(size_t)i * C + c]) * (bp ? bp[(size_t)i * C + c] : 1.f);
    s = fmaf(v, wp[i], s);
  }
  part[((size_t)l * gridDim.z + blockIdx.z) * C + c] = s;
}

// dst[c] += sum over nb consecutive cells and their chunks of part[cell][chunk][c]; dst = dst_tab[first cell] if a pointer
// table is given (the nb cells of a batch that share a layer's gradient), else dst_base + cell * C (nb = 1).
// grid: (ceil(C / 256), cells / nb), block: 256.
__global__ __launch_bounds__(256) void colsum_finish_kernel(const float* __restrict__ part, int chunks, float* const* __restrict__ dst_tab,
                                                            float* __restrict__ dst_base, int first, int C, int nb) {
  const int l = first + blockIdx.y * nb, c = blockIdx.x * 256 + threadIdx.x;      // destination of cells l .. l + nb - 1
  if (c >= C) return;
  float s = 0.f;
  for (int b = 0; b < nb; ++b)
    for (int k = 0; k < chunks; ++k) s += part[((size_t)(l + b) * chunks + k) * C + c];
  float* dst = dst_tab ? dst_tab[l] : dst_base + (size_t)l * C;
  dst[c] += s;
}

// u = silu(gate) * up from the stored [gate | up] rows.  GU: [cells][T][2F]; U: [cells][T][F].
template <typename T>
__global__ void swiglu_kernel(const T* __restrict__ GU, T* __restrict__ U, size_t rows, int F) {
  const size_t n = rows * F;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
    const size_t r = i / F, c = i % F;
    const float g = to_f32(GU[r * 2 * F + c]), u = to_f32(GU[r * 2 * F + F + c]);
    U[i] = from_f32<T>(g / (1.f + expf(-g)) * u);
  }
}

// In place on [gate | up]: dgate = dU up sig(g) (1 + g (1 - sig(g))), dup = dU silu(g).
template <typename T>
__global__ void swiglu_bwd_kernel(T* __restrict__ GU, const T* __restrict__ dU, size_t rows, int F) {
  const size_t n = rows * F;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
    const size_t r = i / F, c = i % F;
    const float g = to_f32(GU[r * 2 * F + c]), u = to_f32(GU[r * 2 * F + F + c]), du = to_f32(dU[i]);
    const float sg = 1.f / (1.f + expf(-g));
    GU[r * 2 * F + c] = from_f32<T>(du * u * sg * (1.f + g * (1.f - sg)));
    GU[r * 2 * F + F + c] = from_f32<T>(du * g * sg);
  }
}

// bf16 versions of the two SwiGLU kernels that also leave the transposed copy the weight-gradient GEMMs need, written
// straight into a layer's window rows (row stride ldd; the cell z of the launch belongs to layer z / batch and puts its
// T columns at column offset (z % batch) * Tp): 64 x 64 tiles, 16-byte accesses, the transposed half through LDS as in
// transpose_bf16_kernel (tile rows past T are written as zeros: the padding of the reduction dimension).
// Forward (BWD = false): u = silu(gate) up; U^T -> dst rows [c]; U itself only for rows >= first_row (the memory rows, all
//   the recomputed down projection reads).  GU: [cells][T][2F], U: [cells][T][F].
// Backward (BWD = true): [gate | up] <- [dgate | dup] in place from dU, and the same values transposed -> dst rows [c] (dgate)
//   and [F + c] (dup).
// grid: (F / 64, ceil(T / 64), cells), block: 256.  F a multiple of 64.
template <bool BWD>
__global__ __launch_bounds__(256) void swiglu_tiles_kernel(bf16* __restrict__ GU, bf16* __restrict__ U /* BWD: dU (read) */,
                                                           int Trows, int F, int first_row, bf16* __restrict__ dst,
                                                           size_t dst_layer, int ldd, int batch, int Tp) {
  __shared__ unsigned int tg[64 * 33], tu[64 * 33];
  const int z = blockIdx.z, c0 = blockIdx.x * 64, r0 = blockIdx.y * 64;
  bf16* gu = GU + (size_t)z * Trows * 2 * F;
  bf16* uu = U + (size_t)z * Trows * F;
  bf16* o = dst + (size_t)(z / batch) * dst_layer + (size_t)(z % batch) * Tp;
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const int idx = threadIdx.x + 256 * k, r = idx >> 3, ch = idx & 7, row = r0 + r, col = c0 + 8 * ch;
    bf16x8 a = {0, 0, 0, 0, 0, 0, 0, 0}, b = a;           // what goes to the transposed copy
    if (row < Trows) {
      const bf16x8 g = *(const bf16x8*)(gu + (size_t)row * 2 * F + col), up = *(const bf16x8*)(gu + (size_t)row * 2 * F + F + col);
      if (BWD) {
        const bf16x8 du = *(const bf16x8*)(uu + (size_t)row * F + col);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float gf = (float)g[e], sg = 1.f / (1.f + expf(-gf)), d = (float)du[e];
          a[e] = (bf16)(d * (float)up[e] * sg * (1.f + gf * (1.f - sg)));
          b[e] = (bf16)(d * gf * sg);
        }
        *(bf16x8*)(gu + (size_t)row * 2 * F + col) = a;
        *(bf16x8*)(gu + (size_t)row * 2 * F + F + col) = b;
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float gf = (float)g[e];
          a[e] = (bf16)(gf / (1.f + expf(-gf)) * (float)up[e]);
        }
        if (row >= first_row) *(bf16x8*)(uu + (size_t)row * F + col) = a;
      }
    }
    const uint4 av = __builtin_bit_cast(uint4, a), bv = __builtin_bit_cast(uint4, b);
    unsigned int* t = tg + r * 33 + 4 * ch;
    t[0] = av.x; t[1] = av.y; t[2] = av.z; t[3] = av.w;
    if (BWD) {
      unsigned int* t2 = tu + r * 33 + 4 * ch;
      t2[0] = bv.x; t2[1] = bv.y; t2[2] = bv.z; t2[3] = bv.w;
    }
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const int idx = threadIdx.x + 256 * k, c = idx >> 3, rch = idx & 7;
    if (r0 + 8 * rch + 7 >= Tp) continue;                 // Tp is a multiple of 64: never true for a started tile row block
#pragma unroll
    for (int h = 0; h < (BWD ? 2 : 1); ++h) {
      const unsigned short* th = (const unsigned short*)(h ? tu : tg);
      unsigned int w[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const unsigned int lo = th[(8 * rch + 2 * e) * 66 + c], hi = th[(8 * rch + 2 * e + 1) * 66 + c];
        w[e] = lo | (hi << 16);
      }
      *(uint4*)(o + (size_t)(h * F + c0 + c) * ldd + r0 + 8 * rch) = make_uint4(w[0], w[1], w[2], w[3]);
    }
  }
}

// Backward of the rotary embedding: rotate the gradient of q and k by the opposite angle, in place.
template <typename T>
__global__ __launch_bounds__(256) void rope_bwd_kernel(T* __restrict__ dQKV, const float* __restrict__ cs, int first,
                                                       int Trows, int n_rot_heads, int dh, int ldq) {
  const int l = first + blockIdx.y, p = blockIdx.x, half = dh >> 1;
  T* row = dQKV + ((size_t)l * Trows + p) * ldq;
  for (int i = threadIdx.x; i < n_rot_heads * half; i += blockDim.x) {
    const int h = i / half, j = i % half;
    const float c = cs[2 * (p * half + j)], s = cs[2 * (p * half + j) + 1];
    const float a = to_f32(row[h * dh + j]), b = to_f32(row[h * dh + j + half]);
    row[h * dh + j] = from_f32<T>(a * c + b * s);
    row[h * dh + j + half] = from_f32<T>(b * c - a * s);
  }
}

// ------------------------------------------------------------------------------------------------
// Attention backward, plain fp32 version, two passes.
// Pass 1, one wave per (query row i, head h): recomputes the softmax row, stores its log-sum-exp and
// D_i = dO_i . O_i, and writes dq_i = scale * sum_j p_ij (dO_i . v_j - D_i) k_j.
// QKV / dQKV: [cells][T][(H + 2 Hkv) dh]; O, dO: [cells][T][H dh]; LSE, Dv: [cells][H][T].
// grid: (T, H, g), block: 64; LDS: (2 dh + T) floats.
template <typename T>
__global__ __launch_bounds__(64) void attention_bwd_q_kernel(const T* __restrict__ QKV, const T* __restrict__ O,
                                                             const T* __restrict__ dO, T* __restrict__ dQKV,
                                                             float* __restrict__ LSE, float* __restrict__ Dv, int first,
                                                             int Trows, int H, int Hkv, int dh, float scale) {
  extern __shared__ float sm[];
  float* q = sm;
  float* go = sm + dh;
  float* p = sm + 2 * dh;
  const int i = blockIdx.x, h = blockIdx.y, l = first + blockIdx.z, lane = threadIdx.x;
  const int ldq = (H + 2 * Hkv) * dh, kvh = h / (H / Hkv);
  const T* base = QKV + (size_t)l * Trows * ldq;
  const T* kbase = base + H * dh + kvh * dh;
  const T* vbase = base + (H + Hkv) * dh + kvh * dh;
  const size_t orow = ((size_t)l * Trows + i) * (H * dh) + h * dh;
  float dsum = 0.f;
  for (int c = lane; c < dh; c += 64) {
    q[c] = to_f32(base[(size_t)i * ldq + h * dh + c]);
    go[c] = to_f32(dO[orow + c]);
    dsum = fmaf(go[c], to_f32(O[orow + c]), dsum);
  }
  dsum = wave_sum(dsum);
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
  for (int j = lane; j <= i; j += 64) sum += expf(p[j] - mx);
  sum = wave_sum(sum);
  const float lse = mx + logf(sum);
  for (int j = lane; j <= i; j += 64) {
    const T* vr = vbase + (size_t)j * ldq;
    float dp = 0.f;
    for (int c = 0; c < dh; ++c) dp = fmaf(go[c], to_f32(vr[c]), dp);
    p[j] = expf(p[j] - lse) * (dp - dsum) * scale;      // dS_ij
  }
  __syncthreads();
  for (int c = lane; c < dh; c += 64) {
    float a = 0.f;
    for (int j = 0; j <= i; ++j) a = fmaf(p[j], to_f32(kbase[(size_t)j * ldq + c]), a);
    dQKV[((size_t)l * Trows + i) * ldq + h * dh + c] = from_f32<T>(a);
  }
  if (lane == 0) {
    LSE[((size_t)l * H + h) * Trows + i] = lse;
    Dv[((size_t)l * H + h) * Trows + i] = dsum;
  }
}

// Pass 2, one wave per (key row j, KV head): dk_j = scale * sum_{h in group} sum_{i >= j} p_ij (dO_i . v_j - D_i) q_i,
// dv_j = sum p_ij dO_i, with p_ij = exp(scale q_i . k_j - LSE_i).  Query rows are taken 64 at a time: every lane
// computes p and dS for one i, then the lanes turn to the head-dimension columns and add the 64 contributions.
// grid: (T, Hkv, g), block: 64; LDS: (2 dh + 128) floats.
template <typename T>
__global__ __launch_bounds__(64) void attention_bwd_kv_kernel(const T* __restrict__ QKV, const T* __restrict__ dO,
                                                              T* __restrict__ dQKV, const float* __restrict__ LSE,
                                                              const float* __restrict__ Dv, int first, int Trows, int H,
                                                              int Hkv, int dh, float scale) {
  extern __shared__ float sm[];
  float* kj = sm;
  float* vj = sm + dh;
  float* pp = sm + 2 * dh;       // p_ij of the current 64 query rows
  float* ds = pp + 64;           // dS_ij
  const int j = blockIdx.x, kvh = blockIdx.y, l = first + blockIdx.z, lane = threadIdx.x;
  const int ldq = (H + 2 * Hkv) * dh, rep = H / Hkv;
  const T* base = QKV + (size_t)l * Trows * ldq;
  for (int c = lane; c < dh; c += 64) {
    kj[c] = to_f32(base[(size_t)j * ldq + (H + kvh) * dh + c]);
    vj[c] = to_f32(base[(size_t)j * ldq + (H + Hkv + kvh) * dh + c]);
  }
  __syncthreads();
  float dk[2] = {0.f, 0.f}, dv[2] = {0.f, 0.f};          // columns lane and lane + 64 (dh <= 128)
  for (int h = kvh * rep; h < (kvh + 1) * rep; ++h) {
    const float* lse = LSE + ((size_t)l * H + h) * Trows;
    const float* dvec = Dv + ((size_t)l * H + h) * Trows;
    for (int i0 = j; i0 < Trows; i0 += 64) {
      const int i = i0 + lane;
      float pv = 0.f, dsv = 0.f;
      if (i < Trows) {
        const T* qr = base + (size_t)i * ldq + h * dh;
        const T* gr = dO + ((size_t)l * Trows + i) * (H * dh) + h * dh;
        float s = 0.f, dp = 0.f;
        for (int c = 0; c < dh; ++c) {
          s = fmaf(to_f32(qr[c]), kj[c], s);
          dp = fmaf(to_f32(gr[c]), vj[c], dp);
        }
        pv = expf(s * scale - lse[i]);
        dsv = pv * (dp - dvec[i]) * scale;
      }
      __syncthreads();
      pp[lane] = pv;
      ds[lane] = dsv;
      __syncthreads();
      const int n = min(64, Trows - i0);
      for (int t = 0; t < n; ++t) {
        const T* qr = base + (size_t)(i0 + t) * ldq + h * dh;
        const T* gr = dO + ((size_t)l * Trows + i0 + t) * (H * dh) + h * dh;
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          const int c = lane + 64 * e;
          if (c < dh) {
            dk[e] = fmaf(ds[t], to_f32(qr[c]), dk[e]);
            dv[e] = fmaf(pp[t], to_f32(gr[c]), dv[e]);
          }
        }
      }
    }
  }
#pragma unroll
  for (int e = 0; e < 2; ++e) {
    const int c = lane + 64 * e;
    if (c < dh) {
      dQKV[((size_t)l * Trows + j) * ldq + (H + kvh) * dh + c] = from_f32<T>(dk[e]);
      dQKV[((size_t)l * Trows + j) * ldq + (H + Hkv + kvh) * dh + c] = from_f32<T>(dv[e]);
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Backward of the DPFP feature map for one vector: k[dm] (LDS), df[Phi] (LDS) -> dk[c] for c = threadIdx.x ...
// r = [relu(k), relu(-k)], phi[(j-1) n + i] = r[i] r[(i - j) mod n]: r[i] appears as the first factor of entry
// (j, i) and as the second factor of entry (j, (i + j) mod n).
__device__ __forceinline__ float dpfp_dr(const float* k, const float* df, int dm, int nu, int i) {
  const int n = 2 * dm;
  float s = 0.f;
  for (int j = 1; j <= nu; ++j) {
    int a = i - j; if (a < 0) a += n;
    int b = i + j; if (b >= n) b -= n;
    s = fmaf(df[(j - 1) * n + i], dpfp_r(k, dm, a), s);
    s = fmaf(df[(j - 1) * n + b], dpfp_r(k, dm, b), s);
  }
  return s;
}
__device__ __forceinline__ float dpfp_dk(const float* k, const float* df, int dm, int nu, int c) {
  if (k[c] > 0.f) return dpfp_dr(k, df, dm, nu, c);
  if (k[c] < 0.f) return -dpfp_dr(k, df, dm, nu, c + dm);
  return 0.f;
}

// Read backward, row part 1 (Eq. 6: x1 = x + num / den): from dx1 (gradient of the read's output), x1 and x,
// dnum = dx1 / den (activation type, operand of the following GEMMs) and dden = -(dnum . (x1 - x)).
// grid: (T, g), block: 256.
template <typename T>
__global__ __launch_bounds__(256) void read_bwd_rows_kernel(const float* __restrict__ dX1, size_t dx_cell,
                                                            const float* __restrict__ X1, size_t x1_cell,
                                                            const float* __restrict__ Xin, size_t xin_cell,
                                                            const float* __restrict__ RDen, int first, int Trows, int d,
                                                            T* __restrict__ DNum, float* __restrict__ DDen) {
  __shared__ float red[17];
  const int l = first + blockIdx.y, i = blockIdx.x;
  const float* g = dX1 + (size_t)l * dx_cell + (size_t)i * d;
  const float* x1 = X1 + (size_t)l * x1_cell + (size_t)i * d;
  const float* x0 = Xin + (size_t)l * xin_cell + (size_t)i * d;
  const float rden = RDen[(size_t)l * Trows + i];
  // dden is formed from the ROUNDED dnum: df = A^T dnum + dden z removes from A^T dnum its component along the
  // read direction, and the two terms only cancel as they should if both see the same dnum
  float s = 0.f;
  for (int c = threadIdx.x; c < d; c += blockDim.x) {
    const T dn = from_f32<T>(g[c] * rden);
    s = fmaf(to_f32(dn), x1[c] - x0[c], s);
    DNum[((size_t)l * Trows + i) * d + c] = dn;
  }
  s = block_sum(s, red);
  if (threadIdx.x == 0) DDen[(size_t)l * Trows + i] = -s;
}

// Read backward, row part 2: df = dnum A (from the GEMM, fp32) + dden z, pushed through the feature map:
// dq = dphi(q)^T df, written in the activation type with row stride ldq (padding columns stay zero).
// grid: (T, g), block: 128; LDS: (dm + Phi) floats.
template <typename T>
__global__ __launch_bounds__(128) void read_bwd_dpfp_kernel(const float* __restrict__ Qm, const float* __restrict__ DF,
                                                            const float* __restrict__ DDen, const LayerAux* __restrict__ aux,
                                                            int first, int Trows, int dm, int nu, T* __restrict__ DQ, int ldq) {
  extern __shared__ float sm[];
  float* k = sm;
  float* df = sm + dm;
  const int l = first + blockIdx.y, Phi = 2 * nu * dm;
  const size_t r = (size_t)l * Trows + blockIdx.x;
  const float* z = aux[l].z;
  const float dden = DDen[r];
  for (int c = threadIdx.x; c < dm; c += blockDim.x) k[c] = Qm[r * dm + c];
  for (int c = threadIdx.x; c < Phi; c += blockDim.x) df[c] = fmaf(dden, z[c], DF[r * Phi + c]);
  __syncthreads();
  for (int c = threadIdx.x; c < dm; c += blockDim.x) DQ[r * ldq + c] = from_f32<T>(dpfp_dk(k, df, dm, nu, c));
}

// ------------------------------------------------------------------------------------------------
// Backward of the delta rule (Eq. 3-5), part 1: everything that is local to a row r of A.
// With G = dA' (gradient of the updated matrix), P_i[r] = G[r,:] . f_i, v_bar_i[r] = A[r,:] . f_i / den_i:
//   dv_i[r]      = beta_i P_i[r]                                   -> DV [cells][m][d]
//   w_i[r]       = -beta_i P_i[r] / den_i    (gradient of v_bar_i[r], divided by den_i)
//   G[r,:]      += sum_i w_i[r] f_i          (in place: becomes the gradient of the OLD matrix)
//   partial sums over the block's rows:  dbeta_i += (v_i[r] - v_bar_i[r]) P_i[r],
//        dden_i += beta_i v_bar_i[r] P_i[r] / den_i,   df_i[:] += beta_i (v_i[r] - v_bar_i[r]) G_old[r,:] + w_i[r] A[r,:]
// Part[cells][blocks][m][Phi + 2] holds the partial df_i, dbeta_i, dden_i of every block.
// Coef as written by memupd_prep_kernel ({beta, gamma, 1/den (0 = memory empty), z.f}).
// The memory tokens are taken in chunks of UB_M (their partial feature gradients live in registers); a wave re-reads
// its rows of A and G for every chunk, carries the running update of G between chunks in Upd and writes G with the last.
// grid: (ceil(d / UB_ROWS), g), block: 256; Phi <= 64 * NPL; LDS: UB_M * (2 Phi + 2) floats.
constexpr int UB_ROWS = 32, UB_M = 16;
template <int NPL>
__global__ __launch_bounds__(256) void update_bwd_rows_kernel(const float* __restrict__ KV, const float* __restrict__ Fm,
                                                              const float* __restrict__ Coef,
                                                              const float* __restrict__ Aold, float* __restrict__ DA,
                                                              float* __restrict__ Upd, float* __restrict__ DV,
                                                              float* __restrict__ Part, int first, int m, int d, int dm, int Phi) {
  extern __shared__ float sm[];
  float* F = sm;                               // [UB_M][Phi]: the f_i of the current chunk of memory tokens
  float* acc = sm + (size_t)UB_M * Phi;        // [UB_M][Phi + 2]
  const int l = first + blockIdx.y, lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const float* Fl = Fm + (size_t)l * m * Phi;
  const float* cf = Coef + (size_t)l * m * 4;
  const float* A = Aold + (size_t)l * d * Phi;
  float* G = DA + (size_t)l * d * Phi;
  float* U = Upd + (size_t)l * d * Phi;        // sum_i w_i[r] f_i over the chunks so far (used only if m > UB_M)
  const float* V = KV + (size_t)l * m * (dm + d) + dm;
  const int r0 = blockIdx.x * UB_ROWS, r1 = min(d, r0 + UB_ROWS);
  const int stride = Phi + 2;
  float* out = Part + ((size_t)l * gridDim.x + blockIdx.x) * m * stride;

  for (int i0 = 0; i0 < m; i0 += UB_M) {       // memory tokens in chunks of UB_M; every chunk needs the ORIGINAL G
    const int n = min(UB_M, m - i0);
    __syncthreads();                           // the previous chunk's F and acc are no longer read
    for (int c = threadIdx.x; c < n * Phi; c += blockDim.x) F[c] = Fl[(size_t)i0 * Phi + c];
    __syncthreads();
    float dfp[UB_M][NPL], db[UB_M], dd[UB_M];
#pragma unroll
    for (int i = 0; i < UB_M; ++i) {
      db[i] = dd[i] = 0.f;
#pragma unroll
      for (int k = 0; k < NPL; ++k) dfp[i][k] = 0.f;
    }
    for (int r = r0 + w; r < r1; r += 4) {
      float a[NPL], g[NPL], upd[NPL];
#pragma unroll
      for (int k = 0; k < NPL; ++k) {
        const int c = lane + 64 * k;
        a[k] = c < Phi ? A[(size_t)r * Phi + c] : 0.f;
        g[k] = c < Phi ? G[(size_t)r * Phi + c] : 0.f;
        upd[k] = (i0 > 0 && c < Phi) ? U[(size_t)r * Phi + c] : 0.f;
      }
#pragma unroll
      for (int i = 0; i < UB_M; ++i) {
        if (i >= n) continue;                  // uniform; `continue` keeps the loop unrollable (dfp[][] stays in registers)
        float pa = 0.f, pg = 0.f;
#pragma unroll
        for (int k = 0; k < NPL; ++k) {
          const int c = lane + 64 * k;
          const float f = c < Phi ? F[i * Phi + c] : 0.f;
          pa = fmaf(a[k], f, pa);
          pg = fmaf(g[k], f, pg);
        }
        pa = wave_sum(pa);
        pg = wave_sum(pg);
        const int it = i0 + i;
        const float beta = cf[it * 4 + 0], rden = cf[it * 4 + 2];
        const float vbar = pa * rden, e = V[(size_t)it * (dm + d) + r] - vbar;
        const float wi = -beta * pg * rden;
        if (lane == 0) DV[((size_t)l * m + it) * d + r] = beta * pg;
        db[i] = fmaf(e, pg, db[i]);
        dd[i] = fmaf(beta * vbar * rden, pg, dd[i]);
#pragma unroll
        for (int k = 0; k < NPL; ++k) {
          const int c = lane + 64 * k;
          const float f = c < Phi ? F[i * Phi + c] : 0.f;
          dfp[i][k] = fmaf(beta * e, g[k], fmaf(wi, a[k], dfp[i][k]));
          upd[k] = fmaf(wi, f, upd[k]);
        }
      }
      const bool last = i0 + UB_M >= m;
#pragma unroll
      for (int k = 0; k < NPL; ++k) {
        const int c = lane + 64 * k;
        if (c < Phi) {
          if (last) G[(size_t)r * Phi + c] = g[k] + upd[k];      // rows are private to a wave: nobody reads this G again
          else U[(size_t)r * Phi + c] = upd[k];
        }
      }
    }
    // the four waves' partial sums -> one partial per block (the waves add into one LDS image in turn)
    for (int ww = 0; ww < 4; ++ww) {
      if (w == ww) {
#pragma unroll
        for (int i = 0; i < UB_M; ++i) {
          if (i >= n) continue;
#pragma unroll
          for (int k = 0; k < NPL; ++k) {
            const int c = lane + 64 * k;
            if (c < Phi) acc[(size_t)i * stride + c] = (ww ? acc[(size_t)i * stride + c] : 0.f) + dfp[i][k];
          }
          if (lane == 0) {
            acc[(size_t)i * stride + Phi] = (ww ? acc[(size_t)i * stride + Phi] : 0.f) + db[i];
            acc[(size_t)i * stride + Phi + 1] = (ww ? acc[(size_t)i * stride + Phi + 1] : 0.f) + dd[i];
          }
        }
      }
      __syncthreads();
    }
    for (int c = threadIdx.x; c < n * stride; c += blockDim.x) out[(size_t)i0 * stride + c] = acc[c];
  }
}

// Part 2, one block per memory token i: sums the partials, adds the terms that come through z and gamma, pushes
// df_i through the feature map and writes the operands of the projection gradients:
//   dgamma_i = dz' . f_i,  dzf_i = dden_i - dgamma_i / (|f_i|^2 + eps),  dn_i = dgamma_i zf_i / (|f_i|^2 + eps)^2
//   df_i = partial + gamma_i dz' + 2 dn_i f_i + dzf_i z
//   DKV[i] = [dk_i | dv_i] (activation type, row stride ldkv, padding stays zero), DB[i] = dbeta_i beta_i (1 - beta_i),
//   DZF[i] = dzf_i (for update_bwd_z_kernel).
// grid: (m, g), block: 128; LDS: (dm + Phi + 17) floats.
template <typename T>
__global__ __launch_bounds__(128) void update_bwd_tokens_kernel(const float* __restrict__ KV, const float* __restrict__ Fm,
                                                                const float* __restrict__ Coef, const float* __restrict__ Part,
                                                                int nblocks, const float* __restrict__ DV,
                                                                const float* __restrict__ Zold, const float* __restrict__ DZ,
                                                                int first, int m, int d, int dm, int nu, float eps,
                                                                T* __restrict__ DKV, int ldkv, float* __restrict__ DB,
                                                                float* __restrict__ DZF) {
  extern __shared__ float sm[];
  float* k = sm;
  float* df = sm + dm;
  float* red = df + 2 * nu * dm;
  const int l = first + blockIdx.y, i = blockIdx.x, Phi = 2 * nu * dm, stride = Phi + 2;
  const size_t mi = (size_t)l * m + i;
  const float* f = Fm + mi * Phi;
  const float* z = Zold + (size_t)l * Phi;
  const float* dz = DZ + (size_t)l * Phi;
  const float* part = Part + (size_t)l * nblocks * m * stride + (size_t)i * stride;
  for (int c = threadIdx.x; c < dm; c += blockDim.x) k[c] = KV[mi * (dm + d) + c];
  float dg = 0.f, ff = 0.f;
  for (int c = threadIdx.x; c < Phi; c += blockDim.x) {
    float s = 0.f;
    for (int b = 0; b < nblocks; ++b) s += part[(size_t)b * m * stride + c];
    df[c] = s;
    dg = fmaf(dz[c], f[c], dg);
    ff = fmaf(f[c], f[c], ff);
  }
  dg = block_sum(dg, red);
  ff = block_sum(ff, red);
  float dbeta = 0.f, dden = 0.f;
  if (threadIdx.x == 0)
    for (int b = 0; b < nblocks; ++b) {
      dbeta += part[(size_t)b * m * stride + Phi];
      dden += part[(size_t)b * m * stride + Phi + 1];
    }
  const float beta = Coef[mi * 4 + 0], gamma = Coef[mi * 4 + 1], zf = Coef[mi * 4 + 3];
  const float inv = 1.0f / (ff + eps);
  __shared__ float dzf_s;
  if (threadIdx.x == 0) {
    dzf_s = dden - dg * inv;
    DZF[mi] = dzf_s;
    DB[mi] = dbeta * beta * (1.f - beta);
  }
  __syncthreads();
  const float dzf = dzf_s, dn = dg * zf * inv * inv;
  for (int c = threadIdx.x; c < Phi; c += blockDim.x) df[c] += gamma * dz[c] + 2.f * dn * f[c] + dzf * z[c];
  __syncthreads();
  for (int c = threadIdx.x; c < dm; c += blockDim.x) DKV[mi * ldkv + c] = from_f32<T>(dpfp_dk(k, df, dm, nu, c));
  for (int c = threadIdx.x; c < d; c += blockDim.x) DKV[mi * ldkv + dm + c] = from_f32<T>(DV[mi * d + c]);
}

// Part 3: dz (in place: gradient of the OLD z) += sum_i dzf_i f_i.  grid: (ceil(Phi / 256), g), block: 256.
__global__ __launch_bounds__(256) void update_bwd_z_kernel(const float* __restrict__ Fm, const float* __restrict__ DZF,
                                                           float* __restrict__ DZ, int first, int m, int Phi) {
  const int l = first + blockIdx.y, c = blockIdx.x * 256 + threadIdx.x;
  if (c >= Phi) return;
  float s = 0.f;
  for (int i = 0; i < m; ++i) s = fmaf(DZF[(size_t)l * m + i], Fm[((size_t)l * m + i) * Phi + c], s);
  DZ[(size_t)l * Phi + c] += s;
}

// beta_i = sigmoid(w_b . y_i): the memory rows of the output gradient get db_i w_b, and part[cell] = sum_i db_i y_i.
// dY: gradient slots (row 0 of the memory rows of cell l at dY + l * dy_cell); Ym: [cells][m][d] memory rows of the output.
// grid: (ceil(d / 256), g), block: 256.
template <typename T>
__global__ __launch_bounds__(256) void beta_bwd_kernel(const float* __restrict__ DB, const T* __restrict__ Ym, size_t ym_cell,
                                                       const LayerAux* __restrict__ aux, float* __restrict__ dY,
                                                       size_t dy_cell, float* __restrict__ part, int first, int m, int d) {
  const int l = first + blockIdx.y, c = blockIdx.x * 256 + threadIdx.x;
  if (c >= d) return;
  const float wb = to_f32(((const T*)aux[l].wm_b)[c]);
  float s = 0.f;
  for (int i = 0; i < m; ++i) {
    const float db = DB[(size_t)l * m + i];
    dY[(size_t)l * dy_cell + (size_t)i * d + c] += db * wb;
    s = fmaf(db, to_f32(Ym[(size_t)l * ym_cell + (size_t)i * d + c]), s);
  }
  part[(size_t)l * d + c] = s;       // per cell; colsum_finish_kernel adds the cells of a layer into dw_b
}

// ------------------------------------------------------------------------------------------------
// Tape of the training forward: inputs of a cell that the backward pass cannot recompute from its neighbours.
// Per cell (segment s, layer l, sequence b), record index s * n_cells + l * batch + b: the cell input [T][d] fp32, the layer's A [d][Phi] and
// z [Phi] from BEFORE the cell's update.  save = 1 copies slots / state into the tape, save = 0 copies back.
// Cell l of a launch belongs to layer l / batch and to segment t - l / batch.  grid: (blocks, g), block: 256.
__global__ __launch_bounds__(256) void tape_kernel(float* __restrict__ tape, size_t rec_floats, float* __restrict__ X,
                                                   size_t x_cell, const LayerAux* __restrict__ aux, float* __restrict__ Aw,
                                                   float* __restrict__ zw, int first, int t, int n_cells, int batch, size_t nx,
                                                   size_t nA, size_t nz, int save) {
  const int l = first + blockIdx.y;            // cell = layer * batch + sequence
  float* rec = tape + ((size_t)(t - l / batch) * n_cells + l) * rec_floats;
  float* x = X + (size_t)l * x_cell;
  float* A = save ? aux[l].A : Aw + (size_t)l * nA;
  float* z = save ? aux[l].z : zw + (size_t)l * nz;
  const size_t total = nx + nA + nz;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
    float* p = i < nx ? x + i : (i < nx + nA ? A + (i - nx) : z + (i - nx - nA));
    if (save) rec[i] = *p; else *p = rec[i];
  }
}

// Memory-state gradients between the caller's order [batch][layers][n] and the cell order [layers][batch][n] of a step.
// to_cells = 1: cells <- caller; 0: caller <- cells.  grid: (blocks, layers * batch), block: 256.
__global__ __launch_bounds__(256) void state_permute_kernel(float* __restrict__ dst, const float* __restrict__ src, int n_layers,
                                                            int batch, size_t n, int to_cells) {
  const int v = blockIdx.y, l = v / batch, b = v % batch;
  const size_t cell = (size_t)v * n, user = ((size_t)b * n_layers + l) * n;
  float* d = dst + (to_cells ? cell : user);
  const float* s = src + (to_cells ? user : cell);
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) d[i] = s[i];
}

// Gradient of the top layer's output: token rows from the caller's d_hidden, memory rows zero.
template <typename T>
__global__ __launch_bounds__(256) void load_dhidden_kernel(const T* __restrict__ dh, int S, int d, float* __restrict__ slot) {
  const int r = blockIdx.x;
  for (int c = threadIdx.x; c < d; c += blockDim.x) slot[(size_t)r * d + c] = r < S ? to_f32(dh[(size_t)r * d + c]) : 0.f;
}

// Gradient of a layer-0 cell's input: token rows -> dx of the segment (if asked for), memory rows += d_mem_emb.
__global__ __launch_bounds__(256) void store_dx_kernel(const float* __restrict__ slot, int S, int d, float* __restrict__ dx,
                                                       float* __restrict__ dmem) {
  const int r = blockIdx.x;
  for (int c = threadIdx.x; c < d; c += blockDim.x) {
    const float v = slot[(size_t)r * d + c];
    if (r < S) { if (dx) dx[(size_t)r * d + c] = v; }
    else dmem[(size_t)(r - S) * d + c] += v;
  }
}

}  // namespace armt
