// Shared device/host definitions of the ARMT forward library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace armt {

typedef __bf16 bf16;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kWave = 64;   // CDNA wavefront width

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16 v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16 from_f32<bf16>(float v) { return (bf16)v; }   // round to nearest even

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
  return v;
}

// Sum over the threads of a block (blockDim.x a multiple of 64, at most 1024); every thread gets it.
__device__ __forceinline__ float block_sum(float v, float* red /* >= 17 floats of LDS */) {
  v = wave_sum(v);
  const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[w] = v;
  __syncthreads();
  if (threadIdx.x == 0) {
    float s = 0.f;
    for (int i = 0; i < nw; ++i) s += red[i];
    red[16] = s;
  }
  __syncthreads();
  return red[16];
}

// ---------------------------------------------------------------------------------------------
// One entry of a grouped-GEMM pointer table: the operands of ONE group (= one layer's cell).
// The table of a GEMM kind holds one entry per layer; a launch covers entries [first, first + g).
// This is how every group multiplies by its own layer's weights without stacking them
// (paper Section 3.3 item 1).
struct GemmGroup {
  const void* A;          // [M, K] activations, row stride lda
  const void* B0;         // weight block 0: rows [0, n0) of the logical [N, K] operand
  const void* B1;         // weight block 1: rows [n0, n0 + n1)  (SwiGLU: the "up" weight)
  const void* B2;         // weight block 2: the remaining rows
  void* C;                // primary output
  void* C2;               // optional copy of C in the activation type (or null)
  const float* R;         // residual [M, ldr] (or null); EPI_QKV_ROPE: cos/sin table
  const float* rowscale;  // per-row factor applied to the accumulator (or null)
  const void* gain;       // EPI_RESID_F32: C2 = (bf16)(result * gain[col]) instead of (bf16)result (or null)
  float* ssq_out;         // EPI_RESID_F32: [M][tiles_n] per-row sums of squares of the result, one per N-tile (or null)
  const void* pad_[6];    // keep entries at 128 bytes
};
static_assert(sizeof(GemmGroup) == 128, "pointer-table entries are 128 bytes");

enum GemmEpilogue : int {
  EPI_STORE_ACT = 0,   // C (activation type) = acc * rowscale[row]
  EPI_STORE_F32 = 1,   // C (fp32) = acc * rowscale[row]
  EPI_RESID_F32 = 2,   // C (fp32) = R + acc * rowscale[row]; C2 (activation type) = same, if given
  EPI_SWIGLU = 3,      // C (activation type) = silu(rs * acc over B0) * (rs * acc over B1), rs = rowscale[row]; N = rows of B0
  EPI_DPFP_READ = 5,   // read side of the associative memory (Eq. 6) fused behind the W_Q projection: the N = n0 = d_mem result
                       // columns q of a row never leave the workgroup; written are phi(q) (DPFP-nu, nu = ldr; activation
                       // type, C [M][ldc], ldc >= 2 nu d_mem) and 1 / (z . phi(q) + fparam) (fp32, C2 [M]); z = R [2 nu d_mem].
                       // All N columns must lie in one output tile.
  EPI_QKV_ROPE = 4     // EPI_STORE_ACT of the fused q | k | v projection with the rotary embedding applied to the q and k
                       // columns [0, n0 + n1): heads of ldr columns, rotate-half pairing, position = row; R = cos/sin table
                       // [M][ldr / 2][2].  Heads must not straddle output tiles (tile width a multiple of ldr).
                       // With ldc2 > 0 the v columns [n0 + n1, N) are not stored in C but transposed in C2:
                       // C2[(n - n0 - n1) * ldc2 + m]; n0 + n1 must then be a multiple of the tile width.
};

struct GemmShape {
  int M, N, K;          // N = output columns (for EPI_SWIGLU: d_ff, each column needs two dot products)
  int lda, ldc, ldc2, ldr;   // ldr: row stride of R; EPI_QKV_ROPE: head dimension
  int n0, n1;           // rows in weight blocks 0 and 1 (block 2 holds N - n0 - n1)
  int epi;              // GemmEpilogue
  int tag;              // which GEMM of the step this is (profiling only)
  int dbg;              // A/B switches for benchmarks: bit 5 (32) multiplies the 16 memory rows as a tile of their own
                        // instead of a strip of the last M-tile (same results up to rounding order)
  int ldb;              // row stride of the weight blocks in elements (>= K); the weights of the model are dense: ldb = K
  float fparam = 0.f;   // EPI_DPFP_READ: assoc_eps
  int a_rows = 0;       // rows of A that may be READ in every group (0: M).  Operand buffers that are padded to whole
                        // tiles let a ragged M take the copies without per-lane clamping; rows >= M are never stored
};

}  // namespace armt
