// Segment attention on the CDNA4 matrix cores (paper Section 4.2): causal softmax(q k^T / sqrt(dh)) v
// over the T rows of each cell, grouped-query heads, batched over the cells of the group.
//
// One workgroup = one KV head of one cell x NQ x 32 query rows; wave w handles query head kv * GROUP + w % GROUP and
// the 32 rows of sub-tile w / GROUP, so all waves share the K / V tiles in LDS.  NQ = 1 for grouped-query heads (all
// waves have the same causal extent); with one query head per KV head a workgroup of a single wave would leave the CU
// nearly empty, so NQ = 4 consecutive row tiles share the stream of K / V tiles (a wave skips the tiles past its rows).  Per 64-key tile a wave
// computes S^T = K Q^T with v_mfma_f32_32x32x16_bf16 (keys along the rows, so a lane holds ONE query
// column: the running max / sum of the online softmax are per-lane scalars and need a single exchange
// between the two half-waves), turns it into P^T in registers -- the MFMA result layout is directly the
// B-operand layout of the second product -- and accumulates O^T += V^T P^T.  V is needed with the key
// index contiguous, so a pre-pass stores it transposed ([dh][T]) next to rotating q and k.
// K / V^T tiles are double buffered and filled with direct global-to-LDS loads.
#pragma once

#include "common.h"
#include "gemm_mfma.h"

namespace armt {

constexpr int AT_KT = 64;      // keys per tile
constexpr int AT_QT = 32;      // query rows per wave / workgroup
constexpr float AT_LAZY_SUM = 4096.f;  // the online softmax lets a lane's 16 unnormalised probabilities of a half-tile add up to this

// Which key of a 64-key tile sits in LDS row `row` of the K tile.  The 32 x 32 MFMA leaves S^T[row][query] of a lane in
// registers r = 0..15 <-> rows 8 (r / 4) + 4 half + r % 4, and registers 8 ss .. 8 ss + 7 become the lane's B operand
// of k-step ss of the second product.  With the rows of every 16-row group holding the keys in 4-key blocks ordered
// 0, 2, 1, 3, those eight registers are the eight CONSECUTIVE keys 16 ss + 8 half .. + 7, so the matching A operand is one
// 16-byte piece of a V^T row.  The permutation costs nothing: it only changes which global row a copy lane reads.
// max of a value over the two half-waves (lanes i and i ^ 32), in every lane: one lane-half swap instead of a
// round trip through the LDS crossbar
__device__ __forceinline__ float at_max_halves(float v) {
  typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
  const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

__device__ __forceinline__ int at_key_of_row(int row) {
  return (row & ~12) | ((row & 4) << 1) | ((row & 8) >> 1);
}

// V of every cell transposed: Vt[l][kvh][c][j] = V[l][j][kvh*dh + c], j padded with zeros to Tp.
// grid: (Tp / 64, Hkv, g), block: 256.
__global__ __launch_bounds__(256) void v_transpose_kernel(const bf16* __restrict__ QKV, bf16* __restrict__ Vt,
                                                          int first, int Trows, int Tp, int H, int Hkv, int dh) {
  extern __shared__ __align__(16) unsigned char smraw[];
  bf16* tile = (bf16*)smraw;                   // [64][dh + 2]
  const int l = first + blockIdx.z, kvh = blockIdx.y, j0 = blockIdx.x * 64;
  const int ldq = (H + 2 * Hkv) * dh, ldt = dh + 2;
  const bf16* src = QKV + (size_t)l * Trows * ldq + (H + Hkv) * dh + kvh * dh;
  for (int idx = threadIdx.x; idx < 64 * dh; idx += blockDim.x) {
    const int jr = idx / dh, c = idx - jr * dh;
    tile[jr * ldt + c] = (j0 + jr < Trows) ? src[(size_t)(j0 + jr) * ldq + c] : (bf16)0.f;
  }
  __syncthreads();
  bf16* dst = Vt + ((size_t)(l * Hkv + kvh) * dh) * Tp + j0;
  for (int idx = threadIdx.x; idx < 64 * dh; idx += blockDim.x) {
    const int c = idx >> 6, jr = idx & 63;
    dst[(size_t)c * Tp + jr] = tile[jr * ldt + c];
  }
}

// QKV: [L][T][(H + 2 Hkv) dh] with q, k already rotated; Vt as above; Out: [L][T][H dh]; lse2: optional, see the end.
// grid: 1-D, 8 * ceil(Hkv g / 8) * nqt workgroups with nqt = ceil(T / (32 NQ)); block: NQ * GROUP * 64 with GROUP = H / Hkv.
// Workgroup b belongs to XCD b % 8 (the hardware deals consecutive workgroups round the 8 XCDs).  A (cell, KV head)
// pair stays on ONE XCD, so its K / V tiles are fetched into one L2 only, and inside an XCD the workgroups are ordered
// by their length over ALL pairs, longest (latest query rows) first: a workgroup of the last row tile runs 2 nqt / NQ
// times as long as one of the first, and in a per-pair order the long workgroups of the last pairs would start when
// most of the chip has already run dry.
template <int DH>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(DH == 64 ? 4 : 3))) void attention_mfma_kernel(const bf16* __restrict__ QKV, const bf16* __restrict__ Vt,
                                                             bf16* __restrict__ Out, int first, int Trows, int Tp,
                                                             int H, int Hkv, int nq, float scale_log2e,
                                                             float* __restrict__ lse2, int nqt, int npairs) {
  // a K tile is DH / 64 sub-tiles [64 keys][64 dims] with 128-byte rows
  constexpr int K_BYTES = AT_KT * DH * 2;
  constexpr int V_BYTES = DH * AT_KT * 2;          // V^T tile: [DH dims][64 keys], 128-byte rows
  constexpr int STAGE = K_BYTES + V_BYTES;
  constexpr int K_SLABS = K_BYTES / 1024, V_SLABS = V_BYTES / 1024;
  constexpr int KS = DH / 16;                      // k-steps of the first product
  constexpr int OT = DH / 32;                      // 32-row tiles of O^T
  extern __shared__ __align__(16) unsigned char smem[];   // [2][STAGE]

  const int ppx = (npairs + 7) >> 3;               // pairs per XCD
  const int xj = blockIdx.x >> 3;                  // index inside the XCD
  const int qt = nqt - 1 - xj / ppx;               // long (late) query tiles first
  const int pair = (xj % ppx) * 8 + (blockIdx.x & 7);
  if (pair >= npairs) return;                      // padding of the last XCD round (whole workgroup)
  const int kvh = pair % Hkv, l = first + pair / Hkv;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int nw = blockDim.x >> 6, group = H / Hkv;
  const int head = kvh * group + wave % group;
  const int ldq = (H + 2 * Hkv) * DH;
  const int q0 = (qt * nq + wave / group) * AT_QT;  // first row of this wave (may lie past the cell in the last workgroup)
  const bool live = q0 < Trows;
  const int qcol = lane & 31, half = lane >> 5;

  const bf16* cell = QKV + (size_t)l * Trows * ldq;
  const char* kbase = (const char*)(cell + H * DH + kvh * DH);
  const char* vbase = (const char*)(Vt + (size_t)(l * Hkv + kvh) * DH * Tp);

  // ---- Q fragments (B operand: lane holds query row qcol, 8 consecutive dims per k-step)
  bf16x8 qf[KS];
  {
    const int qrow = min(q0 + qcol, Trows - 1);
    const bf16* qp = cell + (size_t)qrow * ldq + head * DH + half * 8;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[ks] = *(const bf16x8*)(qp + ks * 16);
  }

  // ---- tile copies: slab = 8 rows x 128 bytes; lane i fills row i/8, physical chunk i%8.
  // A copy is addressed as scalar base + one 32-bit lane offset: the LDS row of slab sl is 8 (sl % 8) + R, whose key
  // (see at_key_of_row) splits into a part of R alone and a part of the slab alone, and whose swizzle depends on the
  // slab only through its parity (bit 6 of the byte offset).  Issuing a copy then costs scalar instructions and one
  // vector XOR instead of a dozen 64-bit vector operations per copy, which the SIMD would have to fit between the
  // matrix instructions of its other waves.  Only the K rows of a cell's last tile (keys past T, clamped per lane) take the
  // general form.
  const int R = lane >> 3, pc = lane & 7;
  const unsigned chunk0 = (unsigned)((pc ^ mf_swz(R)) << 4);
  const unsigned voffK = (unsigned)((R & 3) + ((R >> 2) << 3)) * (unsigned)ldq * 2u + chunk0;
  const unsigned voffV = (unsigned)R * (unsigned)Tp * 2u + chunk0;
  const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) void*)smem;
  auto dma = [&](const char* base, unsigned voff, unsigned lds) {
    asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(voff), "s"(base), "s"(lds) : "memory", "m0");
  };
  auto issue_tile = [&](int kt, int buf) {
    typedef const __attribute__((address_space(1))) void* gptr_t;
    typedef __attribute__((address_space(3))) void* lptr_t;
    unsigned char* Ks = smem + buf * STAGE;
    const unsigned ldsK = lds0 + buf * STAGE, ldsV = ldsK + K_BYTES;
    const int k0 = kt * AT_KT;
    const bool whole = k0 + AT_KT <= Trows;          // wave-uniform: every key of the tile exists
    for (int sl = wave; sl < K_SLABS + V_SLABS; sl += nw) {
      if (sl < K_SLABS) {
        const int sub = sl >> 3, a = sl & 7;
        if (whole) {
          const int keyS = k0 + ((a & 1) << 2) + ((a >> 1) << 4);
          dma(kbase + ((size_t)keyS * ldq + sub * 64) * 2, voffK ^ ((unsigned)(a & 1) << 6), ldsK + sl * 1024);
        } else {
          const int row = a * 8 + R;                                     // row of the tile in LDS
          const int key = min(k0 + at_key_of_row(row), Trows - 1);       // keys past T are masked by causality
          const char* src = kbase + ((size_t)key * ldq + sub * 64 + ((pc ^ mf_swz(row)) << 3)) * 2;
          __builtin_amdgcn_global_load_lds((gptr_t)src, (lptr_t)(Ks + sl * 1024), 16, 0, 0);
        }
      } else {
        const int vs = sl - K_SLABS;                                     // dim rows 8 vs .. 8 vs + 7 of V^T
        dma(vbase + ((size_t)vs * 8 * Tp + k0) * 2, voffV ^ ((unsigned)(vs & 1) << 6), ldsV + vs * 1024);
      }
    }
  };

  const int fl = mf_swz(lane & 31);
  f32x16 o[OT];
#pragma unroll
  for (int t = 0; t < OT; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[t][r] = 0.f;
  float m = -INFINITY, lsum = 0.f, lsum1 = 0.f;

  const int nkt = (min((qt + 1) * nq * AT_QT, Trows) + AT_KT - 1) / AT_KT;   // key tiles of the workgroup's last rows
  issue_tile(0, 0);
  __builtin_amdgcn_s_waitcnt(0x0F70);
  __syncthreads();

  for (int kt = 0; kt < nkt; ++kt) {
    const int cur = kt & 1, k0 = kt * AT_KT;
    if (kt + 1 < nkt) issue_tile(kt + 1, cur ^ 1);
    const unsigned char* Ks = smem + cur * STAGE;
    const unsigned char* Vs = Ks + K_BYTES;
    if (live && k0 < q0 + AT_QT) {                 // wave-uniform: the tile holds keys this wave's rows may see

    // The tile's two 32-key halves one after the other: S^T[key][query] of a half, its share of the online softmax,
    // its share of O^T.  (A half at a time keeps 16 instead of 32 score registers and 2 instead of 4 P fragments
    // alive: under 128 registers per lane, four waves per SIMD.)
#pragma unroll
    for (int jj = 0; jj < 2; ++jj) {
      if (k0 + jj * 32 >= q0 + AT_QT) continue;      // wave-uniform: every key of this half lies after the wave's rows
      f32x16 sc;
#pragma unroll
      for (int r = 0; r < 16; ++r) sc[r] = 0.f;
      const unsigned char* krow = Ks + (jj * 32 + (lane & 31)) * MF_ROW_BYTES;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const bf16x8 kf = *(const bf16x8*)(krow + (ks >> 2) * (AT_KT * MF_ROW_BYTES) + (((2 * (ks & 3) + half) ^ fl) << 4));
        sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], sc, 0, 0, 0);
      }
      if (k0 + jj * 32 + 31 > q0) {     // the half crosses the diagonal: mask keys after the query
        const int qi = q0 + qcol;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = k0 + jj * 32 + 16 * (r >> 3) + 8 * half + (r & 7);   // see at_key_of_row
          if (key > qi) sc[r] = -INFINITY;
        }
      }
      // online softmax: every lane owns one query column; 16 of the half's keys here, the other 16 in lane ^ 32.
      // m is the REFERENCE of the exponents, not the running maximum (the result does not depend on it: numerator and
      // denominator carry the same factor).  The first half-tile sets it to that half's maximum; after that the common
      // case does not look for the maximum at all: the probabilities are formed against the current reference, and only
      // if some lane's 16 of them add up to more than AT_LAZY_SUM = 2^12 (or the sum is not finite) the wave takes the
      // maximum, moves the reference, rescales O and the sums, and forms them again.
      float pr[16], hs0, hs1;
      auto form = [&](float mc) __attribute__((always_inline)) {
        hs0 = hs1 = 0.f;
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
          pr[r] = __builtin_amdgcn_exp2f(fmaf(sc[r], scale_log2e, -mc));
          pr[r + 1] = __builtin_amdgcn_exp2f(fmaf(sc[r + 1], scale_log2e, -mc));
          // two running sums in plain fp32 adds.  (A dot instruction on the packed pair, v_dot2c_f32_bf16, would halve
          // the count, but the sums it produced shifted every gradient of the backward pass by 2 - 3 %: the backward pass
          // takes P from this row sum and cancels a common component of dP against D = dO.O, which amplifies any bias.)
          if (r & 2) hs1 += pr[r] + pr[r + 1];
          else hs0 += pr[r] + pr[r + 1];
        }
      };
      if (jj == 0 && kt == 0) {         // a query's first half-tile: start the reference at its maximum (wave-uniform)
        float mx = sc[0];
#pragma unroll
        for (int r = 1; r < 16; ++r) mx = fmaxf(mx, sc[r]);
        m = at_max_halves(mx);
      }
      form(m * scale_log2e);
      if (__builtin_amdgcn_ballot_w64(!(hs0 + hs1 <= AT_LAZY_SUM)) != 0) {
        float mx = sc[0];
#pragma unroll
        for (int r = 1; r < 16; ++r) mx = fmaxf(mx, sc[r]);
        mx = at_max_halves(mx);
        const float m_new = fmaxf(m, mx);
        const float alpha = __builtin_amdgcn_exp2f((m - m_new) * scale_log2e);
        m = m_new;
        lsum *= alpha;
        lsum1 *= alpha;
#pragma unroll
        for (int t = 0; t < OT; ++t)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[t][r] *= alpha;
        form(m * scale_log2e);
      }
      lsum += hs0;
      lsum1 += hs1;
      // P^T as the B operand of the second product: two 16-key k-steps, packed to bf16 in pairs
      bf16x8 pf[2];
#pragma unroll
      for (int r = 0; r < 16; r += 2) {
        typedef float f32x2 __attribute__((ext_vector_type(2)));
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        const bf16x2 pk = __builtin_convertvector(f32x2{pr[r], pr[r + 1]}, bf16x2);
        pf[r >> 3][r & 7] = pk[0];
        pf[r >> 3][(r & 7) + 1] = pk[1];
      }
      // O^T[dim][query] += V^T[dim][key] P^T[key][query]; k-step ss of half jj covers the keys
      // jj*32 + 16*ss + 8*half + 0..7 (see at_key_of_row): registers 8*ss .. 8*ss+7 of sc, one 16-byte piece of a V^T row
#pragma unroll
      for (int t = 0; t < OT; ++t) {
        const unsigned char* vrow = Vs + (t * 32 + (lane & 31)) * MF_ROW_BYTES;
#pragma unroll
        for (int ss = 0; ss < 2; ++ss) {
          const bf16x8 vf = *(const bf16x8*)(vrow + (((jj * 4 + 2 * ss + half) ^ fl) << 4));
          o[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[ss], o[t], 0, 0, 0);
        }
      }
    }
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
  }

  lsum += lsum1;
  lsum += __shfl_xor(lsum, 32, kWave);
  const float inv = 1.0f / lsum;
  const int qi = q0 + qcol;
  // log2 of the row's sum of exponentials, [cells][H][T]: what the backward pass needs to rebuild P
  if (lse2 && qi < Trows && half == 0) lse2[((size_t)l * H + head) * Trows + qi] = fmaf(m, scale_log2e, __builtin_amdgcn_logf(lsum));
  if (qi < Trows) {
    bf16* dst = Out + ((size_t)l * Trows + qi) * (H * DH) + head * DH;
#pragma unroll
    for (int t = 0; t < OT; ++t)
#pragma unroll
      for (int rg = 0; rg < 4; ++rg) {         // registers 4*rg .. 4*rg+3 hold 4 consecutive dims
        bf16x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = (bf16)(o[t][4 * rg + e] * inv);
        *(bf16x4*)(dst + t * 32 + 8 * rg + 4 * half) = v;
      }
  }
}

inline int attention_tp(int Trows) { return (Trows + AT_KT - 1) / AT_KT * AT_KT; }

// bytes of V^T scratch for g cells
inline size_t attention_vt_bytes(int g, int Trows, int Hkv, int dh) {
  return (size_t)g * Hkv * dh * attention_tp(Trows) * 2;
}

inline hipError_t launch_attention_mfma(const bf16* QKV, bf16* Vt, bf16* Out, int first, int g, int Trows, int H,
                                        int Hkv, int dh, bool vt_ready, hipStream_t st, float* lse2 = nullptr) {
  const int Tp = attention_tp(Trows), group = H / Hkv;
  hipError_t e = hipSuccess;
  if (!vt_ready) {      // V^T not yet written by the producer of QKV
    v_transpose_kernel<<<dim3(Tp / 64, Hkv, g), 256, 64 * (dh + 2) * 2, st>>>(QKV, Vt, first, Trows, Tp, H, Hkv, dh);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  const float scale_log2e = 1.4426950408889634f / sqrtf((float)dh);
  const int nq = group == 1 ? 4 : (group == 2 ? 2 : 1);       // row tiles per workgroup: at least 4 waves share the K / V tiles
  const int nqt = (Trows + nq * AT_QT - 1) / (nq * AT_QT), npairs = Hkv * g;
  const dim3 grid(8 * ((npairs + 7) / 8) * nqt);
  if (dh == 64)
    attention_mfma_kernel<64><<<grid, nq * group * 64, 2 * (64 * 64 * 2 * 2), st>>>(QKV, Vt, Out, first, Trows, Tp, H, Hkv, nq, scale_log2e, lse2, nqt, npairs);
  else
    attention_mfma_kernel<128><<<grid, nq * group * 64, 2 * (64 * 128 * 2 * 2), st>>>(QKV, Vt, Out, first, Trows, Tp, H, Hkv, nq, scale_log2e, lse2, nqt, npairs);
  return hipGetLastError();
}

}  // namespace armt
