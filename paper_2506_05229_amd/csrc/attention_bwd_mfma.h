// Backward of the segment attention on the CDNA4 matrix cores (bf16, head_dim 64 or 128).
//
// With P = softmax(scale Q K^T) (causal), O = P V and upstream gradient dO:
//   D_i = dO_i . O_i,   dP = dO V^T,   dS = P (dP - D) scale,   dQ = dS K,   dK = dS^T Q,   dV = P^T dO.
// P is recomputed from the log-sum-exp the forward kernel leaves behind (log2 domain), so no T x T matrix is stored.
// Two kernels, both built like the forward one (v_mfma_f32_32x32x16_bf16, a lane owns ONE column of every 32 x 32
// result, so the result of one product is directly the B operand of the next):
//   dq kernel:  a lane owns a query.  S^T = K Q^T and dP^T = V dO^T (keys along the rows), dS^T in registers,
//               dQ^T += K^T dS^T.  K, V and K^T tiles of a KV head are shared in LDS by the waves of its query heads.
//   dkv kernel: a lane owns a key.  S = Q K^T and dP = dO V^T (queries along the rows), P and dS in registers,
//               dV^T += dO^T P, dK^T += Q^T dS.  A wave keeps its 32 keys for the whole kernel and adds up all query
//               heads of the KV group; the waves of a workgroup share the Q, dO, Q^T, dO^T tiles of the current head in LDS.
// Operands with the sequence index contiguous (K^T, Q^T, dO^T) come from head_transpose_kernel.
#pragma once

#include "attention_mfma.h"
#include "common.h"

namespace armt {

// Xt[l][h][c][j] = X[l][j][col0 + h * dh + c], j padded with zeros to Tp.  X: [cells][T][ldx].
// grid: (Tp / 64, heads, g), block: 256; LDS: 64 * (dh + 2) bf16.
__global__ __launch_bounds__(256) void head_transpose_kernel(const bf16* __restrict__ X, int ldx, int col0, bf16* __restrict__ Xt,
                                                             int first, int Trows, int Tp, int heads, int dh) {
  extern __shared__ __align__(16) unsigned char smraw[];
  bf16* tile = (bf16*)smraw;                   // [64][dh + 2]
  const int l = first + blockIdx.z, h = blockIdx.y, j0 = blockIdx.x * 64;
  const int ldt = dh + 2;
  const bf16* src = X + (size_t)l * Trows * ldx + col0 + h * dh;
  for (int idx = threadIdx.x; idx < 64 * dh; idx += blockDim.x) {
    const int jr = idx / dh, c = idx - jr * dh;
    tile[jr * ldt + c] = (j0 + jr < Trows) ? src[(size_t)(j0 + jr) * ldx + c] : (bf16)0.f;
  }
  __syncthreads();
  bf16* dst = Xt + ((size_t)(l * heads + h) * dh) * Tp + j0;
  for (int idx = threadIdx.x; idx < 64 * dh; idx += blockDim.x) {
    const int c = idx >> 6, jr = idx & 63;
    dst[(size_t)c * Tp + jr] = tile[jr * ldt + c];
  }
}

// D[l][h][i] = dO[l][i][h*dh : (h+1)*dh] . O[same].  grid: (ceil(T / 4), g), block: 256 (a wave per row, all heads).
__global__ __launch_bounds__(256) void attention_dvec_kernel(const bf16* __restrict__ O, const bf16* __restrict__ dO,
                                                             float* __restrict__ Dv, int first, int Trows, int H, int dh) {
  const int l = first + blockIdx.y, i = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (i >= Trows) return;
  const size_t row = ((size_t)l * Trows + i) * (H * dh);
  for (int h = 0; h < H; ++h) {
    float s = 0.f;
    for (int c = lane; c < dh; c += 64) s = fmaf((float)dO[row + h * dh + c], (float)O[row + h * dh + c], s);
    s = wave_sum(s);
    if (lane == 0) Dv[((size_t)l * H + h) * Trows + i] = s;
  }
}

// dQ.  QKV: [cells][T][(H + 2 Hkv) dh] (q, k rotated); Kt: [cells][Hkv][dh][Tp]; dO: [cells][T][H dh];
// LSE2 (log2 domain), Dv: [cells][H][T]; dQKV: gradient rows, q columns written here.
// As in the forward kernel a workgroup takes NQ consecutive 32-row tiles (NQ > 1 when a KV head has fewer than four
// query heads): wave w handles query head kv * GROUP + w % GROUP and row tile w / GROUP.
// grid: 1-D, 8 * ceil(Hkv g / 8) * ceil(T / (32 NQ)) workgroups, block: NQ * GROUP * 64; LDS: 2 stages of K, V, K^T tiles.
template <int DH>
__global__ __launch_bounds__(512) void attention_bwd_dq_kernel(const bf16* __restrict__ QKV, const bf16* __restrict__ Kt,
                                                               const bf16* __restrict__ dO, const float* __restrict__ LSE2,
                                                               const float* __restrict__ Dv, bf16* __restrict__ dQKV,
                                                               int first, int Trows, int Tp, int H, int Hkv, int nq, float scale,
                                                               int nqt, int npairs) {
  constexpr int K_BYTES = AT_KT * DH * 2;          // K and V tiles: DH / 64 sub-tiles [64 keys][64 dims], 128-byte rows
  constexpr int T_BYTES = DH * AT_KT * 2;          // K^T tile: [DH dims][64 keys]
  constexpr int STAGE = 2 * K_BYTES + T_BYTES;
  constexpr int K_SLABS = K_BYTES / 1024, T_SLABS = T_BYTES / 1024;
  constexpr int KS = DH / 16, OT = DH / 32;
  extern __shared__ __align__(16) unsigned char smem[];   // [2][STAGE]

  // work order of the forward kernel: a (cell, KV head) pair stays on one XCD, longest row tiles first over all pairs
  const int ppx = (npairs + 7) >> 3, xj = blockIdx.x >> 3;
  const int qt = nqt - 1 - xj / ppx;
  const int pair = (xj % ppx) * 8 + (blockIdx.x & 7);
  if (pair >= npairs) return;
  const int kvh = pair % Hkv, l = first + pair / Hkv;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int nw = blockDim.x >> 6, group = H / Hkv;
  const int head = kvh * group + wave % group;
  const int ldq = (H + 2 * Hkv) * DH;
  const int q0 = (qt * nq + wave / group) * AT_QT;   // may lie past the cell in the last workgroup
  const bool live = q0 < Trows;
  const int qcol = lane & 31, half = lane >> 5;
  const float scale_log2e = scale * 1.4426950408889634f;

  const bf16* cell = QKV + (size_t)l * Trows * ldq;
  const char* kbase = (const char*)(cell + H * DH + kvh * DH);
  const char* vbase = (const char*)(cell + (H + Hkv) * DH + kvh * DH);
  const char* tbase = (const char*)(Kt + (size_t)(l * Hkv + kvh) * DH * Tp);

  const int qrow = min(q0 + qcol, Trows - 1);
  bf16x8 qf[KS], gf[KS];       // B operands: this lane's query row of Q and of dO
  {
    const bf16* qp = cell + (size_t)qrow * ldq + head * DH + half * 8;
    const bf16* gp = dO + ((size_t)l * Trows + qrow) * (H * DH) + head * DH + half * 8;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      qf[ks] = *(const bf16x8*)(qp + ks * 16);
      gf[ks] = *(const bf16x8*)(gp + ks * 16);
    }
  }
  const float lse = LSE2[((size_t)l * H + head) * Trows + qrow];
  const float dvec = Dv[((size_t)l * H + head) * Trows + qrow];

  const int R = lane >> 3, pc = lane & 7;
  auto issue_tile = [&](int kt, int buf) {
    typedef const __attribute__((address_space(1))) void* gptr_t;
    typedef __attribute__((address_space(3))) void* lptr_t;
    unsigned char* Ks = smem + buf * STAGE;
    const int k0 = kt * AT_KT;
    for (int sl = wave; sl < 2 * K_SLABS + T_SLABS; sl += nw) {
      if (sl < 2 * K_SLABS) {
        const bool isv = sl >= K_SLABS;
        const int s2 = isv ? sl - K_SLABS : sl;
        const int sub = s2 >> 3, row = (s2 & 7) * 8 + R;
        const int key = min(k0 + row, Trows - 1);
        const char* src = (isv ? vbase : kbase) + ((size_t)key * ldq + sub * 64 + ((pc ^ mf_swz(row)) << 3)) * 2;
        __builtin_amdgcn_global_load_lds((gptr_t)src, (lptr_t)(Ks + sl * 1024), 16, 0, 0);
      } else {
        const int ts = sl - 2 * K_SLABS, row = ts * 8 + R;
        const char* src = tbase + ((size_t)row * Tp + k0 + ((pc ^ mf_swz(row)) << 3)) * 2;
        __builtin_amdgcn_global_load_lds((gptr_t)src, (lptr_t)(Ks + 2 * K_BYTES + ts * 1024), 16, 0, 0);
      }
    }
  };

  const int fl = mf_swz(lane & 31);
  f32x16 o[OT];
#pragma unroll
  for (int t = 0; t < OT; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[t][r] = 0.f;

  const int qi = q0 + qcol;
  const int nkt = (min((qt + 1) * nq * AT_QT, Trows) + AT_KT - 1) / AT_KT;   // key tiles of the workgroup's last rows
  issue_tile(0, 0);
  __builtin_amdgcn_s_waitcnt(0x0F70);
  __syncthreads();

  for (int kt = 0; kt < nkt; ++kt) {
    const int cur = kt & 1, k0 = kt * AT_KT;
    if (kt + 1 < nkt) issue_tile(kt + 1, cur ^ 1);
    const unsigned char* Ks = smem + cur * STAGE;
    const unsigned char* Vs = Ks + K_BYTES;
    const unsigned char* Ts = Ks + 2 * K_BYTES;
    if (live && k0 < q0 + AT_QT) {                 // wave-uniform: the tile holds keys this wave's rows may see
    bf16x8 dsf[2][2];
#pragma unroll
    for (int jj = 0; jj < 2; ++jj) {
      f32x16 s, dp;
#pragma unroll
      for (int r = 0; r < 16; ++r) s[r] = dp[r] = 0.f;
      const int roff = (jj * 32 + (lane & 31)) * MF_ROW_BYTES;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const int off = roff + (ks >> 2) * (AT_KT * MF_ROW_BYTES) + (((2 * (ks & 3) + half) ^ fl) << 4);
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const bf16x8*)(Ks + off), qf[ks], s, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const bf16x8*)(Vs + off), gf[ks], dp, 0, 0, 0);
      }
      if (k0 + jj * 32 + 31 > q0) {              // this half crosses the diagonal: keys after the query contribute nothing
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = k0 + jj * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
          const float p = key > qi ? 0.f : __builtin_amdgcn_exp2f(fmaf(s[r], scale_log2e, -lse));
          dsf[jj][r >> 3][r & 7] = (bf16)(p * (dp[r] - dvec) * scale);
        }
      } else {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float p = __builtin_amdgcn_exp2f(fmaf(s[r], scale_log2e, -lse));
          dsf[jj][r >> 3][r & 7] = (bf16)(p * (dp[r] - dvec) * scale);
        }
      }
    }
    // dQ^T[dim][query] += K^T[dim][key] dS^T[key][query]
#pragma unroll
    for (int t = 0; t < OT; ++t) {
      const unsigned char* trow = Ts + (t * 32 + (lane & 31)) * MF_ROW_BYTES + 8 * half;
#pragma unroll
      for (int jj = 0; jj < 2; ++jj)
#pragma unroll
        for (int ss = 0; ss < 2; ++ss) {
          const int ch = jj * 4 + 2 * ss;
          const bf16x4 lo = *(const bf16x4*)(trow + ((ch ^ fl) << 4));
          const bf16x4 hi = *(const bf16x4*)(trow + (((ch + 1) ^ fl) << 4));
          bf16x8 tf;
          tf[0] = lo[0]; tf[1] = lo[1]; tf[2] = lo[2]; tf[3] = lo[3];
          tf[4] = hi[0]; tf[5] = hi[1]; tf[6] = hi[2]; tf[7] = hi[3];
          o[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tf, dsf[jj][ss], o[t], 0, 0, 0);
        }
    }
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
  }

  if (qi < Trows) {
    bf16* dst = dQKV + ((size_t)l * Trows + qi) * ldq + head * DH;
#pragma unroll
    for (int t = 0; t < OT; ++t)
#pragma unroll
      for (int rg = 0; rg < 4; ++rg) {
        bf16x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = (bf16)o[t][4 * rg + e];
        *(bf16x4*)(dst + t * 32 + 8 * rg + 4 * half) = v;
      }
  }
}

// dK, dV.  Qt, dOt: [cells][H][dh][Tp] (sequence index contiguous, zero padded); dQKV: k and v columns written here.
// One workgroup = one KV head of one cell x 256 keys; wave w (of 8) owns keys [32 w, 32 w + 32) of them (K, V rows in registers
// as B operands) for the whole kernel and adds the contributions of all query heads of the KV group, one after the
// other, in its registers: no reduction between waves or workgroups.  The eight waves share the tiles of the current
// (query head, 64 query rows): Q and dO rows, Q^T and dO^T columns, the rows' log-sum-exp and D, double buffered in LDS.
// grid: 1-D, 8 * ceil(Hkv g / 8) * ceil(T / 256) workgroups, block: 512; LDS: 2 stages of 4 tiles + 512 bytes.
constexpr int DKV_WAVES = 8;
template <int DH>
__global__ __launch_bounds__(512) void attention_bwd_dkv_kernel(const bf16* __restrict__ QKV, const bf16* __restrict__ Qt,
                                                                const bf16* __restrict__ dO, const bf16* __restrict__ dOt,
                                                                const float* __restrict__ LSE2, const float* __restrict__ Dv,
                                                                bf16* __restrict__ dQKV, int first, int Trows, int Tp, int H,
                                                                int Hkv, float scale, int npairs) {
  constexpr int Q_BYTES = 64 * DH * 2;             // one tile: 64 x DH or DH x 64 bf16
  constexpr int STAGE = 4 * Q_BYTES + 512;         // Q, dO, Q^T, dO^T, then lse[64], D[64]
  constexpr int Q_SLABS = Q_BYTES / 1024;
  constexpr int KS = DH / 16, OT = DH / 32;
  extern __shared__ __align__(16) unsigned char smem[];   // [2][STAGE]

  // key block 0 meets every query row, the last one a few: longest first over all (cell, KV head) pairs, a pair on one XCD
  const int ppx = (npairs + 7) >> 3, xj = blockIdx.x >> 3;
  const int kb = xj / ppx;
  const int pair = (xj % ppx) * 8 + (blockIdx.x & 7);
  if (pair >= npairs) return;
  const int kvh = pair % Hkv, l = first + pair / Hkv;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int group = H / Hkv;
  const int ldq = (H + 2 * Hkv) * DH, ldo = H * DH;
  const int k0 = kb * (32 * DKV_WAVES) + wave * 32;
  const int half = lane >> 5;
  const float scale_log2e = scale * 1.4426950408889634f;
  const int ki = k0 + (lane & 31);

  const bf16* cell = QKV + (size_t)l * Trows * ldq;
  const bf16* gcell = dO + (size_t)l * Trows * ldo;
  bf16x8 kf[KS], vf[KS];       // B operands: this lane's key row of K and of V
  {
    const int krow = min(ki, Trows - 1);
    const bf16* kp = cell + (size_t)krow * ldq + (H + kvh) * DH + half * 8;
    const bf16* vp = cell + (size_t)krow * ldq + (H + Hkv + kvh) * DH + half * 8;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      kf[ks] = *(const bf16x8*)(kp + ks * 16);
      vf[ks] = *(const bf16x8*)(vp + ks * 16);
    }
  }

  const int qt_first = kb * (DKV_WAVES / 2);       // first 64-row query tile that can see these keys
  const int nq = Tp / 64 - qt_first;               // query tiles per head
  const int iters = group * nq;
  const int R = lane >> 3, pc = lane & 7;
  auto issue_tile = [&](int it, int buf) {
    typedef const __attribute__((address_space(1))) void* gptr_t;
    typedef __attribute__((address_space(3))) void* lptr_t;
    const int head = kvh * group + it / nq, q0 = (qt_first + it % nq) * 64;
    unsigned char* base = smem + buf * STAGE;
    const char* qrows = (const char*)(cell + head * DH);
    const char* grows = (const char*)(gcell + head * DH);
    const char* qcols = (const char*)(Qt + (size_t)(l * H + head) * DH * Tp);
    const char* gcols = (const char*)(dOt + (size_t)(l * H + head) * DH * Tp);
    for (int sl = wave; sl < 4 * Q_SLABS; sl += DKV_WAVES) {
      const int which = sl / Q_SLABS, s2 = sl - which * Q_SLABS;
      const char* src;
      if (which < 2) {           // rows of Q / dO: DH / 64 sub-tiles [64 rows][64 dims]
        const int sub = s2 >> 3, row = (s2 & 7) * 8 + R;
        const int q = min(q0 + row, Trows - 1);
        src = (which == 0 ? qrows + (size_t)q * ldq * 2 : grows + (size_t)q * ldo * 2) + (sub * 64 + ((pc ^ mf_swz(row)) << 3)) * 2;
      } else {                   // columns: [DH dims][64 rows of the sequence]
        const int row = s2 * 8 + R;
        src = (which == 2 ? qcols : gcols) + ((size_t)row * Tp + q0 + ((pc ^ mf_swz(row)) << 3)) * 2;
      }
      __builtin_amdgcn_global_load_lds((gptr_t)src, (lptr_t)(base + sl * 1024), 16, 0, 0);
    }
    if (wave < 2) {              // lse (wave 0) and D (wave 1) of the 64 rows, also as direct loads: a load through
      const float* srcf = (wave == 0 ? LSE2 : Dv) + ((size_t)l * H + head) * Trows + min(q0 + lane, Trows - 1);   // registers
      __builtin_amdgcn_global_load_lds((gptr_t)srcf, (lptr_t)(base + 4 * Q_BYTES + wave * 256), 4, 0, 0);         // would make the
    }                            // wave wait for the whole prefetch before it starts on the current tile
  };

  const int fl = mf_swz(lane & 31);
  f32x16 dk[OT], dv[OT];
#pragma unroll
  for (int t = 0; t < OT; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) dk[t][r] = dv[t][r] = 0.f;

  issue_tile(0, 0);
  __builtin_amdgcn_s_waitcnt(0x0F70);
  __syncthreads();

  for (int it = 0; it < iters; ++it) {
    const int cur = it & 1, q0 = (qt_first + it % nq) * 64;
    if (it + 1 < iters) issue_tile(it + 1, cur ^ 1);
    const unsigned char* Qs = smem + cur * STAGE;
    const unsigned char* Gs = Qs + Q_BYTES;
    const unsigned char* QTs = Qs + 2 * Q_BYTES;
    const unsigned char* GTs = Qs + 3 * Q_BYTES;
    const float* sL = (const float*)(Qs + 4 * Q_BYTES);
    const float* sD = sL + 64;
    if (k0 <= q0 + 63 && k0 < Trows) {             // wave-uniform: some query of the tile can see some key of this wave
#pragma unroll
      for (int jj = 0; jj < 2; ++jj) {
        if (q0 + jj * 32 + 31 < k0) continue;      // this half of the tile lies before the keys
        f32x16 s, dp;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = dp[r] = 0.f;
        const int roff = (jj * 32 + (lane & 31)) * MF_ROW_BYTES;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          const int off = roff + (ks >> 2) * (64 * MF_ROW_BYTES) + (((2 * (ks & 3) + half) ^ fl) << 4);
          s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const bf16x8*)(Qs + off), kf[ks], s, 0, 0, 0);
          dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const bf16x8*)(Gs + off), vf[ks], dp, 0, 0, 0);
        }
        bf16x8 pf[2], dsf[2];
        // all 32 queries of this half exist and lie at or after all 32 keys of the wave: nothing to mask
        const bool interior = q0 + jj * 32 >= k0 + 31 && q0 + jj * 32 + 31 < Trows;
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) {         // registers 4 rg .. 4 rg + 3 hold four consecutive query rows
          const int j4 = jj * 32 + 8 * rg + 4 * half;
          const f32x4 l4 = *(const f32x4*)(sL + j4), d4 = *(const f32x4*)(sD + j4);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int r = 4 * rg + e, q = q0 + j4 + e;
            const bool live = interior || (q < Trows && ki <= q);
            const float p = live ? __builtin_amdgcn_exp2f(fmaf(s[r], scale_log2e, -l4[e])) : 0.f;
            pf[r >> 3][r & 7] = (bf16)p;
            dsf[r >> 3][r & 7] = (bf16)(p * (dp[r] - d4[e]) * scale);
          }
        }
        // dV^T[dim][key] += dO^T[dim][query] P[query][key],  dK^T[dim][key] += Q^T[dim][query] dS[query][key]
#pragma unroll
        for (int t = 0; t < OT; ++t) {
          const int toff = (t * 32 + (lane & 31)) * MF_ROW_BYTES + 8 * half;
#pragma unroll
          for (int ss = 0; ss < 2; ++ss) {
            const int ch = jj * 4 + 2 * ss;
            const int o0 = toff + ((ch ^ fl) << 4), o1 = toff + (((ch + 1) ^ fl) << 4);
            const bf16x4 glo = *(const bf16x4*)(GTs + o0), ghi = *(const bf16x4*)(GTs + o1);
            const bf16x4 qlo = *(const bf16x4*)(QTs + o0), qhi = *(const bf16x4*)(QTs + o1);
            bf16x8 ga, qa;
            ga[0] = glo[0]; ga[1] = glo[1]; ga[2] = glo[2]; ga[3] = glo[3]; ga[4] = ghi[0]; ga[5] = ghi[1]; ga[6] = ghi[2]; ga[7] = ghi[3];
            qa[0] = qlo[0]; qa[1] = qlo[1]; qa[2] = qlo[2]; qa[3] = qlo[3]; qa[4] = qhi[0]; qa[5] = qhi[1]; qa[6] = qhi[2]; qa[7] = qhi[3];
            dv[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ga, pf[ss], dv[t], 0, 0, 0);
            dk[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa, dsf[ss], dk[t], 0, 0, 0);
          }
        }
      }
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
  }

  if (ki < Trows) {
    bf16* dkp = dQKV + ((size_t)l * Trows + ki) * ldq + (H + kvh) * DH;
    bf16* dvp = dQKV + ((size_t)l * Trows + ki) * ldq + (H + Hkv + kvh) * DH;
#pragma unroll
    for (int t = 0; t < OT; ++t)
#pragma unroll
      for (int rg = 0; rg < 4; ++rg) {
        bf16x4 a, b;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          a[e] = (bf16)dk[t][4 * rg + e];
          b[e] = (bf16)dv[t][4 * rg + e];
        }
        *(bf16x4*)(dkp + t * 32 + 8 * rg + 4 * half) = a;
        *(bf16x4*)(dvp + t * 32 + 8 * rg + 4 * half) = b;
      }
  }
}

// bytes of the transposed operands for g cells: K^T [Hkv], Q^T [H], dO^T [H], each [dh][Tp]
inline size_t attention_bwd_scratch_bytes(int g, int Trows, int H, int Hkv, int dh) {
  return (size_t)g * (2 * H + Hkv) * dh * attention_tp(Trows) * 2;
}

// QKV (rotated q, k; v), O, dO as in the kernels above; LSE2 from the forward kernel; scratch as sized above.
inline hipError_t launch_attention_bwd_mfma(const bf16* QKV, const bf16* O, const bf16* dO, const float* LSE2, float* Dv,
                                            bf16* scratch, bf16* dQKV, int first, int g, int Lcells, int Trows, int H, int Hkv,
                                            int dh, hipStream_t st) {
  const int Tp = attention_tp(Trows), group = H / Hkv, ldq = (H + 2 * Hkv) * dh;
  bf16* Kt = scratch;
  bf16* Qt = Kt + (size_t)Lcells * Hkv * dh * Tp;
  bf16* Gt = Qt + (size_t)Lcells * H * dh * Tp;
  const size_t lds_t = 64 * (dh + 2) * 2;
  head_transpose_kernel<<<dim3(Tp / 64, Hkv, g), 256, lds_t, st>>>(QKV, ldq, H * dh, Kt, first, Trows, Tp, Hkv, dh);
  head_transpose_kernel<<<dim3(Tp / 64, H, g), 256, lds_t, st>>>(QKV, ldq, 0, Qt, first, Trows, Tp, H, dh);
  head_transpose_kernel<<<dim3(Tp / 64, H, g), 256, lds_t, st>>>(dO, H * dh, 0, Gt, first, Trows, Tp, H, dh);
  attention_dvec_kernel<<<dim3((Trows + 3) / 4, g), 256, 0, st>>>(O, dO, Dv, first, Trows, H, dh);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const float scale = 1.0f / sqrtf((float)dh);
  const int nq = group == 1 ? 4 : (group == 2 ? 2 : 1);       // row tiles per dQ workgroup, as in the forward kernel
  const int nqt = (Trows + 32 * nq - 1) / (32 * nq), nkb = (Trows + 32 * DKV_WAVES - 1) / (32 * DKV_WAVES), npairs = Hkv * g;
  const dim3 grid(8 * ((npairs + 7) / 8) * nqt), gkv(8 * ((npairs + 7) / 8) * nkb);
  if (dh == 64) {
    attention_bwd_dq_kernel<64><<<grid, nq * group * 64, 2 * 3 * (64 * 64 * 2), st>>>(QKV, Kt, dO, LSE2, Dv, dQKV, first, Trows, Tp, H, Hkv,
                                                                                   nq, scale, nqt, npairs);
    attention_bwd_dkv_kernel<64><<<gkv, 64 * DKV_WAVES, 2 * (4 * 64 * 64 * 2 + 512), st>>>(QKV, Qt, dO, Gt, LSE2, Dv, dQKV, first, Trows, Tp, H, Hkv,
                                                                              scale, npairs);
  } else {
    hipError_t a = hipFuncSetAttribute((const void*)attention_bwd_dq_kernel<128>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       2 * 3 * (64 * 128 * 2));
    if (a != hipSuccess) return a;
    attention_bwd_dq_kernel<128><<<grid, nq * group * 64, 2 * 3 * (64 * 128 * 2), st>>>(QKV, Kt, dO, LSE2, Dv, dQKV, first, Trows, Tp, H,
                                                                                     Hkv, nq, scale, nqt, npairs);
    a = hipFuncSetAttribute((const void*)attention_bwd_dkv_kernel<128>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            2 * (4 * 64 * 128 * 2 + 512));
    if (a != hipSuccess) return a;
    attention_bwd_dkv_kernel<128><<<gkv, 64 * DKV_WAVES, 2 * (4 * 64 * 128 * 2 + 512), st>>>(QKV, Qt, dO, Gt, LSE2, Dv, dQKV, first, Trows, Tp, H,
                                                                                Hkv, scale, npairs);
  }
  return hipGetLastError();
}

}  // namespace armt
