// Grouped bf16 GEMM on the CDNA4 matrix cores (paper Section 3.3 item 1, Section 4.1).
//
//   C_g = A_g B_g^T for every group g of the launch; A_g [M, K] activations, B_g [N, K] the
//   weights of the group's own layer (taken from a pointer table, never stacked), fp32
//   accumulation in v_mfma_f32_16x16x32_bf16, epilogue fused (residual add, row scale,
//   SwiGLU, bf16 copy and sums of squares for the next RMSNorm, rotary embedding and transposed
//   V for the QKV projection).
//
// Tiling: one workgroup per BM x BN output tile, BK = 64.  Both operands are K-contiguous, so a
// tile row is 128 bytes = eight 16-byte chunks; chunks are XOR-swizzled inside a row so that the
// MFMA fragment reads (one row per lane, 16 bytes) spread over all LDS banks.  Tiles are double
// buffered in LDS (NS = 2 stages; more are possible for small tiles) and filled by direct
// global-to-LDS loads (no staging registers): the copies of k-tile i+1 are in flight while k-tile i
// is multiplied.  For regular shapes (template flag REG) the copies are addressed by a scalar base
// and one lane offset per operand, so that issuing them needs no vector-ALU instruction.
// The 1-D grid is laid out so that each XCD (workgroup id mod 8) owns a contiguous run of the
// group-major tile sequence: with 16 groups every XCD streams the weights of 2 layers through its
// own L2, and the M-tiles sharing a weight panel run back to back.
// Template parameters of the kernel: BM x BN tile, WGM x WGN waves, REG (see above), EPI (GemmEpilogue),
// TAIL (see below), NS (LDS stages).  The launcher picks the configuration from the shape and the number of tiles of
// the launch (mfma_pick_config).
#pragma once

#include <atomic>
#include <type_traits>

#include "common.h"
#include "gemm_generic.h"

namespace armt {

constexpr int MF_BK = 64;                 // k-tile (bf16 elements): 128 bytes per tile row
constexpr int MF_ROW_BYTES = MF_BK * 2;
constexpr int MF_CUS = 256;            // compute units of the chip: a round of one tile per unit
constexpr int MF_NUM_CONFIGS = 7;         // tile configuration numbers of launch_gemm_mfma_epi lie below this

// swizzle of the 16-byte chunk index inside a 128-byte tile row; depends on row bits 0..3 only
__device__ __forceinline__ int mf_swz(int row) { return ((row >> 1) & 7) ^ ((row & 1) << 2); }

template <int N>
__device__ __forceinline__ void mf_wait_vmcnt() {      // s_waitcnt vmcnt(N) only (N <= 63)
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0F70);
}

#ifdef ARMT_GEMM_TIMELINE
// Probe build (paper_2506_05229_amd.build.build_timeline, never the product library): one armed launch records, per
// workgroup, where its time goes: [0] hardware id, [1] / [6] wall clock (100 MHz) at start / end, [2] .. [5] shader
// clock at start, after the first k-tile has landed, after the main loop, after the epilogue.
__device__ unsigned long long armt_timeline[8 * 65536];
inline int g_tl_kind = -2, g_tl_countdown = -1;      // host: the n-th next launch of this kind is the armed one
#define TL_STAMP(i)                                                     \
  do {                                                                  \
    if (tl_on && threadIdx.x == 0) tl[i] = __builtin_readcyclecounter(); \
  } while (0)
#else
#define TL_STAMP(i) do {} while (0)
#endif

// LDS bytes of the tile buffers of a configuration: NS buffers of a k-tile (A rows, B rows), and at least the two fp32
// staging tiles [WGM * 16][tile columns + 4] of the epilogue, which reuse them.
template <int BM, int BN, int WGM, int EPI, bool TAIL, int NS>
constexpr int mfma_tile_lds_bytes() {
  const int tiles = NS * ((TAIL ? BM + 16 : BM) + BN) * MF_ROW_BYTES;
  const int stg = 2 * WGM * 16 * (((EPI == EPI_SWIGLU) ? BN / 2 : BN) + 4) * 4;
  return ((tiles > stg ? tiles : stg) + 255) / 256 * 256;
}

// TAIL: the last M-tile of every group also owns the 16 rows that follow it (M = tiles_m * BM + 16).  With
// T = seg_len + 16 memory rows and seg_len a multiple of BM this removes the nearly empty fifth tile a
// 1040-row cell would otherwise need: the 16 memory rows ride along as one extra strip of 16x16x32 MFMAs.
template <int BM, int BN, int WGM, int WGN, bool REG, int EPI, bool TAIL, int NS>
__global__ __launch_bounds__(WGM* WGN * 64) void gemm_mfma_kernel(const GemmGroup* __restrict__ table, int first,
                                                                  GemmShape s, int tiles_m, int tiles_n,
                                                                  int total_tiles, int tile_begin) {
  constexpr int NW = WGM * WGN, BK = MF_BK;
  constexpr int WROWS = BM / WGM, WCOLS = BN / WGN;       // wave tile
  constexpr int TM = WROWS / 16, TN = WCOLS / 16;         // 16x16 MFMA tiles per wave
  constexpr int ROWB = BK * 2;                            // bytes of a tile row
  constexpr int RPS = 1024 / ROWB;                        // rows of a 1 KB slab (one copy instruction)
  constexpr int A_DMA = BM / RPS / NW, B_DMA = BN / RPS / NW;   // slabs each wave copies per k-tile
  constexpr int TAIL_SLABS = 16 / RPS;                    // slabs of the 16 tail rows, copied by the first waves
  constexpr int A_ROWS = TAIL ? BM + 16 : BM;
  constexpr int A_BYTES = A_ROWS * ROWB, B_BYTES = BN * ROWB;
  constexpr int BN_OUT = (EPI == EPI_SWIGLU) ? BN / 2 : BN;   // output columns per tile
  static_assert(BM % (WGM * 32) == 0 && BN % (WGN * 32) == 0, "wave tile must be a multiple of 32x32");
  static_assert(EPI != EPI_SWIGLU || WCOLS % 64 == 0, "SwiGLU: a wave owns whole gate/up pairs of 32-row weight blocks");
  static_assert(BM % (RPS * NW) == 0 && BN % (RPS * NW) == 0, "tile rows must divide into slabs per wave");
  static_assert(!TAIL || (BN <= NW * 32 && NW >= 2), "the tail strip gives each of the first BN / 32 waves two 16-column tiles");

  extern __shared__ __align__(16) unsigned char smem[];   // [NS][A_BYTES], [NS][B_BYTES], then A_ROWS row scales

#ifdef ARMT_GEMM_TIMELINE
  const bool tl_on = (s.dbg >> 20) & 1;
  unsigned long long* tl = armt_timeline + 8 * (size_t)(blockIdx.x & 65535);
  if (tl_on && threadIdx.x == 0) {
    unsigned hw, xcc;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID)" : "=s"(hw));
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
    tl[0] = ((unsigned long long)xcc << 32) | hw;
    tl[1] = __builtin_amdgcn_s_memrealtime();
    tl[2] = __builtin_readcyclecounter();
  }
#endif
  // XCD-aware tile order: workgroup b runs on XCD b % 8; give each XCD a contiguous range.  The launch covers the
  // total_tiles tiles from tile_begin on of the order (group, N-tile, M-tile).
  const int per_xcd = (total_tiles + 7) >> 3;
  const int lid0 = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (lid0 >= total_tiles) return;
  const int lid = tile_begin + lid0;
  const int per_group = tiles_m * tiles_n;
  const int grp = lid / per_group, rem = lid - grp * per_group;
  const int tn = rem / tiles_m, tm = rem - tn * tiles_m;    // M-tiles of one weight panel are adjacent
  const GemmGroup g = table[first + grp];
  const int m0 = tm * BM, n0 = tn * BN_OUT;
  const bool tail_blk = TAIL && (tm == tiles_m - 1);        // block-uniform

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // per-row scale of the result (1 / rms of a fused RMSNorm, or 1 / denominator of the associative read),
  // fetched once; visible to everybody after the first barrier of the main loop
  float* rs_lds = (float*)(smem + mfma_tile_lds_bytes<BM, BN, WGM, EPI, TAIL, NS>());
  for (int r = tid; r < A_ROWS; r += NW * 64) rs_lds[r] = (g.rowscale && m0 + r < s.M) ? g.rowscale[m0 + r] : 1.f;
  const int wm = wave / WGN, wn = wave % WGN;
  const bool tail = tail_blk && wave < (TAIL ? BN / 32 : 0);   // wave-uniform: this wave computes part of the strip

  // ---- global -> LDS copies go straight to LDS (global_load_lds_dwordx4): one instruction moves 64 x 16
  // bytes into 1 KB of consecutive LDS = 8 tile rows.  Lane i fills row i / 8, physical chunk i % 8 of the
  // slab, so it fetches the logical chunk (i % 8) ^ swz(row) of that row from global memory.
  // first element of row `row` of this block's weight tile
  // row n of the logical [N, K] weight, which comes in up to three blocks (selected by value: the table entry must not
  // be indexed dynamically, or it ends up in scratch memory instead of scalar registers)
  const bf16 *wB0 = (const bf16*)g.B0, *wB1 = (const bf16*)g.B1, *wB2 = (const bf16*)g.B2;
  auto w_row = [&](int n) -> const bf16* {
    if (n < s.n0) return wB0 + (size_t)n * s.ldb;
    n -= s.n0;
    if (n < s.n1) return wB1 + (size_t)n * s.ldb;
    return wB2 + (size_t)(n - s.n1) * s.ldb;
  };
  auto b_row = [&](int row) -> const bf16* {
    if (EPI == EPI_SWIGLU) {
      // tile rows come in 32-row blocks: even blocks from the gate weight, odd from the up weight,
      // both for output columns n0 + (block / 2) * 32 ...
      const int blk = row >> 5;
      const int n = min(n0 + (blk >> 1) * 32 + (row & 31), s.N - 1);
      return (const bf16*)((blk & 1) ? g.B1 : g.B0) + (size_t)n * s.ldb;
    }
    return w_row(min(n0 + row, s.N - 1));
  };
  const int dR = lane >> 3, dpc = lane & 7;
  // source of this lane for A slab j / the tail slab / B slab j, at k = 0
  auto a_src = [&](int j) -> const char* {
    const int row = (wave + j * NW) * 8 + dR;
    const int m = min(m0 + row, s.M - 1);                  // rows past M re-read the last row; masked on store
    return (const char*)g.A + ((size_t)m * s.lda + ((dpc ^ mf_swz(row)) << 3)) * 2;
  };
  auto t_src = [&]() -> const char* {                      // tail rows: copying waves 0 and 1 move one extra slab each
    const int row = BM + (wave & 1) * 8 + dR;
    const int m = min(m0 + row, s.M - 1);
    return (const char*)g.A + ((size_t)m * s.lda + ((dpc ^ mf_swz(row)) << 3)) * 2;
  };
  auto b_src = [&](int j) -> const char* {
    const int row = (wave + j * NW) * 8 + dR;
    return (const char*)(b_row(row) + ((dpc ^ mf_swz(row)) << 3));
  };
  // Two ways to address the sources.
  // General shapes: every lane keeps one 64-bit pointer per slab (rows past M or N are clamped per lane).
  // Regular shapes (REG: no ragged M or N, weight blocks that end on tile boundaries): all sources of a lane
  // differ by wave-uniform amounts, because the swizzle of row 8 * slab + lane / 8 depends on the slab's parity
  // only and a wave's slabs wave + NW * j all have the parity of the wave.  One 32-bit lane offset per operand
  // plus a scalar base per slab then address everything, and issuing a copy takes scalar instructions only.
  // That matters: a wave's vector-ALU instructions are not issued while other waves keep the SIMD's
  // matrix core busy with back-to-back MFMAs, scalar and memory instructions are.  Address arithmetic in the
  // vector ALU would hold the copies back until the multiplying waves pause.
  constexpr bool KEEP_PTRS = !REG;
  static_assert(!REG || NW % 2 == 0, "slabs of a wave must share their parity");
  const char* ap[KEEP_PTRS ? A_DMA : 1];
  const char* bp[KEEP_PTRS ? B_DMA : 1];
  const char* tp = nullptr;
  unsigned a_off0 = 0, b_off0 = 0;
  if (KEEP_PTRS) {
#pragma unroll
    for (int j = 0; j < (KEEP_PTRS ? A_DMA : 0); ++j) ap[j] = a_src(j);
    if (TAIL) tp = t_src();
#pragma unroll
    for (int j = 0; j < (KEEP_PTRS ? B_DMA : 0); ++j) bp[j] = b_src(j);
  } else {
    // lane i fills row i / 8, physical chunk i % 8 of its slab
    const int chunk = (dpc ^ mf_swz((wave & 1) * 8 + dR)) << 4;
    a_off0 = (unsigned)dR * (unsigned)s.lda * 2u + chunk;
    b_off0 = (unsigned)dR * (unsigned)s.ldb * 2u + chunk;
  }
  // scalar source of the first row of slab `slab` (REG only)
  auto a_base = [&](int slab) -> const char* { return (const char*)g.A + (size_t)(m0 + RPS * slab) * s.lda * 2; };
  auto b_base = [&](int slab) -> const char* {
    if (EPI == EPI_SWIGLU) {   // tile rows 32 * blk ..: blk even from the gate, odd from the up weight, columns n0 + 32 * (blk / 2) ..
      const int row = slab * RPS, blk = row >> 5;
      const int n = n0 + (blk >> 1) * 32 + (row & 31);
      return (const char*)((blk & 1) ? g.B1 : g.B0) + (size_t)n * s.ldb * 2;
    }
    return (const char*)w_row(n0 + RPS * slab);
  };
  const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) void*)smem;
  // one copy: 64 lanes x 16 bytes from base + lane offset to LDS address `lds` (M0) onwards; scalar operands only
  auto dma = [&](const char* base, unsigned voff, unsigned lds) {
    asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(voff), "s"(base), "s"(lds) : "memory", "m0");
  };
  // the same copy from one 64-bit pointer per lane.  Written as an instruction like the one above: the compiler then
  // does not count it among the outstanding memory operations, so the fence of a barrier does not wait for the
  // copies of the younger k-tiles that are meant to stay in flight (the waits for the copies are explicit, below)
  auto dma_ptr = [&](const char* src, unsigned lds) {
    asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(src), "s"(lds) : "memory", "m0");
  };
  auto issue_tile = [&](int kt, int buf) {
    const size_t ka = (size_t)kt * ROWB, kb = ka;
    if (KEEP_PTRS) {
      const unsigned ldsA = lds0 + buf * A_BYTES, ldsB = lds0 + NS * A_BYTES + buf * B_BYTES;
#pragma unroll
      for (int j = 0; j < A_DMA; ++j)
        dma_ptr(ap[KEEP_PTRS ? j : 0] + ka, ldsA + (wave + j * NW) * 1024);
      if (TAIL && tail_blk && wave < 2)
        dma_ptr(tp + ka, ldsA + BM * MF_ROW_BYTES + wave * 1024);
#pragma unroll
      for (int j = 0; j < B_DMA; ++j)
        dma_ptr(bp[KEEP_PTRS ? j : 0] + kb, ldsB + (wave + j * NW) * 1024);
    } else {
      const unsigned As = lds0 + buf * A_BYTES, Bs = lds0 + NS * A_BYTES + buf * B_BYTES;
#pragma unroll
      for (int j = 0; j < A_DMA; ++j) dma(a_base(wave + j * NW) + ka, a_off0, As + (wave + j * NW) * 1024);
      if (TAIL && tail_blk && wave < TAIL_SLABS) dma(a_base(BM / RPS + wave) + ka, a_off0, As + BM * ROWB + wave * 1024);
#pragma unroll
      for (int j = 0; j < B_DMA; ++j) dma(b_base(wave + j * NW) + kb, b_off0, Bs + (wave + j * NW) * 1024);
    }
  };

  // ---- MFMA fragment addresses (v_mfma_f32_16x16x32_bf16: under random operands this instruction sustains
  // 1.9 PFLOP/s on the chip against 1.35 for the 32x32x16 form, which draws more power per flop; measured with
  // register-only loops): lane reads tile row (lane % 16) of each 16-row block, 16-byte chunk 4 * ks2 + lane / 16
  // of the 128-byte row; a 16x16 result tile has lane = column lane % 16 and registers = rows 4 * (lane / 16) + r.
  constexpr int KS2 = BK / 32;                 // MFMA k-steps per k-tile
  const int t_sw = mf_swz(lane & 15), t_q = lane >> 4;
  int koff[KS2];
#pragma unroll
  for (int ks2 = 0; ks2 < KS2; ++ks2) koff[ks2] = ((4 * ks2 + t_q) ^ t_sw) << 4;
  const int a_frag = (wm * WROWS + (lane & 15)) * ROWB;
  const int b_frag = (wn * WCOLS + (lane & 15)) * ROWB;
  // tail strip: the same instruction on the 16 extra rows.  Wave w owns two 16-column
  // tiles whose B rows lie 32 apart, so that for SwiGLU tile 0 is the gate and tile 1 the up projection of the
  // same 16 output columns: B tile rows ((w / 2) * 2 + t) * 32 + (w % 2) * 16 + lane % 16.
  const int t_a = (BM + (lane & 15)) * ROWB;
  const int t_brow = ((wave >> 1) * 2) * 32 + (wave & 1) * 16 + (lane & 15);
  const int t_b = t_brow * ROWB;

  f32x4 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
  f32x4 tacc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};

  {
    // main loop: NS tile buffers; the copies of k-tiles kt+1 .. kt+NS-1 are in flight while k-tile kt is
    // multiplied (copies complete in issue order, so waiting for tile kt+1 leaves the younger ones outstanding);
    // one barrier per k-tile
    constexpr int CNT = A_DMA + B_DMA;                 // copy instructions per wave and tile (+1 on the tail waves)
    const bool extra = TAIL && tail_blk && wave < TAIL_SLABS;
    const int nk = s.K / BK;
#pragma unroll
    for (int p = 0; p < NS - 1; ++p)
      if (p < nk) issue_tile(p, p);
    if (NS > 2 && nk > NS - 2) {
      if (extra) mf_wait_vmcnt<(NS - 2) * (CNT + 1)>(); else mf_wait_vmcnt<(NS - 2) * CNT>();
    } else {
      mf_wait_vmcnt<0>();
    }
    __syncthreads();
    TL_STAMP(3);
    int cur = 0, nxt = NS - 1;                           // buffers of tile kt and of tile kt + NS - 1
    for (int kt = 0; kt < nk; ++kt) {
      // buffer nxt was last read in iteration kt - 1, which ended with a barrier
      if (kt + NS - 1 < nk) issue_tile(kt + NS - 1, nxt);
      const unsigned char* As = smem + cur * A_BYTES;
      const unsigned char* Bs = smem + NS * A_BYTES + cur * B_BYTES;
#pragma unroll
      for (int ks2 = 0; ks2 < KS2; ++ks2) {
        bf16x8 af[TM], bfr[TN];
#pragma unroll
        for (int i = 0; i < TM; ++i) af[i] = *(const bf16x8*)(As + a_frag + i * 16 * ROWB + koff[ks2]);
#pragma unroll
        for (int j = 0; j < TN; ++j) bfr[j] = *(const bf16x8*)(Bs + b_frag + j * 16 * ROWB + koff[ks2]);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
      }
      if (TAIL && tail) {
#pragma unroll
        for (int ks2 = 0; ks2 < KS2; ++ks2) {
          const int ko = koff[ks2];
          const bf16x8 ta = *(const bf16x8*)(As + t_a + ko);
#pragma unroll
          for (int t = 0; t < 2; ++t) {
            const bf16x8 tb = *(const bf16x8*)(Bs + t_b + t * 32 * ROWB + ko);
            tacc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ta, tb, tacc[t], 0, 0, 0);
          }
        }
      }
      // tile kt+1 must have landed; tiles kt+2 .. kt+NS-1 (if they were issued) may stay in flight
      if (NS > 2 && kt + NS - 1 < nk) {
        if (extra) mf_wait_vmcnt<(NS - 2) * (CNT + 1)>(); else mf_wait_vmcnt<(NS - 2) * CNT>();
      } else {
        mf_wait_vmcnt<0>();
      }
      __syncthreads();
      cur = (cur + 1 == NS) ? 0 : cur + 1;
      nxt = (nxt + 1 == NS) ? 0 : nxt + 1;
    }
  }

  TL_STAMP(4);
  // ---- epilogue, staged through LDS so that global memory sees whole rows: a 16x16 result tile has lane =
  // column (lane % 16) and registers = rows 4 * (lane / 16) + r, which written directly would touch global
  // memory in 32- or 64-byte pieces.  Instead, in TM passes every wave drops one 16-row block of its tile into
  // a fp32 staging tile [WGM * 16][BN_OUT + 4] (the +4 puts the four row groups of a wave on different banks),
  // and all threads then walk the staging tile row-major, C4 = BN_OUT / 4 lanes per row: 16-byte accesses, full rows
  // of R, C, C2.  The tail strip goes through the same path as one more pass of 16 rows.
  // There are two staging tiles (the tile buffers are free: the main loop ended with a barrier): pass p + 1 is staged
  // while pass p is still being drained, so a pass costs one barrier, and nothing of it waits for global memory
  // between the barriers: what a pass reads from global memory (residual rows, rotary table) is requested before its
  // staging writes, and the barriers wait for LDS traffic only.
  constexpr int SLD = BN_OUT + 4, SR = WGM * 16, C4 = BN_OUT / 4, NT = NW * 64;
  constexpr int STG_FLOATS = SR * SLD;
  static_assert(2 * STG_FLOATS * 4 <= mfma_tile_lds_bytes<BM, BN, WGM, EPI, TAIL, NS>(), "two staging tiles must fit in the tile buffers");
  static_assert(C4 == 16 || C4 == 32 || C4 == 64, "a staged row is handled by 16, 32 or 64 consecutive lanes");
  static_assert(NT % C4 == 0, "a thread keeps its columns from one row of the walk to the next");
  const bool vec_ok = ((s.N | s.ldc | s.ldr | s.ldc2) & 3) == 0;
  // silu(gate) * up; the reciprocal is the hardware's (1 ulp), the result is rounded to bf16 afterwards
  auto silu_mul = [](float gt, float up) { return gt * __builtin_amdgcn_rcpf(1.f + __expf(-gt)) * up; };
  auto row_scale = [&](int m) { return rs_lds[m - m0]; };
  // EPI_DPFP_READ: feature idx = lane + 64 k of phi(q) = r[i] r[(i - j) mod 2 d_mem], r = [relu(q), relu(-q)], j = 1..nu
  // (the untrained feature map of Section 2.1) is max(sa q[ia], 0) max(sb q[ib], 0); which columns and signs, and the
  // lane's entries of z, are the same for every row: set up once per thread
  constexpr int DP_MAXK = (EPI == EPI_DPFP_READ) ? 8 : 1;      // 2 nu d_mem <= 512 features
  int dp_ia[DP_MAXK], dp_ib[DP_MAXK], dp_phi = 0;
  float dp_sa[DP_MAXK], dp_sb[DP_MAXK], dp_z[DP_MAXK];
  if constexpr (EPI == EPI_DPFP_READ) {
    const int dm = s.n0, n2 = 2 * dm;
    dp_phi = s.ldr * n2;
#pragma unroll
    for (int k = 0; k < DP_MAXK; ++k) {
      const int idx = min(k * 64 + lane, dp_phi - 1);
      const int j = idx / n2 + 1, i = idx - (j - 1) * n2;
      int i2 = i - j;
      if (i2 < 0) i2 += n2;
      dp_ia[k] = i < dm ? i : i - dm;   dp_sa[k] = i < dm ? 1.f : -1.f;
      dp_ib[k] = i2 < dm ? i2 : i2 - dm; dp_sb[k] = i2 < dm ? 1.f : -1.f;
      dp_z[k] = g.R[idx];
    }
  }
  // The walk: thread tid takes column group c4 = tid % C4 (4 columns) of the staged rows tid / C4 + it * (NT / C4).
  const int c4 = tid % C4, sr_first = tid / C4;
  const int n = n0 + c4 * 4;
  // per-thread constants of the walk: the gain of its four columns (EPI_RESID_F32 with a normalised copy)
  f32x4 gq = {1.f, 1.f, 1.f, 1.f};
  if (EPI == EPI_RESID_F32 && g.C2 && g.gain) {
#pragma unroll
    for (int e = 0; e < 4; ++e) gq[e] = (float)((const bf16*)g.gain)[min(n + e, s.N - 1)];
  }
  // sum over the 32 lanes that hold 128 consecutive columns of a row: four steps inside a row of 16 lanes with
  // data-parallel moves (no LDS), one exchange between the two rows
  auto sum32 = [](float v) __attribute__((always_inline)) {
    auto dpp = [](float x, auto ctrl) {
      return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), decltype(ctrl)::value, 0xF, 0xF, true));
    };
    v += dpp(v, std::integral_constant<int, 0xB1>{});      // quad_perm [1, 0, 3, 2]
    v += dpp(v, std::integral_constant<int, 0x4E>{});      // quad_perm [2, 3, 0, 1]
    v += dpp(v, std::integral_constant<int, 0x141>{});     // row_half_mirror
    v += dpp(v, std::integral_constant<int, 0x140>{});     // row_mirror
    v += __builtin_bit_cast(float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, v), 0x401F));   // lane ^ 16
    return v;
  };
  // What one pass of the walk reads from global memory, requested ahead of the pass.
  constexpr int MAX_ITER = (SR * C4 + NT - 1) / NT;
  struct Pre { f32x4 r[MAX_ITER]; };
  auto prefetch = [&](auto nrows_c, auto m_of, Pre& pre) __attribute__((always_inline)) {
    constexpr int NROWS = decltype(nrows_c)::value, ITER = (NROWS * C4 + NT - 1) / NT;
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
      const int sr = sr_first + it * (NT / C4);
      const int m = m_of(min(sr, NROWS - 1));
      const bool valid = sr < NROWS && m < s.M && n < s.N;
      pre.r[it] = f32x4{0.f, 0.f, 0.f, 0.f};
      if (EPI == EPI_RESID_F32 && g.R && valid) {
        if (vec_ok) {
          pre.r[it] = *(const f32x4*)(g.R + (size_t)m * s.ldr + n);
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (n + e < s.N) pre.r[it][e] = g.R[(size_t)m * s.ldr + n + e];
        }
      }
    }
  };
  // walk NROWS staged rows of staging tile stg; staged row sr is output row m_of(sr)
  auto drain = [&](const float* stg, auto nrows_c, auto m_of, const Pre& pre) __attribute__((always_inline)) {
    constexpr int NROWS = decltype(nrows_c)::value, ITER = (NROWS * C4 + NT - 1) / NT;
    if constexpr (EPI == EPI_DPFP_READ) {
      // One wave per staged row: the row's d_mem values q sit in the staging tile; lane L computes the features
      // L, L + 64, ... of phi(q) (dp_* above), stores them in the activation type and adds up its share of z . phi(q).
      // The summation order (lane-strided partial sums, then the wave reduction) does not depend on the tile
      // configuration, so every configuration produces the same bits.
      // A wave takes the staged rows wave, wave + NW, ...: all of them side by side (features of every row first, then the
      // row sums, then the stores), so that the LDS reads and the wave reductions of different rows overlap.
      constexpr int RW = (NROWS + NW - 1) / NW;           // rows per wave
      float f[RW][DP_MAXK], den[RW];
      int mrow[RW];
#pragma unroll
      for (int j = 0; j < RW; ++j) {
        const int sr = min(wave + j * NW, NROWS - 1);
        mrow[j] = (wave + j * NW < NROWS) ? m_of(sr) : s.M;      // rows past the tile or past M are skipped below
        const float* q = stg + sr * SLD;
        den[j] = 0.f;
#pragma unroll
        for (int k = 0; k < DP_MAXK; ++k) {
          f[j][k] = fmaxf(dp_sa[k] * q[dp_ia[k]], 0.f) * fmaxf(dp_sb[k] * q[dp_ib[k]], 0.f);
          if (k * 64 + lane < dp_phi) den[j] = fmaf(f[j][k], dp_z[k], den[j]);
        }
      }
#pragma unroll
      for (int off = 32; off > 0; off >>= 1)
#pragma unroll
        for (int j = 0; j < RW; ++j) den[j] += __shfl_xor(den[j], off, kWave);
#pragma unroll
      for (int j = 0; j < RW; ++j) {
        if (mrow[j] >= s.M) continue;                    // wave-uniform
        bf16* frow = (bf16*)g.C + (size_t)mrow[j] * s.ldc + lane;
#pragma unroll
        for (int k = 0; k < DP_MAXK; ++k)
          if (k * 64 + lane < dp_phi) frow[k * 64] = (bf16)f[j][k];
        if (lane == 0) ((float*)g.C2)[mrow[j]] = 1.0f / (den[j] + s.fparam);
      }
      return;
    }
    // EPI_QKV_ROPE: the cos / sin pairs of all rows of the walk first (stores to C could alias the table as far as
    // the compiler knows, so loads placed between the stores would wait for one another)
    f32x4 rc0[EPI == EPI_QKV_ROPE ? ITER : 1], rc1[EPI == EPI_QKV_ROPE ? ITER : 1];
    if constexpr (EPI == EPI_QKV_ROPE) {
      const int hd = s.ldr >> 1, j = n % s.ldr;
#pragma unroll
      for (int it = 0; it < ITER; ++it) {
        const int sr = sr_first + it * (NT / C4);
        const int m = m_of(min(sr, NROWS - 1));
        rc0[it] = rc1[it] = f32x4{1.f, 0.f, 1.f, 0.f};
        if (sr < NROWS && m < s.M && n < s.n0 + s.n1 && n < s.N) {
          const float* cs = g.R + 2 * ((size_t)m * hd + (j - (j < hd ? 0 : hd)));
          rc0[it] = *(const f32x4*)cs;                   // c0 s0 c1 s1 | c2 s2 c3 s3
          rc1[it] = *(const f32x4*)(cs + 4);
        }
      }
    }
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
      const int sr = sr_first + it * (NT / C4);
      const int m = m_of(min(sr, NROWS - 1));
      const bool valid = sr < NROWS && m < s.M && n < s.N;
      f32x4 o = {0.f, 0.f, 0.f, 0.f};
      if (valid) {
        o = *(const f32x4*)(stg + sr * SLD + c4 * 4);
        if (EPI != EPI_SWIGLU) o *= row_scale(m);        // SwiGLU applied it before the nonlinearity
        if constexpr (EPI == EPI_QKV_ROPE) {
          if (n < s.n0 + s.n1) {
            // rotary embedding (rotate-half): column j of a head pairs with j +- dh/2, which lies in the same
            // staged row; out_j = x_j cos_j' - x_{j+h} sin_j' (j < h), x_j cos_j' + x_{j-h} sin_j' (j >= h), j' = j mod h
            const int dh = s.ldr, hd = dh >> 1, j = n % dh, lo = j < hd;
            const f32x4 p = *(const f32x4*)(stg + sr * SLD + c4 * 4 + (lo ? hd : -hd)) * row_scale(m);
            const f32x4 cs0 = rc0[it], cs1 = rc1[it];
            const float sg = lo ? -1.f : 1.f;
            o[0] = o[0] * cs0[0] + sg * p[0] * cs0[1];
            o[1] = o[1] * cs0[2] + sg * p[1] * cs0[3];
            o[2] = o[2] * cs1[0] + sg * p[2] * cs1[1];
            o[3] = o[3] * cs1[2] + sg * p[3] * cs1[3];
          }
        }
        if (EPI == EPI_RESID_F32) o += pre.r[it];        // zeros without a residual
        if (!vec_ok) {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (n + e >= s.N) o[e] = 0.f;
        }
        bf16x4 ob, og;
#pragma unroll
        for (int e = 0; e < 4; ++e) ob[e] = (bf16)o[e];
        if (EPI == EPI_RESID_F32 && g.C2) {
          // with a gain the copy is the un-normalised input of the next RMSNorm: x * gain
#pragma unroll
          for (int e = 0; e < 4; ++e) og[e] = g.gain ? (bf16)(o[e] * gq[e]) : ob[e];
        }
        if (vec_ok) {
          if (EPI == EPI_STORE_ACT || EPI == EPI_SWIGLU || EPI == EPI_QKV_ROPE) {
            *(bf16x4*)((bf16*)g.C + (size_t)m * s.ldc + n) = ob;
          } else {
            *(f32x4*)((float*)g.C + (size_t)m * s.ldc + n) = o;
            if (EPI == EPI_RESID_F32 && g.C2) *(bf16x4*)((bf16*)g.C2 + (size_t)m * s.ldc2 + n) = og;
          }
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            if (n + e >= s.N) continue;
            if (EPI == EPI_STORE_ACT || EPI == EPI_SWIGLU || EPI == EPI_QKV_ROPE) {
              ((bf16*)g.C)[(size_t)m * s.ldc + n + e] = ob[e];
            } else {
              ((float*)g.C)[(size_t)m * s.ldc + n + e] = o[e];
              if (EPI == EPI_RESID_F32 && g.C2) ((bf16*)g.C2)[(size_t)m * s.ldc2 + n + e] = og[e];
            }
          }
        }
      }
      if (EPI == EPI_RESID_F32 && g.ssq_out) {
        // sum of squares of this row for the RMSNorm that consumes the row: one partial per (row, 128 columns),
        // summed later in column order (deterministic, no atomics).  The granularity and the order of the additions
        // are fixed, not tied to the tile width, so that every tile configuration produces the same partials bit for bit.
        static_assert(EPI != EPI_RESID_F32 || BN_OUT % 128 == 0, "partials cover 128 columns = 32 lanes");
        const float part = sum32(o[0] * o[0] + o[1] * o[1] + o[2] * o[2] + o[3] * o[3]);
        if ((c4 & 31) == 0 && sr < NROWS && m < s.M)
          g.ssq_out[(size_t)m * ((s.N + 127) >> 7) + tn * (BN_OUT / 128) + (c4 >> 5)] = part;
      }
    }
  };
  // EPI_QKV_ROPE, tiles of the v columns: the attention kernel wants V transposed ([column][row], row stride ldc2),
  // so these tiles are drained column-wise: a thread takes 8 consecutive rows of one column, 16 bytes per store.
  const bool vt_tile = EPI == EPI_QKV_ROPE && s.ldc2 > 0 && n0 >= s.n0 + s.n1;      // block-uniform
  auto drain_vt = [&](const float* stg, int nrows, auto m_of) __attribute__((always_inline)) {
    bf16* vt = (bf16*)g.C2 + (size_t)(n0 - (s.n0 + s.n1)) * s.ldc2;
    for (int u = tid; u < (nrows >> 3) * BN_OUT; u += NT) {
      const int rg = u / BN_OUT, col = u - rg * BN_OUT;
      const int m = m_of(rg * 8);          // rows rg * 8 .. + 7 of the staging tile are consecutive output rows
      if (m >= s.M || n0 + col >= s.N) continue;
      bf16x8 v;
#pragma unroll
      for (int i = 0; i < 8; ++i)
        v[i] = (m + i < s.M) ? (bf16)(stg[(rg * 8 + i) * SLD + col] * rs_lds[m + i - m0]) : (bf16)0.f;
      *(bf16x8*)(vt + (size_t)col * s.ldc2 + m) = v;
    }
  };
  const int col_in = lane & 15;
  Pre pre;
#pragma unroll
  for (int pass = 0; pass < TM; ++pass) {
    const int i = pass;
    float* stg = (float*)smem + (pass & 1) * STG_FLOATS;
    auto pass_row = [&](int sr) { return m0 + (sr >> 4) * WROWS + i * 16 + (sr & 15); };
    if (EPI == EPI_RESID_F32) prefetch(std::integral_constant<int, SR>{}, pass_row, pre);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int row16 = 4 * t_q + r;
      float* dst = stg + (wm * 16 + row16) * SLD + col_in;
      if (EPI == EPI_SWIGLU) {
        // the wave's weight rows come in 32-row blocks, gate / up alternating: tiles 4q + h (gate) and 4q + 2 + h
        // (up), h = 0, 1, give output columns (wn * WCOLS / 64 + q) * 32 + h * 16 + lane % 16
        const float rs = row_scale(m0 + wm * WROWS + i * 16 + row16);
#pragma unroll
        for (int j = 0; j < TN; ++j)
          if ((j & 2) == 0)
            dst[(wn * (WCOLS / 64) + (j >> 2)) * 32 + (j & 1) * 16] = silu_mul(rs * acc[i][j][r], rs * acc[i][j + 2][r]);
      } else {
#pragma unroll
        for (int j = 0; j < TN; ++j) dst[wn * WCOLS + j * 16] = acc[i][j][r];
      }
    }
    __syncthreads();         // pass p is staged; everybody has left the walk of pass p - 1, whose tile pass p + 1 reuses
    if (vt_tile) drain_vt(stg, SR, pass_row);
    else drain(stg, std::integral_constant<int, SR>{}, pass_row, pre);
  }
  if (TAIL && tail_blk) {     // 16x16 result tile: lane holds column lane % 16, rows 4*(lane/16) + r
    float* stg = (float*)smem + (TM & 1) * STG_FLOATS;
    auto tail_row = [&](int sr) { return m0 + BM + sr; };
    if (EPI == EPI_RESID_F32) prefetch(std::integral_constant<int, 16>{}, tail_row, pre);
    if (tail) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        float* dst = stg + (4 * t_q + r) * SLD;
        if (EPI == EPI_SWIGLU) {
          const float rs = row_scale(m0 + BM + 4 * t_q + r);
          dst[(wave >> 1) * 32 + (wave & 1) * 16 + (lane & 15)] = silu_mul(rs * tacc[0][r], rs * tacc[1][r]);
        } else {
          dst[t_brow] = tacc[0][r];
          dst[t_brow + 32] = tacc[1][r];
        }
      }
    }
    __syncthreads();
    if (vt_tile) drain_vt(stg, 16, tail_row);
    else drain(stg, std::integral_constant<int, 16>{}, tail_row, pre);
  }
#ifdef ARMT_GEMM_TIMELINE
  if (tl_on && threadIdx.x == 0) { tl[5] = __builtin_readcyclecounter(); tl[6] = __builtin_amdgcn_s_memrealtime(); }
#endif
}

// Part of a launch's work, so that two tile sizes can share it: weight panels [begin, end) counted over the groups in
// units of unit_cols output columns (units_per_group = N / unit_cols of them per group).  unit_cols = 0: everything.
struct TileRange { int unit_cols = 0, units_per_group = 0, begin = 0, end = 0; };

template <int BM, int BN, int WGM, int WGN, bool REG, int EPI, bool TAIL, int NS>
inline hipError_t launch_mfma_tail(const GemmGroup* table, int first, int g, const GemmShape& s, hipStream_t st,
                                   const TileRange& rng) {
  constexpr int BN_OUT = (EPI == EPI_SWIGLU) ? BN / 2 : BN;
  constexpr int LDS = mfma_tile_lds_bytes<BM, BN, WGM, EPI, TAIL, NS>() + (BM + 16) * 4;
  const int tiles_m = TAIL ? s.M / BM : (s.M + BM - 1) / BM, tiles_n = (s.N + BN_OUT - 1) / BN_OUT;
  const int all = g * tiles_m * tiles_n;
  // a part of the launch's tiles, in units of whole weight panels (tiles_m M-tiles each) of this tile size
  int begin = 0, total = all;
  if (rng.unit_cols > 0) {
    const int per_group = tiles_m * tiles_n, scale = rng.unit_cols / BN_OUT;    // this configuration's N-tiles per unit
    const auto at = [&](int u) { return (u / rng.units_per_group) * per_group + (u % rng.units_per_group) * scale * tiles_m; };
    begin = at(rng.begin);
    total = (rng.end >= g * rng.units_per_group ? all : at(rng.end)) - begin;
  }
  if (total <= 0) return hipSuccess;
  const int grid = ((total + 7) / 8) * 8;
  auto kern = gemm_mfma_kernel<BM, BN, WGM, WGN, REG, EPI, TAIL, NS>;
  // raising the dynamic-LDS limit is a per-function, per-device, idempotent setting: done once per device (a second
  // thread that gets here first merely repeats it)
  static std::atomic<uint64_t> attr_set{0};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const uint64_t bit = 1ull << (dev & 63);
  if (!(attr_set.load(std::memory_order_acquire) & bit)) {
    e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
    if (e != hipSuccess) return e;
    attr_set.fetch_or(bit, std::memory_order_release);
  }
#ifdef ARMT_GEMM_TIMELINE
  if (s.tag == g_tl_kind && g_tl_countdown >= 0 && g_tl_countdown-- == 0) {
    GemmShape s_tl = s;
    s_tl.dbg |= 1 << 20;
    kern<<<grid, WGM * WGN * 64, LDS, st>>>(table, first, s_tl, tiles_m, tiles_n, total, begin);
    return hipGetLastError();
  }
#endif
  kern<<<grid, WGM * WGN * 64, LDS, st>>>(table, first, s, tiles_m, tiles_n, total, begin);
  return hipGetLastError();
}

// M = tiles * BM + 16 (a cell: seg_len rows + 16 memory rows) takes the tail variant.
// shapes the copy-wave variant addresses with one lane offset per operand
template <int BM, int BN, int EPI>
inline bool mfma_regular_shape(const GemmShape& s) {
  constexpr int BN_OUT = (EPI == EPI_SWIGLU) ? BN / 2 : BN;
  const bool m_ok = s.M % BM == 0 || (s.M > BM && s.M % BM == 16 && !(s.dbg & 32)) || s.a_rows >= (s.M + BM - 1) / BM * BM;
  const int e0 = s.n0, e1 = s.n0 + s.n1;      // ends of weight blocks 0 and 1
  const bool w_ok = EPI == EPI_SWIGLU || ((e0 >= s.N || e0 % BN == 0) && (e1 >= s.N || e1 % BN == 0));
  return m_ok && s.N % BN_OUT == 0 && w_ok && s.K % MF_BK == 0;
}

template <int BM, int BN, int WGM, int WGN, int EPI, bool REG = false, int NS = 2>
inline hipError_t launch_mfma_cfg(const GemmGroup* table, int first, int g, const GemmShape& s, hipStream_t st,
                                  const TileRange& rng = TileRange()) {
  if constexpr (BN <= WGM * WGN * 32) {
    if (s.M > BM && s.M % BM == 16 && !(s.dbg & 32))
      return launch_mfma_tail<BM, BN, WGM, WGN, REG, EPI, true, NS>(table, first, g, s, st, rng);
  }
  return launch_mfma_tail<BM, BN, WGM, WGN, REG, EPI, false, NS>(table, first, g, s, st, rng);
}

// Big tiles move the fewest bytes per flop, but a launch needs about one tile per CU to use the chip: a single
// cell (sequential order, or the first and last steps of the diagonal order) has too few 256x256 tiles.
inline int mfma_pick_config(const GemmShape& s, int g, int force_cfg) {
  if (force_cfg >= 0 && force_cfg < MF_NUM_CONFIGS) return force_cfg;
  // a few rows against wide weights (W_K | W_V on the memory rows): the launch streams the weights once and is bound
  // by how many bytes a CU has in flight, so narrow tiles that give every CU two workgroups
  if (s.M <= 64 && s.epi == EPI_STORE_F32 && (long)g * ((s.N + 127) / 128) < 512) return 3;
  // W_Q of the read with the feature map as its epilogue: one d_mem-wide tile column, so the workgroups are the M-tiles;
  // 32-row tiles put two or more workgroups on a CU, whose waves then fill each other's waits
  if (s.epi == EPI_DPFP_READ && s.M >= 64 && (long)g * ((s.M + 63) / 64) < 1024) return 4;
  if (s.M < 96 || s.N < 96) return 2;
  const int tm = (s.M > 256 && s.M % 256 == 16) ? s.M / 256 : (s.M + 255) / 256;
  const int bn_out = (s.epi == EPI_SWIGLU) ? 128 : 256;
  const long tiles = (long)g * tm * ((s.N + bn_out - 1) / bn_out);
  // measured crossover (1040-row cells, N = 768 ... 3072, K = 768 ... 8192): 128x128 tiles win up to 128 tiles of
  // 256x256 (they still fit the chip in one round of two workgroups per CU), 256x256 tiles from 144 on
  return (s.M >= 192 && s.N >= 192 && tiles >= 136) ? 5 : 6;
}

// Tile configuration by problem shape: big square tiles for the block's linears, small tiles for
// the skinny associative-memory projections (N = d_mem columns, or M = n_mem rows).
template <int EPI>
inline hipError_t launch_gemm_mfma_epi(const GemmGroup* table, int first, int g, const GemmShape& s, hipStream_t st,
                                       int force_cfg) {
  const int cfg = mfma_pick_config(s, g, force_cfg);
  switch (cfg) {
    case 1: return launch_mfma_cfg<128, 128, 2, 2, EPI>(table, first, g, s, st);
    case 3:   // 64 x 64: only instantiated for the plain fp32 store
      // four k-tiles in LDS: the loop of these small tiles is bound by the latency of a copy, not by its arithmetic
      if constexpr (EPI == EPI_STORE_F32) return launch_mfma_cfg<64, 64, 2, 2, EPI, false, 4>(table, first, g, s, st);
      break;
    case 4:   // 32 x 128, waves side by side: only instantiated for the feature-map epilogue of the W_Q projection
      // three k-tiles in LDS (two workgroups still fit on a CU)
      if constexpr (EPI == EPI_DPFP_READ) return launch_mfma_cfg<32, 128, 1, 4, EPI, false, 3>(table, first, g, s, st);
      break;
    case 5:   // 256 x 256, 16 waves, copies addressed by scalar base + lane offset where the shape allows
      if (mfma_regular_shape<256, 256, EPI>(s)) {
        if constexpr (EPI != EPI_SWIGLU) {
          // Whole rounds of the chip with 256 x 256 tiles; if what is left fills at most half of another round, it runs
          // as 128 x 128 tiles (four times as many, two workgroups per CU: one short round instead of a long one
          // that leaves most CUs idle).  Both tile sizes give the same bits (same order of the k-steps, row sums
          // of squares at a fixed granularity), so where the cut falls does not show in the result.
          const int tm = (s.M > 256 && s.M % 256 == 16) ? s.M / 256 : (s.M + 255) / 256, upg = s.N / 256;
          const long tiles = (long)g * tm * upg;
          const int rest_units = (int)((tiles % MF_CUS + tm - 1) / tm);   // weight panels of the last, partial round (rounded up)
          const int units = g * upg;
          if (force_cfg < 0 && tiles > MF_CUS && tiles % MF_CUS != 0 && tiles % MF_CUS <= MF_CUS / 2 && rest_units > 0 &&
              mfma_regular_shape<128, 128, EPI>(s)) {
            TileRange big, rest;
            big.unit_cols = rest.unit_cols = 256;
            big.units_per_group = rest.units_per_group = upg;
            big.begin = 0; big.end = rest.begin = units - rest_units; rest.end = units;
            hipError_t e = launch_mfma_cfg<256, 256, 4, 4, EPI, true>(table, first, g, s, st, big);
            if (e != hipSuccess) return e;
            return launch_mfma_cfg<128, 128, 2, 2, EPI, true>(table, first, g, s, st, rest);
          }
        }
        return launch_mfma_cfg<256, 256, 4, 4, EPI, true>(table, first, g, s, st);
      }
      return launch_mfma_cfg<256, 256, 4, 4, EPI>(table, first, g, s, st);
    case 6:   // as 1, copies addressed by scalar base + lane offset where the shape allows
      if (mfma_regular_shape<128, 128, EPI>(s)) return launch_mfma_cfg<128, 128, 2, 2, EPI, true>(table, first, g, s, st);
      return launch_mfma_cfg<128, 128, 2, 2, EPI>(table, first, g, s, st);
    default: break;
  }
  return launch_mfma_cfg<64, 128, 2, 2, EPI>(table, first, g, s, st);
}

inline hipError_t launch_gemm_mfma(const GemmGroup* table, int first, int g, const GemmShape& s, hipStream_t st,
                                   int force_cfg = -1) {
  if (g <= 0 || s.M <= 0 || s.N <= 0) return hipSuccess;
  switch (s.epi) {
    case EPI_STORE_ACT: return launch_gemm_mfma_epi<EPI_STORE_ACT>(table, first, g, s, st, force_cfg);
    case EPI_STORE_F32: return launch_gemm_mfma_epi<EPI_STORE_F32>(table, first, g, s, st, force_cfg);
    case EPI_RESID_F32: return launch_gemm_mfma_epi<EPI_RESID_F32>(table, first, g, s, st, force_cfg);
    case EPI_SWIGLU: return launch_gemm_mfma_epi<EPI_SWIGLU>(table, first, g, s, st, force_cfg);
    case EPI_DPFP_READ:
      // all d_mem columns of a row in one output tile (the narrowest tile is 128 wide)
      if (s.N != s.n0 || s.N > 128 || s.ldr < 1 || s.ldc < 2 * s.ldr * s.n0 || 2 * s.ldr * s.n0 > 512) return hipErrorInvalidValue;
      return launch_gemm_mfma_epi<EPI_DPFP_READ>(table, first, g, s, st, force_cfg);
    case EPI_QKV_ROPE:
      // the rotation reads its partner column from the staged tile: heads must not straddle tiles (128 or 256 wide)
      if (s.ldr <= 0 || 128 % s.ldr != 0 || (s.N & 3) || (s.ldc & 3)) return hipErrorInvalidValue;
      return launch_gemm_mfma_epi<EPI_QKV_ROPE>(table, first, g, s, st, force_cfg);
  }
  return hipErrorInvalidValue;
}

}  // namespace armt
