// Host side of the ARMT forward library: argument checks, workspace carving, the per-layer
// pointer tables ("per-group weight pointers"), the cell / anti-diagonal scheduler and the
// kernel sequence of one step.  Everything here is plain C++ around HIP launches; the C ABI
// is declared in include/armt.h.
#include "../../include/armt.h"

#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <string>
#include <type_traits>
#include <vector>

#include "attention_generic.h"
#include "attention_bwd_mfma.h"
#include "attention_mfma.h"
#include "backward_kernels.h"
#include "common.h"
#include "gemm_generic.h"
#include "gemm_mfma.h"
#include "rowwise_kernels.h"
#include "token_ends.h"

using namespace armt;

namespace {

thread_local std::string g_hip_error;

#define HIP_TRY(expr)                                                                      \
  do {                                                                                     \
    hipError_t e_ = (expr);                                                                \
    if (e_ != hipSuccess) {                                                                \
      g_hip_error = std::string(#expr) + ": " + hipGetErrorString(e_);                     \
      return ARMT_ERR_HIP;                                                                 \
    }                                                                                      \
  } while (0)

#define ARMT_TRY(expr)                 \
  do {                                 \
    armt_status s_ = (expr);           \
    if (s_ != ARMT_OK) return s_;      \
  } while (0)

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

struct Dims {
  // L counts the cells that can be live in one step: n_layers * batch ("virtual layers": index v = layer * B + b;
  // all per-layer scratch, tables and kernels are indexed by v).  Lr = n_layers, B = batch (1 outside the batched calls).
  int L, Lr, B, d, H, Hkv, dh, F, S, m, T, dm, nu, Phi, Nqkv;
  bool bf16;
  float rms_eps, rope_theta, assoc_eps;
  size_t esz;   // bytes of one activation / weight element
};

armt_status check_config(const armt_config* c, Dims* out) {
  if (!c) return ARMT_ERR_NULL;
  if (c->dtype != ARMT_F32 && c->dtype != ARMT_BF16) return ARMT_ERR_DTYPE;
  if (c->n_layers < 1 || c->d_model < 1 || c->n_heads < 1 || c->n_kv_heads < 1 || c->head_dim < 2 ||
      c->d_ff < 1 || c->seg_len < 1 || c->n_mem < 1 || c->d_mem < 1 || c->dpfp_nu < 1)
    return ARMT_ERR_SHAPE;
  if (c->n_heads % c->n_kv_heads != 0 || (c->head_dim & 1) || (int64_t)c->n_heads * c->head_dim != c->d_model)
    return ARMT_ERR_SHAPE;
  if (c->dpfp_nu >= 2 * c->d_mem) return ARMT_ERR_SHAPE;
  if (!(c->rms_eps >= 0.f) || !(c->rope_theta > 0.f) || !(c->assoc_eps >= 0.f)) return ARMT_ERR_SHAPE;
  Dims D;
  D.L = D.Lr = c->n_layers; D.B = 1; D.d = c->d_model; D.H = c->n_heads; D.Hkv = c->n_kv_heads; D.dh = c->head_dim;
  D.F = c->d_ff; D.S = c->seg_len; D.m = c->n_mem; D.T = D.S + D.m; D.dm = c->d_mem; D.nu = c->dpfp_nu;
  D.Phi = 2 * D.nu * D.dm; D.Nqkv = (D.H + 2 * D.Hkv) * D.dh;
  D.bf16 = (c->dtype == ARMT_BF16);
  D.rms_eps = c->rms_eps; D.rope_theta = c->rope_theta; D.assoc_eps = c->assoc_eps;
  D.esz = D.bf16 ? 2 : 4;
  if (D.Phi > 512) return ARMT_ERR_UNSUPPORTED;          // the delta-rule kernel keeps a row of A in registers
  if (D.bf16) {
    // the MFMA GEMM takes k-tiles of 64 and 16-byte rows
    if (D.d % 64 || D.F % 64 || D.Phi % 64 || D.dm % 8 || D.m % 16) return ARMT_ERR_UNSUPPORTED;
    // the MFMA attention kernel: head_dim 64 or 128, one wave per query head of a KV group
    if ((D.dh != 64 && D.dh != 128) || D.H / D.Hkv > 8) return ARMT_ERR_UNSUPPORTED;
  }
  if (out) *out = D;
  return ARMT_OK;
}

// GEMM kinds of one step, in launch order; each has one table entry per layer.
enum Kind { K_MQ = 0, K_READ, K_QKV, K_O, K_GU, K_DOWN, K_MKV, K_COUNT };
// further kinds of armt_profile_begin: kernels of the associative memory that are not GEMMs, and the attention kernel
enum ProfKind { PK_DPFP_READ = K_COUNT, PK_UPD_PREP, PK_DELTA_RULE, PK_ATTENTION, PK_COUNT };

struct Layout {          // byte offsets into the workspace
  size_t X, Xb, Nrm, QKV, Vt, Att, Hres, Uff, Qm, Fphi, RDen, A16, KVm, Fm, Coef, Rope, Ssq, RStd, Tables, Aux, total;
};

// rows of a cell rounded up to whole tiles of the largest GEMM tile
inline size_t padded_rows(int T) { return ((size_t)T + 255) / 256 * 256; }

Layout carve(const Dims& D) {
  Layout o;
  size_t p = 0;
  auto take = [&](size_t bytes) { size_t at = p; p = align_up(p + bytes); return at; };
  const size_t L = D.L, T = D.T;
  // the bf16 GEMM operands end in `pad` rows nobody writes: the grouped GEMM may read whole 256-row tiles of them
  const size_t pad = D.bf16 ? padded_rows(D.T) - T : 0;
  o.X = take((L + D.B) * T * D.d * 4);                            // residual stream, slot v = input of cell v; output in v + B
  o.Xb = take(D.bf16 ? ((L + D.B) * T + pad) * D.d * 2 : 0);      // bf16 copy of the slots (GEMM operand)
  o.Nrm = take((L * T + pad) * D.d * D.esz);
  o.QKV = take(L * T * D.Nqkv * D.esz);
  o.Vt = take(D.bf16 ? attention_vt_bytes(D.L, D.T, D.Hkv, D.dh) : 0);   // V transposed, for the MFMA attention
  o.Att = take((L * T + pad) * D.d * D.esz);
  o.Hres = take(L * T * D.d * 4);
  o.Uff = take((L * T + pad) * D.F * D.esz);
  o.Qm = take(L * T * D.dm * 4);
  o.Fphi = take((L * T + pad) * D.Phi * D.esz);
  o.RDen = take(L * T * 4);
  o.A16 = take(D.bf16 ? L * (size_t)D.d * D.Phi * 2 : 0);
  o.KVm = take(L * D.m * (size_t)(D.dm + D.d) * 4);
  o.Fm = take(L * D.m * (size_t)D.Phi * 4);
  o.Coef = take(L * D.m * 4 * 4);
  o.Rope = take(T * (D.dh / 2) * 2 * 4);
  o.Ssq = take(D.bf16 ? L * T * (size_t)((D.d + 63) / 64) * 4 : 0);   // per-tile sums of squares (fused RMSNorm)
  o.RStd = take(D.bf16 ? L * T * 4 : 0);
  o.Tables = take((size_t)K_COUNT * L * sizeof(GemmGroup));
  o.Aux = take(L * sizeof(LayerAux));
  o.total = p;
  return o;
}

// ARMT_DEBUG_GENERIC=1 routes bf16 work through the plain fp32-FMA kernels (slow; for debugging only).
bool debug_generic() {
  static const bool v = [] { const char* e = getenv("ARMT_DEBUG_GENERIC"); return e && e[0] == '1'; }();
  return v;
}


int g_gemm_tile_config = -1;     // armt_set_gemm_tile_config
int g_gemm_dbg = 0;              // A/B switches of armt_set_gemm_tile_config (config / 100)

struct Ctx {
  Dims D;
  Layout o;
  char* ws;
  hipStream_t st;
  const GemmGroup* tables;   // device: [K_COUNT][L]
  const LayerAux* aux;       // device: [L]
  GemmShape shape[K_COUNT];
  bool fused_norm;           // bf16 MFMA path: RMSNorm folded into the GEMM epilogues around it
  bool fused_rope;           // bf16 MFMA path: rotary embedding applied by the QKV GEMM epilogue
  bool fused_vt;             // ... which also writes V transposed
  bool fused_dpfp;           // bf16 MFMA path: feature map and denominator of the read in the epilogue of the W_Q projection
  int ssq_parts;             // partial sums of squares per row written by the GEMMs that produce a normalised row
  float* tape = nullptr;     // training forward: per-cell records of what the backward pass cannot recompute
  size_t rec_floats = 0;     // floats per record
  template <typename T> T* at(size_t off) const { return (T*)(ws + off); }
  const GemmGroup* table(int kind) const { return tables + (size_t)kind * D.L; }
};

void fill_shapes(Ctx& c) {
  const Dims& D = c.D;
  auto set = [&](int k, int M, int N, int K, int lda, int ldc, int ldc2, int ldr, int n0, int n1, int epi) {
    GemmShape s;
    s.M = M; s.N = N; s.K = K; s.lda = lda; s.ldc = ldc; s.ldc2 = ldc2; s.ldr = ldr; s.n0 = n0; s.n1 = n1; s.epi = epi;
    s.tag = k;
    s.dbg = g_gemm_dbg;
    s.ldb = K;
    c.shape[k] = s;
  };
  set(K_MQ, D.T, D.dm, D.d, D.d, D.dm, 0, 0, D.dm, 0, EPI_STORE_F32);
  set(K_READ, D.T, D.d, D.Phi, D.Phi, D.d, 0, D.d, D.d, 0, EPI_RESID_F32);
  set(K_QKV, D.T, D.Nqkv, D.d, D.d, D.Nqkv, 0, 0, D.H * D.dh, D.Hkv * D.dh, EPI_STORE_ACT);
  set(K_O, D.T, D.d, D.H * D.dh, D.H * D.dh, D.d, 0, D.d, D.d, 0, EPI_RESID_F32);
  set(K_GU, D.T, D.F, D.d, D.d, D.F, 0, 0, D.F, D.F, EPI_SWIGLU);
  set(K_DOWN, D.T, D.d, D.F, D.F, D.d, D.d, D.d, D.d, 0, EPI_RESID_F32);
  set(K_MKV, D.m, D.dm + D.d, D.d, D.d, D.dm + D.d, 0, 0, D.dm, D.d, EPI_STORE_F32);
  if (D.bf16)      // A operands of the T-row GEMMs are workspace buffers that end in padding rows (carve)
    for (int k : {K_MQ, K_READ, K_QKV, K_O, K_GU, K_DOWN}) c.shape[k].a_rows = (int)padded_rows(D.T);
  c.fused_norm = D.bf16 && !debug_generic();
  // rotary embedding as the epilogue of the QKV GEMM: heads must not straddle its output tiles
  c.fused_rope = D.bf16 && !debug_generic() && 128 % D.dh == 0 && !(g_gemm_dbg & 128);
  if (c.fused_rope) { c.shape[K_QKV].epi = EPI_QKV_ROPE; c.shape[K_QKV].ldr = D.dh; }
  // ... and V written transposed for the attention kernel, if the v columns start on a tile boundary
  c.fused_vt = c.fused_rope && ((D.H + D.Hkv) * D.dh) % 256 == 0 && D.T % 8 == 0 && !(g_gemm_dbg & 64);
  if (c.fused_vt) c.shape[K_QKV].ldc2 = attention_tp(D.T);
  if (c.fused_norm) c.shape[K_READ].ldc2 = c.shape[K_O].ldc2 = D.d;
  // feature map + denominator of the read (Eq. 6) as the epilogue of the W_Q projection: q never goes to memory
  c.fused_dpfp = D.bf16 && !debug_generic() && D.dm <= 128 && !(g_gemm_dbg & 16);
  if (c.fused_dpfp) {
    GemmShape& q = c.shape[K_MQ];
    q.epi = EPI_DPFP_READ; q.ldc = D.Phi; q.ldr = D.nu; q.fparam = D.assoc_eps;
  }
  c.ssq_parts = (D.d + 127) / 128;   // the GEMM epilogue writes one partial sum of squares per 128 columns
}

// Small host tables (pointer tables of the grouped GEMMs and the like) reach the device as KERNEL ARGUMENTS, 3.5 KB per
// launch: the runtime copies the arguments when the launch is enqueued, so the host buffer may die right after the call,
// nothing waits for the stream, and the call can be recorded into a HIP graph (a host-to-device copy from pageable
// memory would need a synchronisation before the buffer is freed).
struct ArgChunk { uint32_t w[896]; };
__global__ __launch_bounds__(256) void arg_upload_kernel(ArgChunk c, uint32_t* __restrict__ dst, int n_words) {
  for (int i = threadIdx.x; i < n_words; i += 256) dst[i] = c.w[i];
}

armt_status upload_bytes(hipStream_t st, void* dst, const void* src, size_t bytes) {
  static_assert(sizeof(ArgChunk) + 16 <= 4096, "kernel arguments are limited to 4 KB");
  const size_t words = (bytes + 3) / 4;          // destinations are carved in multiples of 256 bytes
  ArgChunk c;
  for (size_t w0 = 0; w0 < words; w0 += 896) {
    const size_t n = std::min<size_t>(896, words - w0);
    const size_t nb = std::min(bytes - w0 * 4, n * 4);
    memset(&c, 0, sizeof(c));
    memcpy(c.w, (const char*)src + w0 * 4, nb);
    arg_upload_kernel<<<1, 256, 0, st>>>(c, (uint32_t*)dst + w0, (int)n);
  }
  HIP_TRY(hipGetLastError());
  return ARMT_OK;
}

// Build the per-layer pointer tables on the host and send them into the workspace.
armt_status upload_tables(Ctx& c, const armt_layer_weights* W, float* A, float* z) {
  const Dims& D = c.D;
  const size_t L = D.L, T = D.T;
  std::vector<GemmGroup> tab((size_t)K_COUNT * L);
  std::vector<LayerAux> aux(L);
  memset(tab.data(), 0, tab.size() * sizeof(GemmGroup));
  char* X = c.ws + c.o.X;
  char* Xop = D.bf16 ? c.ws + c.o.Xb : X;       // activation-typed view of the slots
  const size_t slotX = T * D.d * 4, slotXop = T * D.d * D.esz;
  const size_t B = D.B;
  for (size_t l = 0; l < L; ++l) {                 // l = virtual layer: real layer l / B of sequence l % B
    const armt_layer_weights& w = W[l / B];
    const size_t state = (l % B) * D.Lr + l / B;    // the caller's memory state is [B][n_layers][...]
    float* Al = A + state * (size_t)D.d * D.Phi;
    bf16* A16l = D.bf16 ? c.at<bf16>(c.o.A16) + state * (size_t)D.d * D.Phi : nullptr;
    GemmGroup* g;
    g = &tab[K_MQ * L + l];
    g->A = Xop + l * slotXop; g->B0 = w.wm_q; g->C = c.ws + c.o.Qm + l * T * D.dm * 4;
    if (c.fused_dpfp) {
      g->C = c.ws + c.o.Fphi + l * T * D.Phi * D.esz; g->C2 = c.ws + c.o.RDen + l * T * 4;
      g->R = z + state * (size_t)D.Phi;
    }
    g = &tab[K_READ * L + l];
    g->A = c.ws + c.o.Fphi + l * T * D.Phi * D.esz;
    g->B0 = D.bf16 ? (const void*)A16l : (const void*)Al;
    g->C = X + l * slotX; g->R = (const float*)(X + l * slotX);
    g->rowscale = (const float*)(c.ws + c.o.RDen + l * T * 4);
    void* nrm = c.ws + c.o.Nrm + l * T * D.d * D.esz;
    float* ssq = (float*)(c.ws + c.o.Ssq) + l * T * c.ssq_parts;
    const float* rstd = (const float*)(c.ws + c.o.RStd) + l * T;
    if (c.fused_norm) { g->C2 = nrm; g->gain = w.rms1; g->ssq_out = ssq; }   // input of the first norm
    g = &tab[K_QKV * L + l];
    g->A = nrm; g->B0 = w.wq; g->B1 = w.wk; g->B2 = w.wv;
    if (c.fused_rope) g->R = (const float*)(c.ws + c.o.Rope);
    if (c.fused_vt) g->C2 = c.ws + c.o.Vt + l * (size_t)D.Hkv * D.dh * attention_tp(D.T) * 2;
    g->C = c.ws + c.o.QKV + l * T * D.Nqkv * D.esz;
    if (c.fused_norm) g->rowscale = rstd;
    g = &tab[K_O * L + l];
    g->A = c.ws + c.o.Att + l * T * D.d * D.esz; g->B0 = w.wo;
    g->C = c.ws + c.o.Hres + l * T * D.d * 4; g->R = (const float*)(X + l * slotX);
    if (c.fused_norm) { g->C2 = nrm; g->gain = w.rms2; g->ssq_out = ssq; }   // input of the second norm
    g = &tab[K_GU * L + l];
    g->A = nrm; g->B0 = w.wgate; g->B1 = w.wup;
    g->C = c.ws + c.o.Uff + l * T * D.F * D.esz;
    if (c.fused_norm) g->rowscale = rstd;
    g = &tab[K_DOWN * L + l];
    g->A = c.ws + c.o.Uff + l * T * D.F * D.esz; g->B0 = w.wdown;
    g->C = X + (l + B) * slotX; g->C2 = D.bf16 ? Xop + (l + B) * slotXop : nullptr;
    g->R = (const float*)(c.ws + c.o.Hres + l * T * D.d * 4);
    g = &tab[K_MKV * L + l];
    g->A = Xop + (l + B) * slotXop + (size_t)D.S * D.d * D.esz; g->B0 = w.wm_k; g->B1 = w.wm_v;
    g->C = c.ws + c.o.KVm + l * D.m * (size_t)(D.dm + D.d) * 4;
    LayerAux& a = aux[l];
    a.rms1 = w.rms1; a.rms2 = w.rms2; a.wm_b = w.wm_b;
    a.A = Al; a.z = z + state * (size_t)D.Phi; a.A16 = A16l;
  }
  ARMT_TRY(upload_bytes(c.st, c.ws + c.o.Tables, tab.data(), tab.size() * sizeof(GemmGroup)));
  ARMT_TRY(upload_bytes(c.st, c.ws + c.o.Aux, aux.data(), aux.size() * sizeof(LayerAux)));
  c.tables = c.at<GemmGroup>(c.o.Tables);
  c.aux = c.at<LayerAux>(c.o.Aux);
  return ARMT_OK;
}

// Optional timing of one GEMM kind with HIP events on the launch stream (armt_profile_*).
struct Profile {
  int kind = -1;
  std::vector<hipEvent_t> ev;    // start/stop pairs
  size_t used = 0;               // events recorded so far
  int64_t groups = 0;            // groups (cells) covered by the recorded launches
} g_prof;

// Bracket the launches between prof_start and prof_stop with a pair of events if their kind is the one being timed.
inline bool prof_start(int tag, hipStream_t st) {
  if (g_prof.kind < 0 || g_prof.kind != tag || g_prof.used + 2 > g_prof.ev.size()) return false;
  return hipEventRecord(g_prof.ev[g_prof.used], st) == hipSuccess;
}
inline void prof_stop(bool timed, hipStream_t st, int g) {
  if (!timed) return;
  (void)hipEventRecord(g_prof.ev[g_prof.used + 1], st);
  g_prof.used += 2;
  g_prof.groups += g;
}

template <typename T>
armt_status gemm(hipStream_t st, const GemmGroup* table, int first, int g, const GemmShape& s) {
  if (g <= 0) return ARMT_OK;
  const bool timed = prof_start(s.tag, st);
  if (std::is_same<T, bf16>::value && !debug_generic()) {
    HIP_TRY(launch_gemm_mfma(table, first, g, s, st, g_gemm_tile_config));
  } else {
    HIP_TRY(launch_gemm_generic<T>(table, first, g, s, st));
  }
  prof_stop(timed, st, g);
  return ARMT_OK;
}

// ---- the three composite steps, shared by the forward path and the single-step entry points ----

// Associative read of cells [first, first + g): x <- x + A phi(W_Q x) / (z.phi(W_Q x) + eps)   (Eq. 6)
template <typename T>
armt_status step_assoc_read(hipStream_t st, const GemmGroup* t_mq, const GemmShape& s_mq, const GemmGroup* t_read,
                            const GemmShape& s_read, const LayerAux* aux, int first, int g, int Trows, int dm, int nu,
                            float eps, float* Qm, T* Fphi, float* RDen) {
  if (g <= 0) return ARMT_OK;
  ARMT_TRY(gemm<T>(st, t_mq, first, g, s_mq));
  if (s_mq.epi != EPI_DPFP_READ) {       // feature map and denominator not yet produced by the projection's epilogue
    const bool timed = prof_start(PK_DPFP_READ, st);
    dpfp_read_kernel<T><<<dim3(Trows, g), 128, (dm + 17) * 4, st>>>(Qm, aux, first, Trows, dm, nu, eps, Fphi, RDen);
    prof_stop(timed, st, g);
    HIP_TRY(hipGetLastError());
  }
  return gemm<T>(st, t_read, first, g, s_read);
}

// Rotary embedding of q, k and causal grouped-query attention over the rows of each cell.
template <typename T>
armt_status step_attention(hipStream_t st, T* QKV, T* Att, bf16* Vt, const float* rope_cs, int first, int g, int Trows,
                           int H, int Hkv, int dh, bool rotated, bool vt_ready) {
  if (g <= 0) return ARMT_OK;
  const int ldq = (H + 2 * Hkv) * dh;
  if (!rotated) {      // q and k not yet rotated by the producer of QKV
    rope_kernel<T><<<dim3(Trows, g), 256, 0, st>>>(QKV, rope_cs, first, Trows, H + Hkv, dh, ldq);
    HIP_TRY(hipGetLastError());
  }
  if (std::is_same<T, bf16>::value && !debug_generic()) {
    const bool timed = prof_start(PK_ATTENTION, st);
    HIP_TRY(launch_attention_mfma((const bf16*)QKV, Vt, (bf16*)Att, first, g, Trows, H, Hkv, dh, vt_ready, st));
    prof_stop(timed, st, g);
    return ARMT_OK;
  }
  attention_generic_kernel<T><<<dim3(Trows, H, g), 64, (dh + Trows) * 4, st>>>(QKV, Att, first, Trows, H, Hkv, dh,
                                                                              1.0f / sqrtf((float)dh));
  HIP_TRY(hipGetLastError());
  return ARMT_OK;
}

// Delta-rule update of the memories of cells [first, first + g) from their m memory-row outputs (Eq. 3-5).
template <typename T>
armt_status step_assoc_update(hipStream_t st, const GemmGroup* t_mkv, const GemmShape& s_mkv, const LayerAux* aux,
                              int first, int g, int empty_lo, int empty_hi, const T* Y0, size_t y_stride, int m, int d, int dm,
                              int nu, float eps, float* KVm, float* Fm, float* Coef) {
  if (g <= 0) return ARMT_OK;
  const int Phi = 2 * nu * dm;
  ARMT_TRY(gemm<T>(st, t_mkv, first, g, s_mkv));
  bool timed = prof_start(PK_UPD_PREP, st);
  memupd_prep_kernel<T><<<dim3(m, g), 128, (dm + 17) * 4, st>>>(KVm, Y0, y_stride, aux, first, empty_lo, empty_hi, m, d, dm, nu,
                                                               eps, Fm, Coef);
  prof_stop(timed, st, g);
  HIP_TRY(hipGetLastError());
  timed = prof_start(PK_DELTA_RULE, st);
  if (m == 16 && Phi % 64 == 0 && Phi <= 512) {
    const int rows_per_block = 32;
    const dim3 grid((d + rows_per_block - 1) / rows_per_block, g);
#define ARMT_DELTA16(NPL) \
  case NPL: delta_rule16_kernel<NPL><<<grid, 256, 0, st>>>(KVm, Fm, Coef, aux, first, d, dm, rows_per_block); break;
    switch (Phi / 64) {
      ARMT_DELTA16(1) ARMT_DELTA16(2) ARMT_DELTA16(3) ARMT_DELTA16(4) ARMT_DELTA16(5) ARMT_DELTA16(6) ARMT_DELTA16(7)
      ARMT_DELTA16(8)
    }
#undef ARMT_DELTA16
  } else if (m % 16 == 0 && Phi % 64 == 0 && Phi <= 512) {
    const dim3 grid((d + 4 * DRC_ROWS - 1) / (4 * DRC_ROWS), g);
#define ARMT_DELTA16C(NPL) \
  case NPL: delta_rule16c_kernel<NPL><<<grid, 256, 0, st>>>(KVm, Fm, Coef, aux, first, m, d, dm); break;
    switch (Phi / 64) {
      ARMT_DELTA16C(1) ARMT_DELTA16C(2) ARMT_DELTA16C(3) ARMT_DELTA16C(4) ARMT_DELTA16C(5) ARMT_DELTA16C(6) ARMT_DELTA16C(7)
      ARMT_DELTA16C(8)
    }
#undef ARMT_DELTA16C
  } else {
    const int rows_per_block = 4 * DR_ROWS;
    const size_t lds = (size_t)std::min(m, DR_CHUNK) * (Phi + 4) * 4;
    delta_rule_kernel<8><<<dim3((d + rows_per_block - 1) / rows_per_block, g), 256, lds, st>>>(KVm, Fm, Coef, aux, first,
                                                                                             m, d, dm, Phi);
  }
  prof_stop(timed, st, g);
  HIP_TRY(hipGetLastError());
  return ARMT_OK;
}

// One step: the cells of layers [lo, hi] (each on its own segment), as one group.
//   read_hi: highest layer whose memory is non-empty (the associative read applies to [lo, read_hi]);
//   empty_layer: the layer whose memory is still empty (v_bar = 0), or -1.
template <typename T>
armt_status run_group(const Ctx& c, int lo, int hi, int read_hi, int empty_layer) {
  const Dims& D = c.D;
  // real layers -> cells: layer l of the B sequences = cells l * B .. l * B + B - 1
  const int g = (hi - lo + 1) * D.B, gr = (read_hi - lo + 1) * D.B;
  const int e0 = empty_layer < 0 ? -1 : empty_layer * D.B, e1 = empty_layer < 0 ? -1 : e0 + D.B;
  lo *= D.B;
  float* X = c.at<float>(c.o.X);
  T* Xop = D.bf16 ? c.at<T>(c.o.Xb) : (T*)X;
  // (1) associative read
  ARMT_TRY(step_assoc_read<T>(c.st, c.table(K_MQ), c.shape[K_MQ], c.table(K_READ), c.shape[K_READ], c.aux, lo,
                              gr, D.T, D.dm, D.nu, D.assoc_eps, c.at<float>(c.o.Qm), c.at<T>(c.o.Fphi),
                              c.at<float>(c.o.RDen)));
  // (2) decoder block (TransformerLayer of Eq. 2).  On the bf16 path both RMSNorms are folded into the GEMMs
  // around them: the producer of a row (read GEMM, attention-output GEMM) also writes bf16(row * gain) and the
  // row's sum of squares per N-tile; the consumer GEMM multiplies its result rows by 1 / rms.
  float* rstd = c.at<float>(c.o.RStd);
  if (c.fused_norm) {
    if (gr > 0) {
      rstd_kernel<<<dim3((D.T + 255) / 256, gr), 256, 0, c.st>>>(c.at<float>(c.o.Ssq), lo, D.T, c.ssq_parts, D.d, D.rms_eps, rstd);
      HIP_TRY(hipGetLastError());
    }
    if (gr < g) {      // cells that met an empty memory had no read GEMM in front of the norm
      rmsnorm_kernel<T><<<dim3(D.T, g - gr), 256, 0, c.st>>>(X, c.aux, lo + gr, 0, D.T, D.d, D.rms_eps, c.at<T>(c.o.Nrm), rstd);
      HIP_TRY(hipGetLastError());
    }
  } else {
    rmsnorm_kernel<T><<<dim3(D.T, g), 256, 0, c.st>>>(X, c.aux, lo, 0, D.T, D.d, D.rms_eps, c.at<T>(c.o.Nrm), nullptr);
    HIP_TRY(hipGetLastError());
  }
  ARMT_TRY(gemm<T>(c.st, c.table(K_QKV), lo, g, c.shape[K_QKV]));
  ARMT_TRY(step_attention<T>(c.st, c.at<T>(c.o.QKV), c.at<T>(c.o.Att), c.at<bf16>(c.o.Vt), c.at<float>(c.o.Rope), lo, g,
                             D.T, D.H, D.Hkv, D.dh, c.fused_rope, c.fused_vt));
  ARMT_TRY(gemm<T>(c.st, c.table(K_O), lo, g, c.shape[K_O]));
  if (c.fused_norm) {
    rstd_kernel<<<dim3((D.T + 255) / 256, g), 256, 0, c.st>>>(c.at<float>(c.o.Ssq), lo, D.T, c.ssq_parts, D.d, D.rms_eps, rstd);
  } else {
    rmsnorm_kernel<T><<<dim3(D.T, g), 256, 0, c.st>>>(c.at<float>(c.o.Hres), c.aux, lo, 1, D.T, D.d, D.rms_eps,
                                                      c.at<T>(c.o.Nrm), nullptr);
  }
  HIP_TRY(hipGetLastError());
  ARMT_TRY(gemm<T>(c.st, c.table(K_GU), lo, g, c.shape[K_GU]));
  ARMT_TRY(gemm<T>(c.st, c.table(K_DOWN), lo, g, c.shape[K_DOWN]));
  // (3) memory update from the block's output at the memory rows
  const T* Y0 = Xop + ((size_t)D.B * D.T + D.S) * D.d;  // memory row 0 of slot B = output of cell 0
  return step_assoc_update<T>(c.st, c.table(K_MKV), c.shape[K_MKV], c.aux, lo, g, e0, e1, Y0, (size_t)D.T * D.d,
                              D.m, D.d, D.dm, D.nu, D.assoc_eps, c.at<float>(c.o.KVm), c.at<float>(c.o.Fm),
                              c.at<float>(c.o.Coef));
}

// Training forward: record the inputs of the cells of layers [lo, hi] (cell l belongs to segment t - l).
armt_status save_tape(const Ctx& c, int lo, int hi, int t) {
  if (!c.tape) return ARMT_OK;
  const Dims& D = c.D;
  const size_t nx = (size_t)D.T * D.d, nA = (size_t)D.d * D.Phi, nz = D.Phi;
  tape_kernel<<<dim3(128, (hi - lo + 1) * D.B), 256, 0, c.st>>>(c.tape, c.rec_floats, c.at<float>(c.o.X), nx, c.aux, nullptr, nullptr,
                                                              lo * D.B, t, D.L, D.B, nx, nA, nz, 1);
  HIP_TRY(hipGetLastError());
  return ARMT_OK;
}

template <typename T>
armt_status forward_typed(Ctx& c, const void* mem_emb, const void* x, int64_t N, bool carry_in, void* hidden_out,
                          bool diagonal, int split_upto) {
  const Dims& D = c.D;
  const int L = D.Lr;
  const size_t seq = (size_t)N * D.S * D.d;      // elements of one sequence of x / hidden_out
  float* X = c.at<float>(c.o.X);
  T* Xb = D.bf16 ? c.at<T>(c.o.Xb) : nullptr;
  {
    const int n = D.T * (D.dh / 2);
    rope_table_kernel<<<(n + 255) / 256, 256, 0, c.st>>>(c.at<float>(c.o.Rope), D.T, D.dh / 2, (double)D.rope_theta);
    HIP_TRY(hipGetLastError());
    if (c.fused_vt) {      // the QKV epilogue never writes the padding columns [T, Tp) of V^T, which must read as zero
      const size_t nf = attention_vt_bytes(D.L, D.T, D.Hkv, D.dh) / 4;
      fill_f32_kernel<<<(unsigned)((nf + 255) / 256), 256, 0, c.st>>>(c.at<float>(c.o.Vt), nf, 0.f);
      HIP_TRY(hipGetLastError());
    }
  }
  auto ingest = [&](int64_t s) -> armt_status {       // Algorithm 1: ingest a new segment at layer 0
    for (int b = 0; b < D.B; ++b) {                  // sequence b enters at cell b (layer 0)
      const size_t slot = (size_t)b * D.T * D.d;
      pack_segment_kernel<T><<<D.T, 256, 0, c.st>>>((const T*)x + b * seq + (size_t)s * D.S * D.d, (const T*)mem_emb, D.S, D.d,
                                                    X + slot, Xb ? Xb + slot : nullptr);
    }
    HIP_TRY(hipGetLastError());
    return ARMT_OK;
  };
  auto emit = [&](int64_t s) -> armt_status {         // segment s went through all layers
    for (int b = 0; b < D.B; ++b)                    // output of the last layer's cell of sequence b: slot L * B + b
      store_hidden_kernel<T><<<D.S, 256, 0, c.st>>>(X + (size_t)(D.L + b) * D.T * D.d, D.d,
                                                    (T*)hidden_out + b * seq + (size_t)s * D.S * D.d);
    HIP_TRY(hipGetLastError());
    return ARMT_OK;
  };
  if (!diagonal) {
    for (int64_t s = 0; s < N; ++s) {
      ARMT_TRY(ingest(s));
      const bool empty = (s == 0 && !carry_in);
      for (int l = 0; l < L; ++l) {
        ARMT_TRY(save_tape(c, l, l, (int)s + l));
        ARMT_TRY(run_group<T>(c, l, l, empty ? l - 1 : l, empty ? l : -1));
      }
      ARMT_TRY(emit(s));
    }
  } else {
    const int64_t steps = L + N - 1;
    for (int64_t t = 0; t < steps; ++t) {
      int32_t lo, hi;
      armt_diagonal_group(L, (int32_t)N, (int32_t)t, &lo, &hi);
      if (t < N) ARMT_TRY(ingest(t));
      // only the cell of segment 0 (layer t, while t < L) can meet an empty memory
      const bool top_empty = (!carry_in && t < L);
      ARMT_TRY(save_tape(c, lo, hi, (int)t));
      if (hi - lo + 1 <= split_upto) {
        // the cells of a small group one at a time, highest layer first: cell l writes slot l + 1, the input of cell l + 1
        for (int l = hi; l >= lo; --l) {
          const bool e = top_empty && l == hi;
          ARMT_TRY(run_group<T>(c, l, l, e ? l - 1 : l, e ? l : -1));
        }
      } else {
        ARMT_TRY(run_group<T>(c, lo, hi, top_empty ? hi - 1 : hi, top_empty ? hi : -1));
      }
      if (hi == L - 1) ARMT_TRY(emit(t - (L - 1)));
    }
  }
  return ARMT_OK;
}

armt_status forward_impl(const armt_config* cfg, const armt_layer_weights* layers, const void* mem_emb, const void* x,
                         int32_t batch, int64_t n_tokens, const float* A_in, const float* z_in, void* hidden_out, float* A_out,
                         float* z_out, void* workspace, size_t workspace_bytes, void* hip_stream, bool diagonal,
                         float* tape = nullptr, size_t rec_floats = 0, int split_upto = 0) {
  Ctx c;
  c.tape = tape;
  c.rec_floats = rec_floats;
  ARMT_TRY(check_config(cfg, &c.D));
  const Dims& D = c.D;
  if (batch < 1 || (int64_t)batch * D.L > 32768) return ARMT_ERR_SHAPE;      // cells of a step index a launch grid
  if (!layers || !mem_emb || !x || !hidden_out || !A_out || !z_out) return ARMT_ERR_NULL;
  if ((A_in == nullptr) != (z_in == nullptr)) return ARMT_ERR_NULL;
  for (int l = 0; l < D.L; ++l) {
    const armt_layer_weights& w = layers[l];
    if (!w.rms1 || !w.wq || !w.wk || !w.wv || !w.wo || !w.rms2 || !w.wgate || !w.wup || !w.wdown || !w.wm_q ||
        !w.wm_k || !w.wm_v || !w.wm_b)
      return ARMT_ERR_NULL;
  }
  if (n_tokens <= 0 || n_tokens % D.S != 0) return ARMT_ERR_SHAPE;
  const int64_t N = n_tokens / D.S;
  if (N + D.L > (int64_t)1 << 30) return ARMT_ERR_SHAPE;
  c.D.B = batch;
  c.D.L = D.Lr * batch;                    // from here on L counts cells per step (see Dims)
  c.o = carve(D);
  if (!workspace || ((uintptr_t)workspace % kAlign) != 0 || workspace_bytes < c.o.total) return ARMT_ERR_WORKSPACE;
  c.ws = (char*)workspace;
  c.st = (hipStream_t)hip_stream;
  fill_shapes(c);

  // memory state lives in A_out / z_out for the whole call
  const size_t nA = (size_t)D.L * D.d * D.Phi, nz = (size_t)D.L * D.Phi;
  if (A_in) {
    if (A_in != A_out) copy_f32_kernel<<<1024, 256, 0, c.st>>>(A_out, A_in, nA);
    if (z_in != z_out) copy_f32_kernel<<<16, 256, 0, c.st>>>(z_out, z_in, nz);
  } else {
    fill_f32_kernel<<<1024, 256, 0, c.st>>>(A_out, nA, 0.f);      // A_0 = 0, z_0 = 0 (Eq. 3)
    fill_f32_kernel<<<16, 256, 0, c.st>>>(z_out, nz, 0.f);
  }
  HIP_TRY(hipGetLastError());
  if (D.bf16) {
    f32_to_bf16_kernel<<<1024, 256, 0, c.st>>>(c.at<bf16>(c.o.A16), A_out, nA);
    HIP_TRY(hipGetLastError());
  }
  ARMT_TRY(upload_tables(c, layers, A_out, z_out));
  if (D.bf16) return forward_typed<bf16>(c, mem_emb, x, N, A_in != nullptr, hidden_out, diagonal, split_upto);
  return forward_typed<float>(c, mem_emb, x, N, A_in != nullptr, hidden_out, diagonal, split_upto);
}

}  // namespace

namespace {

armt_status step_prologue(const armt_config* cfg, int32_t g, void* workspace, size_t workspace_bytes, void* stream,
                          Ctx* c) {
  ARMT_TRY(check_config(cfg, &c->D));
  if (g < 1 || g > c->D.L) return ARMT_ERR_SHAPE;
  c->o = carve(c->D);
  if (!workspace || ((uintptr_t)workspace % kAlign) != 0 || workspace_bytes < c->o.total) return ARMT_ERR_WORKSPACE;
  c->ws = (char*)workspace;
  c->st = (hipStream_t)stream;
  fill_shapes(*c);
  return ARMT_OK;
}

armt_status upload(Ctx& c, const std::vector<GemmGroup>& tab, const std::vector<LayerAux>& aux) {
  if (!tab.empty()) ARMT_TRY(upload_bytes(c.st, c.ws + c.o.Tables, tab.data(), tab.size() * sizeof(GemmGroup)));
  if (!aux.empty()) ARMT_TRY(upload_bytes(c.st, c.ws + c.o.Aux, aux.data(), aux.size() * sizeof(LayerAux)));
  c.tables = c.at<GemmGroup>(c.o.Tables);
  c.aux = c.at<LayerAux>(c.o.Aux);
  return ARMT_OK;
}

template <typename T>
armt_status gemm_entry(int32_t g, const GemmShape& s, const GemmGroup* table, hipStream_t st) {
  return gemm<T>(st, table, 0, g, s);
}

}  // namespace

namespace {
constexpr int64_t kHeadRows = 1024;    // rows per group of the head GEMM: 4 tiles of 256, like a cell
struct HeadLayout { size_t xg, rstd, table, total; int64_t groups, rem; };
HeadLayout head_layout(const Dims& D, int64_t n_rows) {
  HeadLayout h;
  h.groups = n_rows / kHeadRows;
  h.rem = n_rows % kHeadRows;
  size_t off = 0;
  auto take = [&](size_t bytes) { const size_t at = off; off += (bytes + kAlign - 1) / kAlign * kAlign; return at; };
  h.xg = take((size_t)n_rows * D.d * D.esz);
  h.rstd = take((size_t)n_rows * 4);
  h.table = take((size_t)(h.groups + 1) * sizeof(GemmGroup));
  h.total = off;
  return h;
}

template <typename T>
armt_status lm_head_typed(const Dims& D, const HeadLayout& h, const void* hidden, int64_t n_rows, const void* gain,
                          const void* w_lm, int32_t vocab, float* logits, char* ws, hipStream_t st,
                          GemmGroup* tab /* host, h.groups + 1 entries */) {
  T* xg = (T*)(ws + h.xg);
  float* rstd = (float*)(ws + h.rstd);
  final_norm_kernel<T><<<(unsigned)n_rows, 256, 0, st>>>((const T*)hidden, (const T*)gain, D.d, D.rms_eps, xg, rstd);
  HIP_TRY(hipGetLastError());
  // the rows go through the grouped GEMM in groups of kHeadRows that all point at the same weight: the
  // tile order then keeps the four M-tiles of a weight panel side by side, as for a cell
  memset(tab, 0, (size_t)(h.groups + 1) * sizeof(GemmGroup));
  for (int64_t i = 0; i <= h.groups; ++i) {
    const size_t r0 = (size_t)i * kHeadRows;
    tab[i].A = xg + r0 * D.d; tab[i].B0 = w_lm; tab[i].C = logits + r0 * (size_t)vocab; tab[i].rowscale = rstd + r0;
  }
  ARMT_TRY(upload_bytes(st, ws + h.table, tab, (size_t)(h.groups + 1) * sizeof(GemmGroup)));
  GemmShape s;
  s.M = (int)kHeadRows; s.N = vocab; s.K = D.d; s.lda = D.d; s.ldc = vocab; s.ldc2 = 0; s.ldr = 0; s.n0 = vocab; s.n1 = 0;
  s.epi = EPI_STORE_F32; s.tag = -1; s.dbg = g_gemm_dbg; s.ldb = s.K;
  const GemmGroup* table = (const GemmGroup*)(ws + h.table);
  for (int64_t g0 = 0; g0 < h.groups; g0 += 256)          // at most 256 groups per launch
    ARMT_TRY(gemm<T>(st, table, (int)g0, (int)std::min<int64_t>(256, h.groups - g0), s));
  if (h.rem) {
    s.M = (int)h.rem;
    ARMT_TRY(gemm<T>(st, table, (int)h.groups, 1, s));
  }
  return ARMT_OK;
}
}  // namespace

// ---- scratch memory of armt_lm_head_static, the entry point for callers that cannot allocate.  One copy of the array
// exists on every GPU that loads the library, at its own address: the name below is only a handle for
// hipGetSymbolAddress in host code, never a device address.
static __device__ __align__(256) unsigned char scratch[ARMT_LM_HEAD_STATIC_BYTES];

namespace {
constexpr size_t kStaticHeadGroups = 64;                  // groups of kHeadRows rows the stack-allocated host table holds
constexpr int kMaxDevices = 64;
std::atomic<char*> g_scratch_ptr[kMaxDevices];            // device address of `scratch` on each device, once looked up

// Address of this device's copy of the array; looked up on the first call on a device, with that device current.
armt_status static_scratch(char** out) {
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return ARMT_ERR_UNSUPPORTED;
  char* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    void* sym = nullptr;
    HIP_TRY(hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)));
    if (!sym) { g_hip_error = "hipGetSymbolAddress returned a null address"; return ARMT_ERR_HIP; }
    p = (char*)sym;
    g_scratch_ptr[dev].store(p, std::memory_order_release);   // a second thread can only store the same address
  }
  *out = p;
  return ARMT_OK;
}
}  // namespace

extern "C" {

size_t armt_workspace_bytes(const armt_config* cfg) {
  Dims D;
  if (check_config(cfg, &D) != ARMT_OK) return 0;
  return carve(D).total;
}

armt_status armt_forward_sequential(const armt_config* cfg, const armt_layer_weights* layers, const void* mem_emb,
                                    const void* x, int64_t n_tokens, const float* A_in, const float* z_in,
                                    void* hidden_out, float* A_out, float* z_out, void* workspace,
                                    size_t workspace_bytes, void* hip_stream) {
  return forward_impl(cfg, layers, mem_emb, x, 1, n_tokens, A_in, z_in, hidden_out, A_out, z_out, workspace,
                      workspace_bytes, hip_stream, false);
}

armt_status armt_forward_diagonal(const armt_config* cfg, const armt_layer_weights* layers, const void* mem_emb,
                                  const void* x, int64_t n_tokens, const float* A_in, const float* z_in,
                                  void* hidden_out, float* A_out, float* z_out, void* workspace,
                                  size_t workspace_bytes, void* hip_stream) {
  return forward_impl(cfg, layers, mem_emb, x, 1, n_tokens, A_in, z_in, hidden_out, A_out, z_out, workspace,
                      workspace_bytes, hip_stream, true);
}

armt_status armt_forward_diagonal_split(const armt_config* cfg, const armt_layer_weights* layers, const void* mem_emb,
                                        const void* x, int64_t n_tokens, const float* A_in, const float* z_in,
                                        void* hidden_out, float* A_out, float* z_out, void* workspace,
                                        size_t workspace_bytes, void* hip_stream, int32_t split_upto) {
  if (split_upto < 0) return ARMT_ERR_SHAPE;
  return forward_impl(cfg, layers, mem_emb, x, 1, n_tokens, A_in, z_in, hidden_out, A_out, z_out, workspace,
                      workspace_bytes, hip_stream, true, nullptr, 0, split_upto);
}

int32_t armt_auto_order(const armt_config* cfg, int64_t n_tokens) {
  Dims D;
  if (check_config(cfg, &D) != ARMT_OK || n_tokens <= 0 || n_tokens % D.S != 0) return -1;
  // One segment: every anti-diagonal holds one cell and the two orders launch the same kernels; take the plain one.
  // From two segments on a step of the diagonal order does the work of up to min(L, N) sequential cell executions with
  // the same kernels on larger launches: it was faster at every length and segment size measured, the paper's
  // 4096-token column included.
  return (n_tokens / D.S >= 2 && D.Lr >= 2) ? 1 : 0;
}

armt_status armt_forward_auto(const armt_config* cfg, const armt_layer_weights* layers, const void* mem_emb,
                              const void* x, int64_t n_tokens, const float* A_in, const float* z_in,
                              void* hidden_out, float* A_out, float* z_out, void* workspace,
                              size_t workspace_bytes, void* hip_stream, int32_t* order_used) {
  const int32_t order = armt_auto_order(cfg, n_tokens);
  if (order_used && order >= 0) *order_used = order;
  return forward_impl(cfg, layers, mem_emb, x, 1, n_tokens, A_in, z_in, hidden_out, A_out, z_out, workspace,
                      workspace_bytes, hip_stream, order == 1);
}

size_t armt_workspace_bytes_batched(const armt_config* cfg, int32_t batch) {
  Dims D;
  if (check_config(cfg, &D) != ARMT_OK || batch < 1 || (int64_t)batch * D.L > 32768) return 0;
  D.B = batch;
  D.L = D.Lr * batch;
  return carve(D).total;
}

armt_status armt_forward_sequential_batched(const armt_config* cfg, const armt_layer_weights* layers,
                                            const void* mem_emb, const void* x, int32_t batch, int64_t n_tokens,
                                            const float* A_in, const float* z_in, void* hidden_out, float* A_out,
                                            float* z_out, void* workspace, size_t workspace_bytes, void* hip_stream) {
  return forward_impl(cfg, layers, mem_emb, x, batch, n_tokens, A_in, z_in, hidden_out, A_out, z_out, workspace,
                      workspace_bytes, hip_stream, false);
}

armt_status armt_forward_diagonal_batched(const armt_config* cfg, const armt_layer_weights* layers,
                                          const void* mem_emb, const void* x, int32_t batch, int64_t n_tokens,
                                          const float* A_in, const float* z_in, void* hidden_out, float* A_out,
                                          float* z_out, void* workspace, size_t workspace_bytes, void* hip_stream) {
  return forward_impl(cfg, layers, mem_emb, x, batch, n_tokens, A_in, z_in, hidden_out, A_out, z_out, workspace,
                      workspace_bytes, hip_stream, true);
}

// ---- single-step entry points: build a small table for the caller's buffers, then run the same
// step functions as the forward path.

armt_status armt_grouped_gemm(int32_t dtype, int32_t g, int32_t M, int32_t N, int32_t K, const void* const* a,
                              const void* const* b, void* const* c, void* workspace, size_t workspace_bytes,
                              void* hip_stream) {
  if (dtype != ARMT_F32 && dtype != ARMT_BF16) return ARMT_ERR_DTYPE;
  if (!a || !b || !c) return ARMT_ERR_NULL;
  if (g < 1 || M < 1 || N < 1 || K < 1) return ARMT_ERR_SHAPE;
  if (dtype == ARMT_BF16 && K % 64 != 0) return ARMT_ERR_UNSUPPORTED;
  if (!workspace || ((uintptr_t)workspace % kAlign) != 0 || workspace_bytes < (size_t)g * sizeof(GemmGroup))
    return ARMT_ERR_WORKSPACE;
  std::vector<GemmGroup> tab(g);
  memset(tab.data(), 0, tab.size() * sizeof(GemmGroup));
  for (int i = 0; i < g; ++i) {
    if (!a[i] || !b[i] || !c[i]) return ARMT_ERR_NULL;
    tab[i].A = a[i]; tab[i].B0 = b[i]; tab[i].C = c[i];
  }
  hipStream_t st = (hipStream_t)hip_stream;
  ARMT_TRY(upload_bytes(st, workspace, tab.data(), tab.size() * sizeof(GemmGroup)));
  GemmShape s;
  s.M = M; s.N = N; s.K = K; s.lda = K; s.ldc = N; s.ldc2 = 0; s.ldr = 0; s.n0 = N; s.n1 = 0; s.epi = EPI_STORE_ACT;
  s.tag = -1;
  s.dbg = g_gemm_dbg;
  s.ldb = K;
  if (dtype == ARMT_BF16) return gemm_entry<bf16>(g, s, (const GemmGroup*)workspace, st);
  return gemm_entry<float>(g, s, (const GemmGroup*)workspace, st);
}

// ---- token-level ends of Algorithm 1
armt_status armt_embed_tokens(const armt_config* cfg, const void* emb_table, int32_t vocab, const int32_t* ids,
                              int64_t n_tokens, void* x_out, void* hip_stream) {
  Dims D;
  ARMT_TRY(check_config(cfg, &D));
  if (!emb_table || !ids || !x_out) return ARMT_ERR_NULL;
  if (vocab < 1 || n_tokens < 1 || n_tokens > 0x7fffffff) return ARMT_ERR_SHAPE;
  const int row_bytes = D.d * D.esz;
  if (row_bytes % 16 != 0) return ARMT_ERR_UNSUPPORTED;
  embed_rows_kernel<<<(unsigned)n_tokens, 256, 0, (hipStream_t)hip_stream>>>(
      (const unsigned char*)emb_table, ids, vocab, row_bytes, (unsigned char*)x_out);
  HIP_TRY(hipGetLastError());
  return ARMT_OK;
}


size_t armt_lm_head_workspace_bytes(const armt_config* cfg, int64_t n_rows) {
  Dims D;
  if (check_config(cfg, &D) != ARMT_OK || n_rows < 1) return 0;
  return head_layout(D, n_rows).total;
}

armt_status armt_lm_head(const armt_config* cfg, const void* hidden, int64_t n_rows, const void* final_gain,
                         const void* w_lm, int32_t vocab, float* logits, void* workspace, size_t workspace_bytes,
                         void* hip_stream) {
  Dims D;
  ARMT_TRY(check_config(cfg, &D));
  if (!hidden || !final_gain || !w_lm || !logits) return ARMT_ERR_NULL;
  if (n_rows < 1 || n_rows > 0x7fffffff || vocab < 1) return ARMT_ERR_SHAPE;
  const HeadLayout h = head_layout(D, n_rows);
  if (!workspace || ((uintptr_t)workspace % kAlign) != 0 || workspace_bytes < h.total) return ARMT_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)hip_stream;
  std::vector<GemmGroup> tab((size_t)h.groups + 1);
  if (D.bf16)
    return lm_head_typed<bf16>(D, h, hidden, n_rows, final_gain, w_lm, vocab, logits, (char*)workspace, st, tab.data());
  return lm_head_typed<float>(D, h, hidden, n_rows, final_gain, w_lm, vocab, logits, (char*)workspace, st, tab.data());
}

armt_status armt_lm_head_static(const armt_config* cfg, const void* hidden, int64_t n_rows, const void* final_gain,
                                const void* w_lm, int32_t vocab, float* logits, void* hip_stream) {
  Dims D;
  ARMT_TRY(check_config(cfg, &D));
  if (!hidden || !final_gain || !w_lm || !logits) return ARMT_ERR_NULL;
  if (n_rows < 1 || n_rows > 0x7fffffff || vocab < 1) return ARMT_ERR_SHAPE;
  const HeadLayout h = head_layout(D, n_rows);
  GemmGroup tab[kStaticHeadGroups];                       // host side of the pointer table: on the stack, no heap
  if (h.total > sizeof(scratch) || (size_t)h.groups + 1 > kStaticHeadGroups) return ARMT_ERR_TOO_LARGE;
  char* ws = nullptr;
  ARMT_TRY(static_scratch(&ws));
  hipStream_t st = (hipStream_t)hip_stream;
  // nothing in the scratch array has to start at zero: the normalised rows, the row scales and the table entries the
  // kernels read are all written first by this call
  if (D.bf16) return lm_head_typed<bf16>(D, h, hidden, n_rows, final_gain, w_lm, vocab, logits, ws, st, tab);
  return lm_head_typed<float>(D, h, hidden, n_rows, final_gain, w_lm, vocab, logits, ws, st, tab);
}

armt_status armt_segment_attention(const armt_config* cfg, int32_t g, void* qkv, void* out, void* workspace,
                                   size_t workspace_bytes, void* hip_stream) {
  Ctx c;
  ARMT_TRY(step_prologue(cfg, g, workspace, workspace_bytes, hip_stream, &c));
  if (!qkv || !out) return ARMT_ERR_NULL;
  const Dims& D = c.D;
  const int n = D.T * (D.dh / 2);
  rope_table_kernel<<<(n + 255) / 256, 256, 0, c.st>>>(c.at<float>(c.o.Rope), D.T, D.dh / 2, (double)D.rope_theta);
  HIP_TRY(hipGetLastError());
  if (D.bf16)
    return step_attention<bf16>(c.st, (bf16*)qkv, (bf16*)out, c.at<bf16>(c.o.Vt), c.at<float>(c.o.Rope), 0, g, D.T, D.H,
                                D.Hkv, D.dh, false, false);
  return step_attention<float>(c.st, (float*)qkv, (float*)out, nullptr, c.at<float>(c.o.Rope), 0, g, D.T, D.H, D.Hkv,
                               D.dh, false, false);
}

armt_status armt_assoc_read(const armt_config* cfg, int32_t g, float* x, const void* const* wm_q, const float* A,
                            const float* z, void* workspace, size_t workspace_bytes, void* hip_stream) {
  Ctx c;
  ARMT_TRY(step_prologue(cfg, g, workspace, workspace_bytes, hip_stream, &c));
  if (!x || !wm_q || !A || !z) return ARMT_ERR_NULL;
  const Dims& D = c.D;
  const size_t T = D.T, L = D.L;
  std::vector<GemmGroup> tab((size_t)K_COUNT * L);
  std::vector<LayerAux> aux(L);
  memset(tab.data(), 0, tab.size() * sizeof(GemmGroup));
  memset(aux.data(), 0, aux.size() * sizeof(LayerAux));
  if (D.bf16) {     // bf16 operands of the two GEMMs: the rows of x and the memory matrices
    f32_to_bf16_kernel<<<1024, 256, 0, c.st>>>(c.at<bf16>(c.o.Xb), x, (size_t)g * T * D.d);
    f32_to_bf16_kernel<<<1024, 256, 0, c.st>>>(c.at<bf16>(c.o.A16), A, (size_t)g * D.d * D.Phi);
    HIP_TRY(hipGetLastError());
  }
  for (int i = 0; i < g; ++i) {
    if (!wm_q[i]) return ARMT_ERR_NULL;
    GemmGroup* q = &tab[K_MQ * L + i];
    q->A = D.bf16 ? (const void*)(c.at<bf16>(c.o.Xb) + i * T * D.d) : (const void*)(x + i * T * D.d);
    q->B0 = wm_q[i];
    q->C = c.ws + c.o.Qm + i * T * D.dm * 4;
    if (c.fused_dpfp) {
      q->C = c.ws + c.o.Fphi + i * T * D.Phi * D.esz; q->C2 = c.ws + c.o.RDen + i * T * 4;
      q->R = z + (size_t)i * D.Phi;
    }
    GemmGroup* r = &tab[K_READ * L + i];
    r->A = c.ws + c.o.Fphi + i * T * D.Phi * D.esz;
    r->B0 = D.bf16 ? (const void*)(c.at<bf16>(c.o.A16) + (size_t)i * D.d * D.Phi) : (const void*)(A + (size_t)i * D.d * D.Phi);
    r->C = x + i * T * D.d;
    r->R = x + i * T * D.d;
    r->rowscale = (const float*)(c.ws + c.o.RDen + i * T * 4);
    aux[i].z = const_cast<float*>(z) + (size_t)i * D.Phi;
  }
  ARMT_TRY(upload(c, tab, aux));
  if (D.bf16)
    return step_assoc_read<bf16>(c.st, c.table(K_MQ), c.shape[K_MQ], c.table(K_READ), c.shape[K_READ], c.aux, 0, g, D.T,
                                 D.dm, D.nu, D.assoc_eps, c.at<float>(c.o.Qm), c.at<bf16>(c.o.Fphi), c.at<float>(c.o.RDen));
  return step_assoc_read<float>(c.st, c.table(K_MQ), c.shape[K_MQ], c.table(K_READ), c.shape[K_READ], c.aux, 0, g, D.T,
                                D.dm, D.nu, D.assoc_eps, c.at<float>(c.o.Qm), c.at<float>(c.o.Fphi), c.at<float>(c.o.RDen));
}

armt_status armt_assoc_update(const armt_config* cfg, int32_t g, const float* ym, const void* const* wm_k,
                              const void* const* wm_v, const void* const* wm_b, int32_t empty_group, float* A,
                              float* z, void* workspace, size_t workspace_bytes, void* hip_stream) {
  Ctx c;
  ARMT_TRY(step_prologue(cfg, g, workspace, workspace_bytes, hip_stream, &c));
  if (!ym || !wm_k || !wm_v || !wm_b || !A || !z) return ARMT_ERR_NULL;
  if (empty_group < -1 || empty_group >= g) return ARMT_ERR_SHAPE;
  const Dims& D = c.D;
  const size_t L = D.L, md = (size_t)D.m * D.d;
  std::vector<GemmGroup> tab((size_t)K_COUNT * L);
  std::vector<LayerAux> aux(L);
  memset(tab.data(), 0, tab.size() * sizeof(GemmGroup));
  memset(aux.data(), 0, aux.size() * sizeof(LayerAux));
  if (D.bf16) {
    f32_to_bf16_kernel<<<256, 256, 0, c.st>>>(c.at<bf16>(c.o.Xb), ym, (size_t)g * md);
    HIP_TRY(hipGetLastError());
  }
  for (int i = 0; i < g; ++i) {
    if (!wm_k[i] || !wm_v[i] || !wm_b[i]) return ARMT_ERR_NULL;
    GemmGroup* k = &tab[K_MKV * L + i];
    k->A = D.bf16 ? (const void*)(c.at<bf16>(c.o.Xb) + i * md) : (const void*)(ym + i * md);
    k->B0 = wm_k[i];
    k->B1 = wm_v[i];
    k->C = c.ws + c.o.KVm + (size_t)i * D.m * (D.dm + D.d) * 4;
    aux[i].wm_b = wm_b[i];
    aux[i].A = A + (size_t)i * D.d * D.Phi;
    aux[i].z = z + (size_t)i * D.Phi;
  }
  ARMT_TRY(upload(c, tab, aux));
  if (D.bf16)
    return step_assoc_update<bf16>(c.st, c.table(K_MKV), c.shape[K_MKV], c.aux, 0, g, empty_group, empty_group + 1, c.at<bf16>(c.o.Xb), md,
                                   D.m, D.d, D.dm, D.nu, D.assoc_eps, c.at<float>(c.o.KVm), c.at<float>(c.o.Fm),
                                   c.at<float>(c.o.Coef));
  return step_assoc_update<float>(c.st, c.table(K_MKV), c.shape[K_MKV], c.aux, 0, g, empty_group, empty_group + 1, ym, md, D.m, D.d, D.dm,
                                  D.nu, D.assoc_eps, c.at<float>(c.o.KVm), c.at<float>(c.o.Fm), c.at<float>(c.o.Coef));
}

int32_t armt_diagonal_group(int32_t n_layers, int32_t n_segments, int32_t t, int32_t* l_lo, int32_t* l_hi) {
  if (n_layers < 1 || n_segments < 1 || t < 0 || (int64_t)t > (int64_t)n_layers + n_segments - 2) return 0;
  // cell (l, s = t - l) is live iff 0 <= l < L and 0 <= t - l < N
  const int32_t lo = t - n_segments + 1 > 0 ? t - n_segments + 1 : 0;
  const int32_t hi = t < n_layers - 1 ? t : n_layers - 1;
  if (l_lo) *l_lo = lo;
  if (l_hi) *l_hi = hi;
  return hi - lo + 1;
}

int32_t armt_set_gemm_tile_config(int32_t config) {
  const int32_t old = g_gemm_tile_config;
  g_gemm_dbg = config >= 100 ? config / 100 : 0;
  if (config >= 100) config %= 100;
  g_gemm_tile_config = (config >= 1 && config <= 6) ? config : -1;
  return old;
}

armt_status armt_profile_begin(int32_t gemm_kind, int32_t max_launches) {
  if (gemm_kind < 0 || gemm_kind >= PK_COUNT || max_launches < 1) return ARMT_ERR_SHAPE;
  armt_profile_end(nullptr, nullptr, nullptr);
  g_prof.ev.resize((size_t)max_launches * 2);
  for (size_t i = 0; i < g_prof.ev.size(); ++i) {
    if (hipEventCreate(&g_prof.ev[i]) != hipSuccess) {
      for (size_t j = 0; j < i; ++j) (void)hipEventDestroy(g_prof.ev[j]);
      g_prof.ev.clear();
      g_hip_error = "hipEventCreate failed";
      return ARMT_ERR_HIP;
    }
  }
  g_prof.used = 0;
  g_prof.groups = 0;
  g_prof.kind = gemm_kind;
  return ARMT_OK;
}

armt_status armt_profile_end(double* total_ms, int64_t* launches, int64_t* groups) {
  double sum = 0.0;
  armt_status rc = ARMT_OK;
  for (size_t i = 0; i + 1 < g_prof.used; i += 2) {
    float ms = 0.f;
    if (hipEventSynchronize(g_prof.ev[i + 1]) != hipSuccess ||
        hipEventElapsedTime(&ms, g_prof.ev[i], g_prof.ev[i + 1]) != hipSuccess) {
      g_hip_error = "hipEventElapsedTime failed";
      rc = ARMT_ERR_HIP;
      break;
    }
    sum += ms;
  }
  if (total_ms) *total_ms = sum;
  if (launches) *launches = (int64_t)(g_prof.used / 2);
  if (groups) *groups = g_prof.groups;
  for (hipEvent_t e : g_prof.ev) (void)hipEventDestroy(e);
  g_prof.ev.clear();
  g_prof.used = 0;
  g_prof.groups = 0;
  g_prof.kind = -1;
  return rc;
}

const char* armt_status_str(armt_status s) {
  switch (s) {
    case ARMT_OK: return "ok";
    case ARMT_ERR_NULL: return "a required pointer is NULL";
    case ARMT_ERR_SHAPE: return "inconsistent sizes";
    case ARMT_ERR_DTYPE: return "unknown dtype";
    case ARMT_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case ARMT_ERR_HIP: return "HIP runtime error";
    case ARMT_ERR_UNSUPPORTED: return "shape not supported by this build";
    case ARMT_ERR_TOO_LARGE: return "input exceeds the fixed scratch array of a *_static call";
  }
  return "unknown status";
}

const char* armt_last_hip_error(void) { return g_hip_error.c_str(); }

#ifdef ARMT_GEMM_TIMELINE
// probe build only: arm the n-th next launch of a GEMM kind; read the records back (8 x 64 bits per workgroup)
void armt_timeline_arm(int32_t kind, int32_t nth) { g_tl_kind = kind; g_tl_countdown = nth; }
int32_t armt_timeline_read(unsigned long long* host, int64_t n_words) {
  return (int32_t)hipMemcpyFromSymbol(host, HIP_SYMBOL(armt_timeline), (size_t)n_words * 8, 0, hipMemcpyDeviceToHost);
}
#endif

}  // extern "C"

#include "backward_host.h"
