// Host side of the ARMT backward pass (included at the end of armt_api.hip: it uses that file's Ctx-less helpers,
// the grouped GEMM dispatcher and the forward's step functions).
//
// The training forward (armt_forward_train) is the inference forward plus a tape: per (segment, layer) cell the cell
// input and the layer's memory state from before the cell's update.  The backward pass (armt_backward) walks the cells
// in the reverse of the forward order (anti-diagonals t = L + N - 2 .. 0, or segment by segment, layer by layer): for
// the cells of a step it restores their inputs from the tape, recomputes the forward of these cells keeping every
// intermediate, and runs the backward kernels.  The gradient of the residual stream travels through slots exactly
// like the activations of the forward pass, in the opposite direction: the input gradient of cell l + 1 is the
// output gradient of cell l of the next (earlier) step; the gradients of A and z of a layer travel from segment to
// segment in place.
#pragma once

namespace {

inline int round64(int v) { return (v + 63) / 64 * 64; }

// Weight gradients are accumulated over a window of WG_WIN consecutive steps: the transposed operands of a step go into
// slot (step % WG_WIN) of buffers whose rows hold WG_WIN slots side by side, and one GEMM per kind with the reduction
// dimension WG_WIN x T then adds the window to the fp32 gradient.  The fp32 read-modify-write of a layer's 60.8 M
// weight gradients (486 MB at the 1B shape) is as expensive as the product of one segment; this divides it by WG_WIN.
// Eight against four: 2.7 % faster backward at 128 segments, 1 % slower at 32 (more partial steps), twice the buffers.
// Sixteen against eight: 0.7 % slower at 128 segments (and 27.8 instead of 16.6 GB of workspace at the 1B shape).
constexpr int WG_WIN = 8;

enum TKind {
  // forward recomputation
  TK_MQ = 0, TK_READ, TK_QKV, TK_O, TK_GU, TK_DOWN, TK_MKV,
  // gradients of activations: dY W
  TK_DYM, TK_DU, TK_DN2, TK_DATT, TK_DN1, TK_DF, TK_DXQ,
  // gradients of weights (and of A): dY^T X, accumulated in fp32
  TK_WD, TK_WG, TK_WU, TK_WO, TK_WQ, TK_WK, TK_WV, TK_DA, TK_WMQ, TK_WMK, TK_WMV,
  TK_COUNT
};

struct TrainLayout {
  size_t Xin, X1, Xb, N1, N2, RStd1, RStd2, QKV, Vt, Att, Hres, GU, Uff, Yf, Yb, Qm, Fphi, RDen, KVm, Fm, Coef, Rope;
  size_t Aw, zw, A16w, ATr;
  size_t DX, DYb, DU, DN, DH, DHb, DAtt, DQKV, LSE, Dv, AttS, DNum, DF, DDen, DQr, DKV, DV, Part, DB, DZF, DA, DZ, Upd;
  size_t TA, TB, TmA, TmB, CPart, WinA, WinB;
  size_t wa_rows, wb_rows, aDY, aDGU, aDH, aDQKV, aDQR, bU, bN2, bATT, bN1, bX;   // rows of a layer's window operands
  size_t WdT, WguT, WoT, WqkvT, WmqT, WmkvT;
  size_t Ptrs, Tables, Aux, total;
  int Tp, mp, dmP, Kmkv, nblk, Kw, Km;     // Kw, Km: columns of a window row (WG_WIN slots x batch x Tp or mp)
  size_t ta_rows, tb_rows;
};

TrainLayout carve_train(const Dims& D) {
  TrainLayout o;
  size_t p = 0;
  auto take = [&](size_t bytes) { size_t at = p; p = align_up(p + bytes); return at; };
  // L = cells of a step (layers x batch): everything per cell; Lr = layers: weights, their gradients' window operands
  const size_t L = D.L, Lr = D.Lr, B = D.B, T = D.T, d = D.d, e = D.esz, F = D.F, Hd = (size_t)D.H * D.dh;
  o.Tp = round64(D.T); o.mp = round64(D.m); o.dmP = round64(D.dm); o.Kmkv = round64(D.dm + D.d);
  o.nblk = (D.d + UB_ROWS - 1) / UB_ROWS;
  o.Kw = WG_WIN * (int)B * o.Tp; o.Km = WG_WIN * (int)B * o.mp;
  // bf16 GEMM operands with T rows per cell end in padding rows, so that the grouped GEMM may read whole 256-row tiles
  const size_t LT = L * T + (D.bf16 ? padded_rows(D.T) - T : 0);
  o.Xin = take(L * T * d * 4);
  o.X1 = take(L * T * d * 4);
  o.Xb = take(D.bf16 ? LT * d * 2 : 0);
  o.N1 = take(LT * d * e);
  o.N2 = take(LT * d * e);
  o.RStd1 = take(L * T * 4);
  o.RStd2 = take(L * T * 4);
  o.QKV = take(L * T * D.Nqkv * e);
  o.Vt = take(D.bf16 ? attention_vt_bytes(D.L, D.T, D.Hkv, D.dh) : 0);
  o.Att = take(LT * Hd * e);
  o.Hres = take(L * T * d * 4);
  o.GU = take(LT * 2 * F * e);
  o.Uff = take(L * T * F * e);
  o.Yf = take(L * T * d * 4);
  o.Yb = take(D.bf16 ? L * T * d * 2 : 0);
  o.Qm = take(L * T * D.dm * 4);
  o.Fphi = take(LT * D.Phi * e);
  o.RDen = take(L * T * 4);
  o.KVm = take(L * D.m * (size_t)(D.dm + D.d) * 4);
  o.Fm = take(L * D.m * (size_t)D.Phi * 4);
  o.Coef = take(L * D.m * 4 * 4);
  o.Rope = take(T * (D.dh / 2) * 2 * 4);
  o.Aw = take(L * d * D.Phi * 4);
  o.zw = take(L * (size_t)D.Phi * 4);
  o.A16w = take(D.bf16 ? L * d * D.Phi * 2 : 0);
  o.ATr = take(L * d * D.Phi * e);
  o.DX = take((L + B) * T * d * 4);
  o.DYb = take(LT * d * e);
  o.DU = take(L * T * F * e);
  o.DN = take(L * T * d * e);
  o.DH = take(L * T * d * 4);
  o.DHb = take(LT * d * e);
  o.DAtt = take(L * T * Hd * e);
  o.DQKV = take(LT * D.Nqkv * e);
  o.LSE = take(L * D.H * T * 4);
  o.Dv = take(L * D.H * T * 4);
  o.AttS = take(D.bf16 ? attention_bwd_scratch_bytes(D.L, D.T, D.H, D.Hkv, D.dh) : 0);
  o.DNum = take(LT * d * e);
  o.DF = take(L * T * D.Phi * 4);
  o.DDen = take(L * T * 4);
  o.DQr = take(LT * o.dmP * e);
  o.DKV = take(L * D.m * (size_t)o.Kmkv * e);
  o.DV = take(L * D.m * d * 4);
  o.Part = take(L * o.nblk * D.m * (size_t)(D.Phi + 2) * 4);
  o.DB = take(L * D.m * 4);
  o.DZF = take(L * D.m * 4);
  o.DA = take(L * d * D.Phi * 4);
  o.DZ = take(L * (size_t)D.Phi * 4);
  o.Upd = take(D.m > UB_M ? L * d * D.Phi * 4 : 0);
  o.ta_rows = d;                                   // dnum^T and phi^T of the read: operands of dA += dnum^T phi (every step)
  o.tb_rows = (size_t)D.Phi;
  o.TA = take(L * o.ta_rows * o.Tp * e);
  o.TB = take(L * o.tb_rows * o.Tp * e);
  o.TmA = take(Lr * (size_t)(D.dm + D.d) * o.Km * e);
  o.TmB = take(Lr * d * o.Km * e);
  o.aDY = 0; o.aDGU = d; o.aDH = d + 2 * F; o.aDQKV = 2 * d + 2 * F; o.aDQR = 2 * d + 2 * F + D.Nqkv;
  o.wa_rows = o.aDQR + D.dm;
  o.bU = 0; o.bN2 = F; o.bATT = F + d; o.bN1 = F + d + Hd; o.bX = F + 2 * d + Hd;
  o.wb_rows = o.bX + d;
  o.WinA = take(Lr * o.wa_rows * o.Kw * e);
  o.WinB = take(Lr * o.wb_rows * o.Kw * e);
  o.CPart = take(L * CS_CHUNKS * std::max(d, (size_t)D.Phi) * 4);
  o.WdT = take(Lr * F * d * e);
  o.WguT = take(Lr * d * 2 * F * e);
  o.WoT = take(Lr * Hd * d * e);
  o.WqkvT = take(Lr * d * D.Nqkv * e);
  o.WmqT = take(Lr * d * o.dmP * e);
  o.WmkvT = take(Lr * d * o.Kmkv * e);
  o.Ptrs = take(3 * L * sizeof(float*));
  o.Tables = take((size_t)TK_COUNT * L * sizeof(GemmGroup));
  o.Aux = take(L * sizeof(LayerAux));
  o.total = p;
  return o;
}

size_t tape_record_floats(const Dims& D) {
  const size_t n = (size_t)D.T * D.d + (size_t)D.d * D.Phi + D.Phi;
  return (n + 63) / 64 * 64;
}

armt_status check_backward_config(const armt_config* cfg, Dims* D) {
  ARMT_TRY(check_config(cfg, D));
  // the attention backward kernels hold two head-dimension columns per lane
  if (D->dh > 128) return ARMT_ERR_UNSUPPORTED;
  return ARMT_OK;
}

struct BCtx {
  Dims D;
  TrainLayout o;
  char* ws;
  hipStream_t st;
  const GemmGroup* tables;
  const LayerAux* aux;
  float* const* dg1; float* const* dg2; float* const* dwb;     // device tables of per-layer gradient pointers
  GemmShape shape[TK_COUNT];
  template <typename T> T* at(size_t off) const { return (T*)(ws + off); }
  const GemmGroup* table(int kind) const { return tables + (size_t)kind * D.L; }
};

void fill_train_shapes(BCtx& c) {
  const Dims& D = c.D;
  const TrainLayout& o = c.o;
  const int Hd = D.H * D.dh, Hkd = D.Hkv * D.dh;
  auto set = [&](int k, int M, int N, int K, int lda, int ldc, int epi, int n0 = -1, int n1 = 0, int ldb = 0) {
    GemmShape s;
    s.M = M; s.N = N; s.K = K; s.lda = lda; s.ldc = ldc; s.ldc2 = 0; s.ldr = ldc; s.n0 = n0 < 0 ? N : n0; s.n1 = n1; s.epi = epi;
    s.tag = -1; s.dbg = 0; s.ldb = ldb ? ldb : K;
    c.shape[k] = s;
  };
  set(TK_MQ, D.T, D.dm, D.d, D.d, D.dm, EPI_STORE_F32);
  set(TK_READ, D.T, D.d, D.Phi, D.Phi, D.d, EPI_RESID_F32);
  set(TK_QKV, D.T, D.Nqkv, D.d, D.d, D.Nqkv, EPI_STORE_ACT, Hd, Hkd);
  set(TK_O, D.T, D.d, Hd, Hd, D.d, EPI_RESID_F32);
  set(TK_GU, D.T, 2 * D.F, D.d, D.d, 2 * D.F, EPI_STORE_ACT, D.F, D.F);
  set(TK_DOWN, D.m, D.d, D.F, D.F, D.d, EPI_RESID_F32);      // only the memory rows of the block's output are needed again
  if (D.bf16) c.shape[TK_DOWN].ldc2 = D.d;
  set(TK_MKV, D.m, D.dm + D.d, D.d, D.d, D.dm + D.d, EPI_STORE_F32, D.dm, D.d);
  set(TK_DYM, D.m, D.d, o.Kmkv, o.Kmkv, D.d, EPI_RESID_F32);
  set(TK_DU, D.T, D.F, D.d, D.d, D.F, EPI_STORE_ACT);
  set(TK_DN2, D.T, D.d, 2 * D.F, 2 * D.F, D.d, EPI_STORE_ACT);
  set(TK_DATT, D.T, Hd, D.d, D.d, Hd, EPI_STORE_ACT);
  set(TK_DN1, D.T, D.d, D.Nqkv, D.Nqkv, D.d, EPI_STORE_ACT);
  set(TK_DF, D.T, D.Phi, D.d, D.d, D.Phi, EPI_STORE_F32);
  set(TK_DXQ, D.T, D.d, o.dmP, o.dmP, D.d, EPI_RESID_F32);
  if (D.bf16)      // their A operands end in padding rows (carve_train)
    for (int k : {TK_MQ, TK_READ, TK_QKV, TK_O, TK_GU, TK_DU, TK_DN2, TK_DATT, TK_DN1, TK_DF, TK_DXQ})
      c.shape[k].a_rows = (int)padded_rows(D.T);
  // weight gradients: K = slots of the window actually filled (set at launch), lda = ldb = a whole window row
  const int Kw = o.Kw, Km = o.Km;
  set(TK_WD, D.d, D.F, Kw, Kw, D.F, EPI_RESID_F32, -1, 0, Kw);
  set(TK_WG, D.F, D.d, Kw, Kw, D.d, EPI_RESID_F32, -1, 0, Kw);
  set(TK_WU, D.F, D.d, Kw, Kw, D.d, EPI_RESID_F32, -1, 0, Kw);
  set(TK_WO, D.d, Hd, Kw, Kw, Hd, EPI_RESID_F32, -1, 0, Kw);
  set(TK_WQ, Hd, D.d, Kw, Kw, D.d, EPI_RESID_F32, -1, 0, Kw);
  set(TK_WK, Hkd, D.d, Kw, Kw, D.d, EPI_RESID_F32, -1, 0, Kw);
  set(TK_WV, Hkd, D.d, Kw, Kw, D.d, EPI_RESID_F32, -1, 0, Kw);
  set(TK_DA, D.d, D.Phi, o.Tp, o.Tp, D.Phi, EPI_RESID_F32);
  set(TK_WMQ, D.dm, D.d, Kw, Kw, D.d, EPI_RESID_F32, -1, 0, Kw);
  set(TK_WMK, D.dm, D.d, Km, Km, D.d, EPI_RESID_F32, -1, 0, Km);
  set(TK_WMV, D.d, D.d, Km, Km, D.d, EPI_RESID_F32, -1, 0, Km);
}

armt_status upload_train_tables(BCtx& c, const armt_layer_weights* W, const armt_layer_grads* G) {
  const Dims& D = c.D;
  const TrainLayout& o = c.o;
  const size_t L = D.L, T = D.T, d = D.d, e = D.esz, F = D.F, Hd = (size_t)D.H * D.dh, Hkd = (size_t)D.Hkv * D.dh;
  std::vector<GemmGroup> tab((size_t)TK_COUNT * L);
  std::vector<LayerAux> aux(L);
  std::vector<float*> ptrs(3 * L);
  memset(tab.data(), 0, tab.size() * sizeof(GemmGroup));
  char* ws = c.ws;
  const size_t B = D.B;
  for (size_t l = 0; l < L; ++l) {                 // l = cell: layer lr = l / B of sequence l % B
    const size_t lr = l / B;
    const armt_layer_weights& w = W[lr];
    const armt_layer_grads& gw = G[lr];
    auto E = [&](int k) -> GemmGroup* { return &tab[(size_t)k * L + l]; };
    char* X1 = ws + o.X1 + l * T * d * 4;
    char* Xin = ws + o.Xin + l * T * d * 4;
    char* Xop = D.bf16 ? ws + o.Xb + l * T * d * 2 : Xin;           // activation-typed cell input (before the read)
    char* Yop = D.bf16 ? ws + o.Yb + l * T * d * 2 : ws + o.Yf + l * T * d * 4;
    char* DXl = ws + o.DX + l * T * d * 4;
    char* DXup = ws + o.DX + (l + B) * T * d * 4;       // output gradient of cell l: the slot of the cell one layer up
    char* TA = ws + o.TA + l * o.ta_rows * o.Tp * e;
    char* TB = ws + o.TB + l * o.tb_rows * o.Tp * e;
    char* TmA = ws + o.TmA + lr * (size_t)(D.dm + D.d) * o.Km * e;
    char* TmB = ws + o.TmB + lr * d * o.Km * e;
    const size_t rowb = (size_t)o.Kw * e;               // bytes of one window row
    char* WA = ws + o.WinA + lr * o.wa_rows * rowb;
    char* WB = ws + o.WinB + lr * o.wb_rows * rowb;
    GemmGroup* g;
    g = E(TK_MQ); g->A = Xop; g->B0 = w.wm_q; g->C = ws + o.Qm + l * T * D.dm * 4;
    g = E(TK_READ); g->A = ws + o.Fphi + l * T * D.Phi * e;
    g->B0 = D.bf16 ? ws + o.A16w + l * d * D.Phi * 2 : ws + o.Aw + l * d * D.Phi * 4;
    g->C = X1; g->R = (const float*)X1; g->rowscale = (const float*)(ws + o.RDen + l * T * 4);
    g = E(TK_QKV); g->A = ws + o.N1 + l * T * d * e; g->B0 = w.wq; g->B1 = w.wk; g->B2 = w.wv;
    g->C = ws + o.QKV + l * T * D.Nqkv * e;
    g = E(TK_O); g->A = ws + o.Att + l * T * Hd * e; g->B0 = w.wo; g->C = ws + o.Hres + l * T * d * 4; g->R = (const float*)X1;
    g = E(TK_GU); g->A = ws + o.N2 + l * T * d * e; g->B0 = w.wgate; g->B1 = w.wup; g->C = ws + o.GU + l * T * 2 * F * e;
    const size_t mrow = (size_t)D.S;      // first memory row
    g = E(TK_DOWN); g->A = ws + o.Uff + (l * T + mrow) * F * e; g->B0 = w.wdown; g->C = ws + o.Yf + (l * T + mrow) * d * 4;
    g->C2 = D.bf16 ? ws + o.Yb + (l * T + mrow) * d * 2 : nullptr; g->R = (const float*)(ws + o.Hres + (l * T + mrow) * d * 4);
    g = E(TK_MKV); g->A = Yop + (size_t)D.S * d * e; g->B0 = w.wm_k; g->B1 = w.wm_v;
    g->C = ws + o.KVm + l * D.m * (size_t)(D.dm + D.d) * 4;

    g = E(TK_DYM); g->A = ws + o.DKV + l * D.m * (size_t)o.Kmkv * e; g->B0 = ws + o.WmkvT + lr * d * o.Kmkv * e;
    g->C = DXup + (size_t)D.S * d * 4; g->R = (const float*)g->C;
    g = E(TK_DU); g->A = ws + o.DYb + l * T * d * e; g->B0 = ws + o.WdT + lr * F * d * e; g->C = ws + o.DU + l * T * F * e;
    g = E(TK_DN2); g->A = ws + o.GU + l * T * 2 * F * e; g->B0 = ws + o.WguT + lr * d * 2 * F * e; g->C = ws + o.DN + l * T * d * e;
    g = E(TK_DATT); g->A = ws + o.DHb + l * T * d * e; g->B0 = ws + o.WoT + lr * Hd * d * e; g->C = ws + o.DAtt + l * T * Hd * e;
    g = E(TK_DN1); g->A = ws + o.DQKV + l * T * D.Nqkv * e; g->B0 = ws + o.WqkvT + lr * d * D.Nqkv * e;
    g->C = ws + o.DN + l * T * d * e;
    g = E(TK_DF); g->A = ws + o.DNum + l * T * d * e; g->B0 = ws + o.ATr + l * d * D.Phi * e; g->C = ws + o.DF + l * T * D.Phi * 4;
    g = E(TK_DXQ); g->A = ws + o.DQr + l * T * o.dmP * e; g->B0 = ws + o.WmqT + lr * d * o.dmP * e; g->C = DXl; g->R = (const float*)DXl;

    // weight gradients: one entry per LAYER (index lr), written when its first cell comes by; dA: one per cell
    auto wgrad = [&](int k, char* A, char* Bp, float* C) {
      if (k != TK_DA && l % B != 0) return;
      GemmGroup* q = &tab[(size_t)k * L + (k == TK_DA ? l : lr)]; q->A = A; q->B0 = Bp; q->C = C; q->R = C;
    };
    wgrad(TK_WD, WA + o.aDY * rowb, WB + o.bU * rowb, gw.wdown);
    wgrad(TK_WG, WA + o.aDGU * rowb, WB + o.bN2 * rowb, gw.wgate);
    wgrad(TK_WU, WA + (o.aDGU + F) * rowb, WB + o.bN2 * rowb, gw.wup);
    wgrad(TK_WO, WA + o.aDH * rowb, WB + o.bATT * rowb, gw.wo);
    wgrad(TK_WQ, WA + o.aDQKV * rowb, WB + o.bN1 * rowb, gw.wq);
    wgrad(TK_WK, WA + (o.aDQKV + Hd) * rowb, WB + o.bN1 * rowb, gw.wk);
    wgrad(TK_WV, WA + (o.aDQKV + Hd + Hkd) * rowb, WB + o.bN1 * rowb, gw.wv);
    wgrad(TK_DA, TA, TB, (float*)(ws + o.DA + l * d * D.Phi * 4));
    wgrad(TK_WMQ, WA + o.aDQR * rowb, WB + o.bX * rowb, gw.wm_q);
    wgrad(TK_WMK, TmA, TmB, gw.wm_k);
    wgrad(TK_WMV, TmA + (size_t)D.dm * o.Km * e, TmB, gw.wm_v);

    LayerAux& a = aux[l];
    a.rms1 = w.rms1; a.rms2 = w.rms2; a.wm_b = w.wm_b;
    a.A = (float*)(ws + o.Aw + l * d * D.Phi * 4); a.z = (float*)(ws + o.zw + l * D.Phi * 4);
    a.A16 = D.bf16 ? (bf16*)(ws + o.A16w + l * d * D.Phi * 2) : nullptr;
    ptrs[l] = gw.rms1; ptrs[L + l] = gw.rms2; ptrs[2 * L + l] = gw.wm_b;
  }
  ARMT_TRY(upload_bytes(c.st, ws + o.Tables, tab.data(), tab.size() * sizeof(GemmGroup)));
  ARMT_TRY(upload_bytes(c.st, ws + o.Aux, aux.data(), aux.size() * sizeof(LayerAux)));
  ARMT_TRY(upload_bytes(c.st, ws + o.Ptrs, ptrs.data(), ptrs.size() * sizeof(float*)));
  c.tables = c.at<GemmGroup>(o.Tables);
  c.aux = c.at<LayerAux>(o.Aux);
  c.dg1 = c.at<float*>(o.Ptrs); c.dg2 = c.dg1 + L; c.dwb = c.dg1 + 2 * L;
  return ARMT_OK;
}

template <typename Tin, typename Tout>
armt_status transpose(hipStream_t st, const Tin* src, size_t src_cell, int lds, Tout* dst, size_t dst_cell, int ldd, int R, int C,
                      int g) {
  if (g <= 0 || R <= 0 || C <= 0) return ARMT_OK;
  if constexpr (std::is_same<Tin, bf16>::value && std::is_same<Tout, bf16>::value) {
    if (C % 8 == 0 && lds % 8 == 0 && ldd % 8 == 0 && src_cell % 8 == 0 && dst_cell % 8 == 0 && ((uintptr_t)src % 16) == 0 &&
        ((uintptr_t)dst % 16) == 0) {
      transpose_bf16_kernel<<<dim3((C + 63) / 64, (R + 63) / 64, g), 256, 0, st>>>(src, src_cell, lds, dst, dst_cell, ldd, R, C);
      HIP_TRY(hipGetLastError());
      return ARMT_OK;
    }
  }
  transpose_kernel<Tin, Tout><<<dim3((C + 31) / 32, (R + 31) / 32, g), dim3(32, 8), 0, st>>>(src, src_cell, lds, dst, dst_cell, ldd,
                                                                                          R, C);
  HIP_TRY(hipGetLastError());
  return ARMT_OK;
}

inline unsigned ew_blocks(size_t n) { return (unsigned)std::max<size_t>(1, std::min<size_t>((n + 255) / 256, 65535)); }

// Transposed copies of the weights, once per call: they are the B operands of the activation-gradient GEMMs.
template <typename T>
armt_status transpose_weights(BCtx& c, const armt_layer_weights* W) {
  const Dims& D = c.D;
  const TrainLayout& o = c.o;
  const size_t d = D.d, F = D.F, Hd = (size_t)D.H * D.dh, Hkd = (size_t)D.Hkv * D.dh;
  const size_t nq = (size_t)D.Lr * d * o.dmP, nk = (size_t)D.Lr * d * o.Kmkv;
  fill_f32_kernel<<<ew_blocks(nq), 256, 0, c.st>>>(c.at<float>(o.WmqT), nq * D.esz / 4, 0.f);   // K padding must read as zero
  fill_f32_kernel<<<ew_blocks(nk), 256, 0, c.st>>>(c.at<float>(o.WmkvT), nk * D.esz / 4, 0.f);
  HIP_TRY(hipGetLastError());
  for (int l = 0; l < D.Lr; ++l) {
    const armt_layer_weights& w = W[l];
    T* WdT = c.at<T>(o.WdT) + l * F * d;
    T* WguT = c.at<T>(o.WguT) + l * d * 2 * F;
    T* WoT = c.at<T>(o.WoT) + l * Hd * d;
    T* WqkvT = c.at<T>(o.WqkvT) + l * d * D.Nqkv;
    T* WmqT = c.at<T>(o.WmqT) + l * d * o.dmP;
    T* WmkvT = c.at<T>(o.WmkvT) + l * d * o.Kmkv;
    ARMT_TRY((transpose<T, T>(c.st, (const T*)w.wdown, 0, D.F, WdT, 0, D.d, D.d, D.F, 1)));
    ARMT_TRY((transpose<T, T>(c.st, (const T*)w.wgate, 0, D.d, WguT, 0, 2 * D.F, D.F, D.d, 1)));
    ARMT_TRY((transpose<T, T>(c.st, (const T*)w.wup, 0, D.d, WguT + F, 0, 2 * D.F, D.F, D.d, 1)));
    ARMT_TRY((transpose<T, T>(c.st, (const T*)w.wo, 0, (int)Hd, WoT, 0, D.d, D.d, (int)Hd, 1)));
    ARMT_TRY((transpose<T, T>(c.st, (const T*)w.wq, 0, D.d, WqkvT, 0, D.Nqkv, (int)Hd, D.d, 1)));
    ARMT_TRY((transpose<T, T>(c.st, (const T*)w.wk, 0, D.d, WqkvT + Hd, 0, D.Nqkv, (int)Hkd, D.d, 1)));
    ARMT_TRY((transpose<T, T>(c.st, (const T*)w.wv, 0, D.d, WqkvT + Hd + Hkd, 0, D.Nqkv, (int)Hkd, D.d, 1)));
    ARMT_TRY((transpose<T, T>(c.st, (const T*)w.wm_q, 0, D.d, WmqT, 0, o.dmP, D.dm, D.d, 1)));
    ARMT_TRY((transpose<T, T>(c.st, (const T*)w.wm_k, 0, D.d, WmkvT, 0, o.Kmkv, D.dm, D.d, 1)));
    ARMT_TRY((transpose<T, T>(c.st, (const T*)w.wm_v, 0, D.d, WmkvT + D.dm, 0, o.Kmkv, D.d, D.d, 1)));
  }
  return ARMT_OK;
}

// bf16 with head_dim 64 or 128 (what check_config admits for bf16): attention forward and backward on the matrix cores
template <typename T>
bool mfma_attention_bwd(const Dims& D) {
  return std::is_same<T, bf16>::value && !debug_generic() && (D.dh == 64 || D.dh == 128) && D.H / D.Hkv <= 8;
}

template <typename T>
armt_status bgemm(const BCtx& c, int kind, int first, int g) {
  return gemm<T>(c.st, c.table(kind), first, g, c.shape[kind]);
}

// dst[cell][col] += sum over the T rows of w[row] a[row, col] (b ? b[row, col] : 1), rows added in a fixed order.
template <typename T>
armt_status colsum(const BCtx& c, const T* a, const float* b, size_t b_cell, const float* w, float* const* dst_tab, float* dst_base,
                   int first, int g, int C) {
  if (g <= 0) return ARMT_OK;
  float* part = c.at<float>(c.o.CPart);
  colsum_partial_kernel<T><<<dim3((C + 255) / 256, g, CS_CHUNKS), 256, 0, c.st>>>(a, b, b_cell, w, part, first, c.D.T, C);
  // a per-layer destination (pointer table) takes the B cells of the layer in one thread, in order
  const int nb = dst_tab ? c.D.B : 1;
  colsum_finish_kernel<<<dim3((C + 255) / 256, g / nb), 256, 0, c.st>>>(part, CS_CHUNKS, dst_tab, dst_base, first, C, nb);
  HIP_TRY(hipGetLastError());
  return ARMT_OK;
}

// Forward of the cells [lo, lo + g) from their restored inputs, every intermediate kept.  The first gr cells read
// their memory; cells [e0, e1) meet an empty one.
template <typename T>
armt_status recompute_group(const BCtx& c, int lo, int g, int gr, int e0, int e1, int slot) {
  const Dims& D = c.D;
  const TrainLayout& o = c.o;
  const size_t cell = (size_t)D.T * D.d;
  float* X1 = c.at<float>(o.X1);
  copy_f32_kernel<<<ew_blocks(g * cell), 256, 0, c.st>>>(X1 + lo * cell, c.at<float>(o.Xin) + lo * cell, g * cell);
  if (D.bf16) {
    f32_to_bf16_kernel<<<ew_blocks(g * cell), 256, 0, c.st>>>(c.at<bf16>(o.Xb) + lo * cell, c.at<float>(o.Xin) + lo * cell, g * cell);
    const size_t nA = (size_t)D.d * D.Phi;
    f32_to_bf16_kernel<<<ew_blocks(g * nA), 256, 0, c.st>>>(c.at<bf16>(o.A16w) + lo * nA, c.at<float>(o.Aw) + lo * nA, g * nA);
  }
  HIP_TRY(hipGetLastError());
  ARMT_TRY(step_assoc_read<T>(c.st, c.table(TK_MQ), c.shape[TK_MQ], c.table(TK_READ), c.shape[TK_READ], c.aux, lo, gr, D.T,
                              D.dm, D.nu, D.assoc_eps, c.at<float>(o.Qm), c.at<T>(o.Fphi), c.at<float>(o.RDen)));
  rmsnorm_train_kernel<T><<<dim3(D.T, g), 256, 0, c.st>>>(X1, cell, c.aux, lo, 0, D.T, D.d, D.rms_eps, c.at<T>(o.N1),
                                                         c.at<float>(o.RStd1));
  HIP_TRY(hipGetLastError());
  ARMT_TRY(bgemm<T>(c, TK_QKV, lo, g));
  if (mfma_attention_bwd<T>(D)) {      // the matrix-core forward kernel also leaves the log-sum-exp of every row
    rope_kernel<T><<<dim3(D.T, g), 256, 0, c.st>>>(c.at<T>(o.QKV), c.at<float>(o.Rope), lo, D.T, D.H + D.Hkv, D.dh, D.Nqkv);
    HIP_TRY(hipGetLastError());
    HIP_TRY(launch_attention_mfma(c.at<bf16>(o.QKV), c.at<bf16>(o.Vt), c.at<bf16>(o.Att), lo, g, D.T, D.H, D.Hkv, D.dh, false, c.st,
                                  c.at<float>(o.LSE)));
  } else {
    ARMT_TRY(step_attention<T>(c.st, c.at<T>(o.QKV), c.at<T>(o.Att), c.at<bf16>(o.Vt), c.at<float>(o.Rope), lo, g, D.T, D.H, D.Hkv,
                               D.dh, false, false));
  }
  ARMT_TRY(bgemm<T>(c, TK_O, lo, g));
  rmsnorm_train_kernel<T><<<dim3(D.T, g), 256, 0, c.st>>>(c.at<float>(o.Hres), cell, c.aux, lo, 1, D.T, D.d, D.rms_eps,
                                                         c.at<T>(o.N2), c.at<float>(o.RStd2));
  HIP_TRY(hipGetLastError());
  ARMT_TRY(bgemm<T>(c, TK_GU, lo, g));
  if constexpr (std::is_same<T, bf16>::value) {
    // u = silu(gate) up, written transposed into the window rows of dW_down's B operand; U itself only on the memory rows
    const int Kw = o.Kw;
    const size_t wb_cell = o.wb_rows * Kw;
    bf16* dstB = c.at<bf16>(o.WinB) + (size_t)(lo / D.B) * wb_cell + (size_t)slot * D.B * o.Tp + o.bU * Kw;
    swiglu_tiles_kernel<false><<<dim3(D.F / 64, (D.T + 63) / 64, g), 256, 0, c.st>>>(
        c.at<bf16>(o.GU) + (size_t)lo * D.T * 2 * D.F, c.at<bf16>(o.Uff) + (size_t)lo * D.T * D.F, D.T, D.F, D.S, dstB, wb_cell, Kw, D.B,
        o.Tp);
  } else {
    const size_t rows = (size_t)g * D.T;
    swiglu_kernel<T><<<ew_blocks(rows * D.F), 256, 0, c.st>>>(c.at<T>(o.GU) + (size_t)lo * D.T * 2 * D.F,
                                                              c.at<T>(o.Uff) + (size_t)lo * D.T * D.F, rows, D.F);
  }
  HIP_TRY(hipGetLastError());
  ARMT_TRY(bgemm<T>(c, TK_DOWN, lo, g));
  ARMT_TRY(bgemm<T>(c, TK_MKV, lo, g));
  const T* Yop = D.bf16 ? (const T*)c.at<bf16>(o.Yb) : (const T*)c.at<float>(o.Yf);
  memupd_prep_kernel<T><<<dim3(D.m, g), 128, (D.dm + 17) * 4, c.st>>>(c.at<float>(o.KVm), Yop + (size_t)D.S * D.d, cell, c.aux, lo,
                                                                     e0, e1, D.m, D.d, D.dm, D.nu, D.assoc_eps,
                                                                     c.at<float>(o.Fm), c.at<float>(o.Coef));
  HIP_TRY(hipGetLastError());
  return ARMT_OK;
}

// Backward kernels of the cells [lo, lo + g); the first gr of them have a read to differentiate.
template <typename T>
armt_status backward_group(const BCtx& c, int lo, int g, int gr, int slot) {
  const Dims& D = c.D;
  const TrainLayout& o = c.o;
  hipStream_t st = c.st;
  const size_t cell = (size_t)D.T * D.d, Hd = (size_t)D.H * D.dh;
  const int Tp = o.Tp, Phi = D.Phi;
  const size_t ta_cell = o.ta_rows * Tp, tb_cell = o.tb_rows * Tp;
  T* TA = c.at<T>(o.TA) + lo * ta_cell;
  T* TB = c.at<T>(o.TB) + lo * tb_cell;
  // window operands of the weight gradients: this step's columns of a layer's rows; the B cells of a layer side by side
  const int B = D.B, lo_r = lo / B;
  const int Kw = o.Kw, Km = o.Km;
  const size_t wa_cell = o.wa_rows * Kw, wb_cell = o.wb_rows * Kw;
  T* WA = c.at<T>(o.WinA) + lo_r * wa_cell + (size_t)slot * B * Tp;
  T* WB = c.at<T>(o.WinB) + lo_r * wb_cell + (size_t)slot * B * Tp;
  auto arow = [&](size_t r) { return WA + r * Kw; };
  auto brow = [&](size_t r) { return WB + r * Kw; };
  // transposes of n cells (from cell `lo` on) into window rows: sequence b of every layer goes to columns b * colstep
  auto wtr = [&](const T* src, size_t src_cell, int lds, T* dst, size_t dst_cell, int colstep, int ldd, int R, int C, int n) -> armt_status {
    for (int b = 0; b < B; ++b)
      ARMT_TRY((transpose<T, T>(st, src + (size_t)b * src_cell, (size_t)B * src_cell, lds, dst + (size_t)b * colstep, dst_cell, ldd, R, C,
                                n / B)));
    return ARMT_OK;
  };
  float* DX = c.at<float>(o.DX);
  const T* Yop = D.bf16 ? (const T*)c.at<bf16>(o.Yb) : (const T*)c.at<float>(o.Yf);
  const T* Xop = D.bf16 ? (const T*)c.at<bf16>(o.Xb) : (const T*)c.at<float>(o.Xin);

  // ---- memory update (Eq. 3-5)
  {
    const dim3 grid(o.nblk, g);
    const size_t lds = (size_t)UB_M * (2 * Phi + 2) * 4;
#define ARMT_UB(NPL)                                                                                                      \
  case NPL:                                                                                                              \
    update_bwd_rows_kernel<NPL><<<grid, 256, lds, st>>>(c.at<float>(o.KVm), c.at<float>(o.Fm), c.at<float>(o.Coef),      \
                                                        c.at<float>(o.Aw), c.at<float>(o.DA), c.at<float>(o.Upd), c.at<float>(o.DV), \
                                                        c.at<float>(o.Part), lo, D.m, D.d, D.dm, Phi);                   \
    break;
    switch ((Phi + 63) / 64) { ARMT_UB(1) ARMT_UB(2) ARMT_UB(3) ARMT_UB(4) ARMT_UB(5) ARMT_UB(6) ARMT_UB(7) ARMT_UB(8) }
#undef ARMT_UB
    HIP_TRY(hipGetLastError());
    update_bwd_tokens_kernel<T><<<dim3(D.m, g), 128, (D.dm + Phi + 17) * 4, st>>>(
        c.at<float>(o.KVm), c.at<float>(o.Fm), c.at<float>(o.Coef), c.at<float>(o.Part), o.nblk, c.at<float>(o.DV),
        c.at<float>(o.zw), c.at<float>(o.DZ), lo, D.m, D.d, D.dm, D.nu, D.assoc_eps, c.at<T>(o.DKV), o.Kmkv, c.at<float>(o.DB),
        c.at<float>(o.DZF));
    HIP_TRY(hipGetLastError());
    update_bwd_z_kernel<<<dim3((Phi + 255) / 256, g), 256, 0, st>>>(c.at<float>(o.Fm), c.at<float>(o.DZF), c.at<float>(o.DZ), lo,
                                                                  D.m, Phi);
    HIP_TRY(hipGetLastError());
    ARMT_TRY(bgemm<T>(c, TK_DYM, lo, g));
    beta_bwd_kernel<T><<<dim3((D.d + 255) / 256, g), 256, 0, st>>>(c.at<float>(o.DB), Yop + (size_t)D.S * D.d, cell, c.aux,
                                                                 DX + B * cell + (size_t)D.S * D.d, cell, c.at<float>(o.CPart), lo,
                                                                 D.m, D.d);
    colsum_finish_kernel<<<dim3((D.d + 255) / 256, g / B), 256, 0, st>>>(c.at<float>(o.CPart), 1, c.dwb, nullptr, lo, D.d, B);
    HIP_TRY(hipGetLastError());
    const size_t tma = (size_t)(D.dm + D.d) * Km, tmb = (size_t)D.d * Km;
    ARMT_TRY(wtr(c.at<T>(o.DKV) + (size_t)lo * D.m * o.Kmkv, (size_t)D.m * o.Kmkv, o.Kmkv,
                 c.at<T>(o.TmA) + lo_r * tma + (size_t)slot * B * o.mp, tma, o.mp, Km, D.m, D.dm + D.d, g));
    ARMT_TRY(wtr(Yop + lo * cell + (size_t)D.S * D.d, cell, D.d, c.at<T>(o.TmB) + lo_r * tmb + (size_t)slot * B * o.mp, tmb, o.mp, Km,
                 D.m, D.d, g));
  }
  // ---- feed-forward half of the block
  T* DYb = c.at<T>(o.DYb) + lo * cell;
  convert_kernel<float, T><<<ew_blocks(g * cell), 256, 0, st>>>(DX + (lo + B) * cell, DYb, g * cell);
  HIP_TRY(hipGetLastError());
  ARMT_TRY(bgemm<T>(c, TK_DU, lo, g));
  ARMT_TRY(wtr(DYb, cell, D.d, arow(o.aDY), wa_cell, Tp, Kw, D.T, D.d, g));
  if (!std::is_same<T, bf16>::value)      // bf16: the recomputation wrote U^T already
    ARMT_TRY(wtr(c.at<T>(o.Uff) + (size_t)lo * D.T * D.F, (size_t)D.T * D.F, D.F, brow(o.bU), wb_cell, Tp, Kw, D.T, D.F, g));
  T* GU = c.at<T>(o.GU) + (size_t)lo * D.T * 2 * D.F;
  if constexpr (std::is_same<T, bf16>::value) {
    // [gate | up] <- [dgate | dup] in place, and transposed into the window rows of dW_gate, dW_up's A operand
    swiglu_tiles_kernel<true><<<dim3(D.F / 64, (D.T + 63) / 64, g), 256, 0, st>>>(
        (bf16*)GU, c.at<bf16>(o.DU) + (size_t)lo * D.T * D.F, D.T, D.F, 0, (bf16*)arow(o.aDGU), wa_cell, Kw, B, Tp);
  } else {
    swiglu_bwd_kernel<T><<<ew_blocks((size_t)g * D.T * D.F), 256, 0, st>>>(GU, c.at<T>(o.DU) + (size_t)lo * D.T * D.F, (size_t)g * D.T,
                                                                          D.F);
  }
  HIP_TRY(hipGetLastError());
  ARMT_TRY(bgemm<T>(c, TK_DN2, lo, g));
  if (!std::is_same<T, bf16>::value) ARMT_TRY(wtr(GU, (size_t)D.T * 2 * D.F, 2 * D.F, arow(o.aDGU), wa_cell, Tp, Kw, D.T, 2 * D.F, g));
  ARMT_TRY(wtr(c.at<T>(o.N2) + lo * cell, cell, D.d, brow(o.bN2), wb_cell, Tp, Kw, D.T, D.d, g));
  ARMT_TRY(colsum<T>(c, c.at<T>(o.DN), c.at<float>(o.Hres), cell, c.at<float>(o.RStd2), c.dg2, nullptr, lo, g, D.d));   // d gain 2
  rmsnorm_bwd_kernel<T><<<dim3(D.T, g), 256, 0, st>>>(c.at<T>(o.DN), c.at<float>(o.Hres), cell, c.aux, lo, 1, c.at<float>(o.RStd2),
                                                     DX + B * cell, cell, c.at<float>(o.DH), cell, c.at<T>(o.DHb), D.T, D.d);
  HIP_TRY(hipGetLastError());
  // ---- attention half
  ARMT_TRY(bgemm<T>(c, TK_DATT, lo, g));
  ARMT_TRY(wtr(c.at<T>(o.DHb) + lo * cell, cell, D.d, arow(o.aDH), wa_cell, Tp, Kw, D.T, D.d, g));
  ARMT_TRY(wtr(c.at<T>(o.Att) + lo * D.T * Hd, D.T * Hd, (int)Hd, brow(o.bATT), wb_cell, Tp, Kw, D.T, (int)Hd, g));
  const float scale = 1.0f / sqrtf((float)D.dh);
  if (mfma_attention_bwd<T>(D)) {
    HIP_TRY(launch_attention_bwd_mfma(c.at<bf16>(o.QKV), c.at<bf16>(o.Att), c.at<bf16>(o.DAtt), c.at<float>(o.LSE), c.at<float>(o.Dv),
                                      c.at<bf16>(o.AttS), c.at<bf16>(o.DQKV), lo, g, D.L, D.T, D.H, D.Hkv, D.dh, st));
  } else {
    attention_bwd_q_kernel<T><<<dim3(D.T, D.H, g), 64, (2 * D.dh + D.T) * 4, st>>>(c.at<T>(o.QKV), c.at<T>(o.Att), c.at<T>(o.DAtt),
                                                                                 c.at<T>(o.DQKV), c.at<float>(o.LSE),
                                                                                 c.at<float>(o.Dv), lo, D.T, D.H, D.Hkv, D.dh, scale);
    attention_bwd_kv_kernel<T><<<dim3(D.T, D.Hkv, g), 64, (2 * D.dh + 128) * 4, st>>>(c.at<T>(o.QKV), c.at<T>(o.DAtt), c.at<T>(o.DQKV),
                                                                                    c.at<float>(o.LSE), c.at<float>(o.Dv), lo, D.T,
                                                                                    D.H, D.Hkv, D.dh, scale);
  }
  rope_bwd_kernel<T><<<dim3(D.T, g), 256, 0, st>>>(c.at<T>(o.DQKV), c.at<float>(o.Rope), lo, D.T, D.H + D.Hkv, D.dh, D.Nqkv);
  HIP_TRY(hipGetLastError());
  ARMT_TRY(bgemm<T>(c, TK_DN1, lo, g));
  ARMT_TRY(wtr(c.at<T>(o.DQKV) + (size_t)lo * D.T * D.Nqkv, (size_t)D.T * D.Nqkv, D.Nqkv, arow(o.aDQKV), wa_cell, Tp, Kw, D.T, D.Nqkv, g));
  ARMT_TRY(wtr(c.at<T>(o.N1) + lo * cell, cell, D.d, brow(o.bN1), wb_cell, Tp, Kw, D.T, D.d, g));
  ARMT_TRY(colsum<T>(c, c.at<T>(o.DN), c.at<float>(o.X1), cell, c.at<float>(o.RStd1), c.dg1, nullptr, lo, g, D.d));     // d gain 1
  rmsnorm_bwd_kernel<T><<<dim3(D.T, g), 256, 0, st>>>(c.at<T>(o.DN), c.at<float>(o.X1), cell, c.aux, lo, 0, c.at<float>(o.RStd1),
                                                     c.at<float>(o.DH), cell, DX, cell, (T*)nullptr, D.T, D.d);
  HIP_TRY(hipGetLastError());
  // ---- associative read (Eq. 6)
  if (gr > 0) {
    read_bwd_rows_kernel<T><<<dim3(D.T, gr), 256, 0, st>>>(DX, cell, c.at<float>(o.X1), cell, c.at<float>(o.Xin), cell,
                                                          c.at<float>(o.RDen), lo, D.T, D.d, c.at<T>(o.DNum), c.at<float>(o.DDen));
    HIP_TRY(hipGetLastError());
    const size_t nA = (size_t)D.d * Phi;
    ARMT_TRY((transpose<float, T>(st, c.at<float>(o.Aw) + lo * nA, nA, Phi, c.at<T>(o.ATr) + lo * nA, nA, D.d, D.d, Phi, gr)));
    ARMT_TRY(bgemm<T>(c, TK_DF, lo, gr));
    read_bwd_dpfp_kernel<T><<<dim3(D.T, gr), 128, (D.dm + Phi) * 4, st>>>(c.at<float>(o.Qm), c.at<float>(o.DF), c.at<float>(o.DDen),
                                                                         c.aux, lo, D.T, D.dm, D.nu, c.at<T>(o.DQr), o.dmP);
    HIP_TRY(hipGetLastError());
    // dz += sum_i dden_i f_i over the rows of the cell
    ARMT_TRY(colsum<T>(c, c.at<T>(o.Fphi), nullptr, 0, c.at<float>(o.DDen), nullptr, c.at<float>(o.DZ), lo, gr, Phi));
    ARMT_TRY((transpose<T, T>(st, c.at<T>(o.DNum) + lo * cell, cell, D.d, TA, ta_cell, Tp, D.T, D.d, gr)));
    ARMT_TRY((transpose<T, T>(st, c.at<T>(o.Fphi) + (size_t)lo * D.T * Phi, (size_t)D.T * Phi, Phi, TB, tb_cell, Tp, D.T, Phi, gr)));
    ARMT_TRY(bgemm<T>(c, TK_DA, lo, gr));
    ARMT_TRY(bgemm<T>(c, TK_DXQ, lo, gr));
    ARMT_TRY(wtr(c.at<T>(o.DQr) + (size_t)lo * D.T * o.dmP, (size_t)D.T * o.dmP, o.dmP, arow(o.aDQR), wa_cell, Tp, Kw, D.T, D.dm, gr));
    ARMT_TRY(wtr(Xop + lo * cell, cell, D.d, brow(o.bX), wb_cell, Tp, Kw, D.T, D.d, gr));
  }
  return ARMT_OK;
}

template <typename T>
armt_status backward_typed(BCtx& c, const armt_layer_weights* W, int64_t N, float* tape, size_t rec_floats, bool carry_in,
                           const void* d_hidden, float* d_mem_emb, float* dx, bool diagonal) {
  const Dims& D = c.D;
  const TrainLayout& o = c.o;
  const int L = D.L, Lr = D.Lr, B = D.B;           // cells of a full step, layers, sequences
  const size_t cell = (size_t)D.T * D.d, nA = (size_t)D.d * D.Phi;
  const size_t seq = (size_t)N * D.S * D.d;        // elements of one sequence of d_hidden / dx
  {
    const int n = D.T * (D.dh / 2);
    rope_table_kernel<<<(n + 255) / 256, 256, 0, c.st>>>(c.at<float>(o.Rope), D.T, D.dh / 2, (double)D.rope_theta);
    // zero what is only ever written in part: the reduction padding of the transposed operands, the K padding of
    // dq and [dk | dv], and the gradient slots
    auto zero = [&](size_t off, size_t bytes) {
      fill_f32_kernel<<<ew_blocks(bytes / 4), 256, 0, c.st>>>(c.at<float>(off), bytes / 4, 0.f);
    };
    zero(o.TA, (size_t)L * o.ta_rows * o.Tp * D.esz);
    zero(o.TB, (size_t)L * o.tb_rows * o.Tp * D.esz);
    zero(o.TmA, (size_t)Lr * (D.dm + D.d) * o.Km * D.esz);
    zero(o.TmB, (size_t)Lr * D.d * o.Km * D.esz);
    zero(o.WinA, (size_t)Lr * o.wa_rows * o.Kw * D.esz);
    zero(o.WinB, (size_t)Lr * o.wb_rows * o.Kw * D.esz);
    zero(o.DQr, (size_t)L * D.T * o.dmP * D.esz);
    zero(o.DKV, (size_t)L * D.m * o.Kmkv * D.esz);
    zero(o.DX, (size_t)(L + B) * cell * 4);
    if (D.bf16) zero(o.Vt, attention_vt_bytes(D.L, D.T, D.Hkv, D.dh));
    HIP_TRY(hipGetLastError());
  }
  ARMT_TRY(transpose_weights<T>(c, W));

  // window of steps whose weight-gradient operands are waiting in the slot buffers
  const int win = diagonal ? WG_WIN : 1;       // cell-by-cell order: a step has one layer, nothing to gain from waiting
  struct Slot { int lo, hi, no_read; };        // live layers of the step; the layer whose cell had no read (-1: none)
  Slot slots[WG_WIN];
  int n_slots = 0;
  auto clear_slot = [&](int l, int p, bool read_only) {
    // zero slot p of layer l on the A side (then the stale B side of that slot adds nothing)
    const size_t e = D.esz, rowb = (size_t)o.Kw * e, colb = (size_t)B * o.Tp * e;
    char* WA = c.ws + o.WinA + (size_t)l * o.wa_rows * rowb + (size_t)p * colb;
    const size_t r0 = read_only ? o.aDQR : 0, nr = read_only ? (size_t)D.dm : o.wa_rows;
    zero_columns_kernel<<<dim3((unsigned)nr), 256, 0, c.st>>>(WA + r0 * rowb, rowb, colb);
    if (!read_only) {
      const size_t mrow = (size_t)o.Km * e, mcol = (size_t)B * o.mp * e;
      zero_columns_kernel<<<dim3((unsigned)(D.dm + D.d)), 256, 0, c.st>>>(c.ws + o.TmA + (size_t)l * (D.dm + D.d) * mrow + (size_t)p * mcol,
                                                                         mrow, mcol);
    }
  };
  auto flush = [&]() -> armt_status {
    if (n_slots == 0) return ARMT_OK;
    int LO = slots[0].lo, HI = slots[0].hi;
    for (int p = 1; p < n_slots; ++p) { LO = std::min(LO, slots[p].lo); HI = std::max(HI, slots[p].hi); }
    for (int p = 0; p < n_slots; ++p) {
      for (int l = LO; l <= HI; ++l)
        if (l < slots[p].lo || l > slots[p].hi) clear_slot(l, p, false);
      if (slots[p].no_read >= 0) clear_slot(slots[p].no_read, p, true);
    }
    HIP_TRY(hipGetLastError());
    const int kinds[] = {TK_WD, TK_WG, TK_WU, TK_WO, TK_WQ, TK_WK, TK_WV, TK_WMQ, TK_WMK, TK_WMV};
    for (int k : kinds) {
      GemmShape s = c.shape[k];
      s.K = n_slots * B * ((k == TK_WMK || k == TK_WMV) ? o.mp : o.Tp);
      ARMT_TRY(gemm<T>(c.st, c.table(k), LO, HI - LO + 1, s));
    }
    n_slots = 0;
    return ARMT_OK;
  };

  auto step = [&](int lo, int hi, int t) -> armt_status {       // layers lo .. hi, each on segment t - layer
    const int gc = (hi - lo + 1) * B, loc = lo * B;              // the cells of these layers: layer * B + sequence
    // the cells of segment 0 met an empty memory unless a state was carried in
    const bool top_empty = !carry_in && (t - hi) == 0;
    const int grc = top_empty ? gc - B : gc;
    tape_kernel<<<dim3(128, gc), 256, 0, c.st>>>(tape, rec_floats, c.at<float>(o.Xin), cell, c.aux, c.at<float>(o.Aw),
                                                c.at<float>(o.zw), loc, t, L, B, cell, nA, (size_t)D.Phi, 0);
    if (hi == Lr - 1) {
      const int64_t s = t - (Lr - 1);
      for (int b = 0; b < B; ++b)
        load_dhidden_kernel<T><<<D.T, 256, 0, c.st>>>((const T*)d_hidden + b * seq + (size_t)s * D.S * D.d, D.S, D.d,
                                                     c.at<float>(o.DX) + (size_t)(L + b) * cell);
    }
    HIP_TRY(hipGetLastError());
    ARMT_TRY(recompute_group<T>(c, loc, gc, grc, top_empty ? hi * B : -1, top_empty ? (hi + 1) * B : -1, n_slots));
    ARMT_TRY(backward_group<T>(c, loc, gc, grc, n_slots));
    slots[n_slots++] = Slot{lo, hi, top_empty ? hi : -1};
    if (n_slots == win) ARMT_TRY(flush());
    if (lo == 0) {
      for (int b = 0; b < B; ++b)
        store_dx_kernel<<<D.T, 256, 0, c.st>>>(c.at<float>(o.DX) + (size_t)b * cell, D.S, D.d,
                                               dx ? dx + b * seq + (size_t)t * D.S * D.d : nullptr, d_mem_emb);
      HIP_TRY(hipGetLastError());
    }
    return ARMT_OK;
  };
  if (diagonal) {
    for (int64_t t = Lr + N - 2; t >= 0; --t) {
      int32_t lo, hi;
      armt_diagonal_group(Lr, (int32_t)N, (int32_t)t, &lo, &hi);
      ARMT_TRY(step(lo, hi, (int)t));
    }
  } else {
    for (int64_t s = N - 1; s >= 0; --s)
      for (int l = Lr - 1; l >= 0; --l) ARMT_TRY(step(l, l, (int)s + l));
  }
  return flush();
}

}  // namespace

extern "C" {

size_t armt_tape_bytes_batched(const armt_config* cfg, int32_t batch, int64_t n_tokens) {
  Dims D;
  if (check_backward_config(cfg, &D) != ARMT_OK || n_tokens <= 0 || n_tokens % D.S != 0) return 0;
  if (batch < 1 || (int64_t)batch * D.L > 32768) return 0;
  return (size_t)(n_tokens / D.S) * D.L * batch * tape_record_floats(D) * 4;
}
size_t armt_tape_bytes(const armt_config* cfg, int64_t n_tokens) { return armt_tape_bytes_batched(cfg, 1, n_tokens); }

size_t armt_backward_workspace_bytes_batched(const armt_config* cfg, int32_t batch) {
  Dims D;
  if (check_backward_config(cfg, &D) != ARMT_OK || batch < 1 || (int64_t)batch * D.L > 32768) return 0;
  D.B = batch;
  D.L = D.Lr * batch;
  return carve_train(D).total;
}
size_t armt_backward_workspace_bytes(const armt_config* cfg) { return armt_backward_workspace_bytes_batched(cfg, 1); }

armt_status armt_forward_train_batched(const armt_config* cfg, const armt_layer_weights* layers, const void* mem_emb,
                                       const void* x, int32_t batch, int64_t n_tokens, const float* A_in, const float* z_in,
                                       void* hidden_out, float* A_out, float* z_out, void* tape, size_t tape_bytes,
                                       void* workspace, size_t workspace_bytes, void* hip_stream, int32_t diagonal) {
  Dims D;
  ARMT_TRY(check_backward_config(cfg, &D));
  if (!tape) return ARMT_ERR_NULL;
  if (n_tokens <= 0 || n_tokens % D.S != 0 || batch < 1 || (int64_t)batch * D.L > 32768) return ARMT_ERR_SHAPE;
  if (((uintptr_t)tape % kAlign) != 0 || tape_bytes < armt_tape_bytes_batched(cfg, batch, n_tokens)) return ARMT_ERR_WORKSPACE;
  return forward_impl(cfg, layers, mem_emb, x, batch, n_tokens, A_in, z_in, hidden_out, A_out, z_out, workspace, workspace_bytes,
                      hip_stream, diagonal != 0, (float*)tape, tape_record_floats(D));
}
armt_status armt_forward_train(const armt_config* cfg, const armt_layer_weights* layers, const void* mem_emb, const void* x,
                               int64_t n_tokens, const float* A_in, const float* z_in, void* hidden_out, float* A_out,
                               float* z_out, void* tape, size_t tape_bytes, void* workspace, size_t workspace_bytes,
                               void* hip_stream, int32_t diagonal) {
  return armt_forward_train_batched(cfg, layers, mem_emb, x, 1, n_tokens, A_in, z_in, hidden_out, A_out, z_out, tape, tape_bytes,
                                    workspace, workspace_bytes, hip_stream, diagonal);
}

armt_status armt_backward_batched(const armt_config* cfg, const armt_layer_weights* layers, int32_t batch, int64_t n_tokens,
                                  const void* tape, size_t tape_bytes, int32_t carry_in, const void* d_hidden, const float* dA_out,
                                  const float* dz_out, const armt_layer_grads* grads, float* d_mem_emb, float* dx, float* dA_in,
                                  float* dz_in, void* workspace, size_t workspace_bytes, void* hip_stream, int32_t diagonal) {
  BCtx c;
  ARMT_TRY(check_backward_config(cfg, &c.D));
  const Dims& D = c.D;
  if (!layers || !tape || !d_hidden || !grads || !d_mem_emb) return ARMT_ERR_NULL;
  for (int l = 0; l < D.Lr; ++l) {
    const armt_layer_weights& w = layers[l];
    const armt_layer_grads& g = grads[l];
    if (!w.rms1 || !w.wq || !w.wk || !w.wv || !w.wo || !w.rms2 || !w.wgate || !w.wup || !w.wdown || !w.wm_q || !w.wm_k ||
        !w.wm_v || !w.wm_b)
      return ARMT_ERR_NULL;
    if (!g.rms1 || !g.wq || !g.wk || !g.wv || !g.wo || !g.rms2 || !g.wgate || !g.wup || !g.wdown || !g.wm_q || !g.wm_k ||
        !g.wm_v || !g.wm_b)
      return ARMT_ERR_NULL;
  }
  if (n_tokens <= 0 || n_tokens % D.S != 0 || batch < 1 || (int64_t)batch * D.Lr > 32768) return ARMT_ERR_SHAPE;
  const int64_t N = n_tokens / D.S;
  if (N + D.Lr > (int64_t)1 << 30) return ARMT_ERR_SHAPE;
  if ((dA_out == nullptr) != (dz_out == nullptr) || (dA_in == nullptr) != (dz_in == nullptr)) return ARMT_ERR_NULL;
  if (((uintptr_t)tape % kAlign) != 0 || tape_bytes < armt_tape_bytes_batched(cfg, batch, n_tokens)) return ARMT_ERR_WORKSPACE;
  c.D.B = batch;
  c.D.L = D.Lr * batch;                    // from here on L counts the cells of a full step
  c.o = carve_train(D);
  if (!workspace || ((uintptr_t)workspace % kAlign) != 0 || workspace_bytes < c.o.total) return ARMT_ERR_WORKSPACE;
  c.ws = (char*)workspace;
  c.st = (hipStream_t)hip_stream;
  fill_train_shapes(c);
  ARMT_TRY(upload_train_tables(c, layers, grads));
  // the caller's state gradients are [batch][layers][...]; the cells of a step are ordered layer-major
  const size_t nA = (size_t)D.d * D.Phi, nz = (size_t)D.Phi;
  if (dA_out) {
    state_permute_kernel<<<dim3(64, D.L), 256, 0, c.st>>>(c.at<float>(c.o.DA), dA_out, D.Lr, batch, nA, 1);
    state_permute_kernel<<<dim3(1, D.L), 256, 0, c.st>>>(c.at<float>(c.o.DZ), dz_out, D.Lr, batch, nz, 1);
  } else {
    fill_f32_kernel<<<1024, 256, 0, c.st>>>(c.at<float>(c.o.DA), nA * D.L, 0.f);
    fill_f32_kernel<<<16, 256, 0, c.st>>>(c.at<float>(c.o.DZ), nz * D.L, 0.f);
  }
  HIP_TRY(hipGetLastError());
  armt_status rc;
  if (D.bf16)
    rc = backward_typed<bf16>(c, layers, N, (float*)const_cast<void*>(tape), tape_record_floats(D), carry_in != 0, d_hidden,
                              d_mem_emb, dx, diagonal != 0);
  else
    rc = backward_typed<float>(c, layers, N, (float*)const_cast<void*>(tape), tape_record_floats(D), carry_in != 0, d_hidden,
                               d_mem_emb, dx, diagonal != 0);
  if (rc != ARMT_OK) return rc;
  if (dA_in) {
    state_permute_kernel<<<dim3(64, D.L), 256, 0, c.st>>>(dA_in, c.at<float>(c.o.DA), D.Lr, batch, nA, 0);
    state_permute_kernel<<<dim3(1, D.L), 256, 0, c.st>>>(dz_in, c.at<float>(c.o.DZ), D.Lr, batch, nz, 0);
    HIP_TRY(hipGetLastError());
  }
  return ARMT_OK;
}
armt_status armt_backward(const armt_config* cfg, const armt_layer_weights* layers, int64_t n_tokens, const void* tape,
                          size_t tape_bytes, int32_t carry_in, const void* d_hidden, const float* dA_out, const float* dz_out,
                          const armt_layer_grads* grads, float* d_mem_emb, float* dx, float* dA_in, float* dz_in,
                          void* workspace, size_t workspace_bytes, void* hip_stream, int32_t diagonal) {
  return armt_backward_batched(cfg, layers, 1, n_tokens, tape, tape_bytes, carry_in, d_hidden, dA_out, dz_out, grads, d_mem_emb, dx,
                               dA_in, dz_in, workspace, workspace_bytes, hip_stream, diagonal);
}

}  // extern "C"

// ---- backward of the token-level ends (final RMSNorm + head, embedding gather)
namespace {

constexpr int64_t kHeadBwdRows = 8192;     // rows per pass: the head's weight gradient (V x d fp32) is read and written once per pass
struct HeadBwdLayout { size_t WT, Nn, rstd, DLb, U, DLT, NT, CPart, table, total; int Vp, Rp; int64_t ch; };
HeadBwdLayout head_bwd_layout(const Dims& D, int64_t n_rows, int vocab) {
  HeadBwdLayout h;
  h.ch = std::min<int64_t>(n_rows, kHeadBwdRows);
  h.Vp = round64(vocab);
  h.Rp = round64((int)h.ch);
  size_t off = 0;
  auto take = [&](size_t bytes) { const size_t at = off; off += (bytes + kAlign - 1) / kAlign * kAlign; return at; };
  h.WT = take((size_t)D.d * h.Vp * D.esz);
  h.Nn = take((size_t)h.ch * D.d * D.esz);
  h.rstd = take((size_t)h.ch * 4);
  h.DLb = take((size_t)h.ch * h.Vp * D.esz);
  h.U = take((size_t)h.ch * D.d * 4);
  h.DLT = take((size_t)h.Vp * h.Rp * D.esz);
  h.NT = take((size_t)D.d * h.Rp * D.esz);
  h.CPart = take((size_t)CS_CHUNKS * D.d * 4);
  h.table = take(2 * sizeof(GemmGroup));
  h.total = off;
  return h;
}

template <typename T>
armt_status lm_head_backward_typed(const Dims& D, const HeadBwdLayout& h, const void* hidden, int64_t n_rows, const void* gain,
                                   const void* w_lm, int32_t vocab, const float* d_logits, float* d_hidden, float* d_gain,
                                   float* d_w, char* ws, hipStream_t st) {
  T* WT = (T*)(ws + h.WT);
  T* Nn = (T*)(ws + h.Nn);
  float* rstd = (float*)(ws + h.rstd);
  T* DLb = (T*)(ws + h.DLb);
  float* U = (float*)(ws + h.U);
  T* DLT = (T*)(ws + h.DLT);
  T* NT = (T*)(ws + h.NT);
  float* part = (float*)(ws + h.CPart);
  auto zero = [&](void* p, size_t bytes) { fill_f32_kernel<<<ew_blocks(bytes / 4), 256, 0, st>>>((float*)p, bytes / 4, 0.f); };
  zero(WT, (size_t)D.d * h.Vp * D.esz);                    // the padding of the vocabulary dimension must read as zero
  HIP_TRY(hipGetLastError());
  ARMT_TRY((transpose<T, T>(st, (const T*)w_lm, 0, D.d, WT, 0, h.Vp, vocab, D.d, 1)));
  std::vector<GemmGroup> tab(2);
  memset(tab.data(), 0, tab.size() * sizeof(GemmGroup));
  tab[0].A = DLb; tab[0].B0 = WT; tab[0].C = U;                               // u = dL W
  tab[1].A = DLT; tab[1].B0 = NT; tab[1].C = d_w; tab[1].R = d_w;             // dW += dL^T n
  ARMT_TRY(upload_bytes(st, ws + h.table, tab.data(), tab.size() * sizeof(GemmGroup)));
  const GemmGroup* table = (const GemmGroup*)(ws + h.table);
  GemmShape su, sw;
  su.M = 0; su.N = D.d; su.K = h.Vp; su.lda = h.Vp; su.ldb = h.Vp; su.ldc = D.d; su.ldc2 = 0; su.ldr = 0; su.n0 = D.d; su.n1 = 0;
  su.epi = EPI_STORE_F32; su.tag = -1; su.dbg = 0;
  sw.M = vocab; sw.N = D.d; sw.K = 0; sw.lda = h.Rp; sw.ldb = h.Rp; sw.ldc = D.d; sw.ldc2 = 0; sw.ldr = D.d; sw.n0 = D.d; sw.n1 = 0;
  sw.epi = EPI_RESID_F32; sw.tag = -1; sw.dbg = 0;
  int64_t last_r = -1;
  for (int64_t r0 = 0; r0 < n_rows; r0 += h.ch) {
    const int r = (int)std::min<int64_t>(h.ch, n_rows - r0);
    const T* hs = (const T*)hidden + (size_t)r0 * D.d;
    if (r != last_r) {      // columns past this pass's rows must be zero in both transposed operands
      zero(DLT, (size_t)h.Vp * h.Rp * D.esz);
      zero(NT, (size_t)D.d * h.Rp * D.esz);
      last_r = r;
    }
    final_norm_train_kernel<T><<<r, 256, 0, st>>>(hs, (const T*)gain, D.d, D.rms_eps, Nn, rstd);
    pad_convert_rows_kernel<T><<<r, 256, 0, st>>>(d_logits + (size_t)r0 * vocab, vocab, DLb, h.Vp);
    HIP_TRY(hipGetLastError());
    su.M = r;
    ARMT_TRY(gemm<T>(st, table, 0, 1, su));
    final_norm_bwd_kernel<T><<<r, 256, 0, st>>>(U, hs, (const T*)gain, rstd, D.d, d_hidden + (size_t)r0 * D.d);
    colsum_partial_kernel<T><<<dim3((D.d + 255) / 256, 1, CS_CHUNKS), 256, 0, st>>>(hs, U, 0, rstd, part, 0, r, D.d);
    colsum_finish_kernel<<<dim3((D.d + 255) / 256, 1), 256, 0, st>>>(part, CS_CHUNKS, nullptr, d_gain, 0, D.d, 1);
    HIP_TRY(hipGetLastError());
    ARMT_TRY((transpose<T, T>(st, DLb, 0, h.Vp, DLT, 0, h.Rp, r, h.Vp, 1)));
    ARMT_TRY((transpose<T, T>(st, Nn, 0, D.d, NT, 0, h.Rp, r, D.d, 1)));
    sw.K = round64(r);
    ARMT_TRY(gemm<T>(st, table, 1, 1, sw));
  }
  return ARMT_OK;
}

}  // namespace

extern "C" {

size_t armt_lm_head_backward_workspace_bytes(const armt_config* cfg, int64_t n_rows, int32_t vocab) {
  Dims D;
  if (check_config(cfg, &D) != ARMT_OK || n_rows < 1 || vocab < 1) return 0;
  return head_bwd_layout(D, n_rows, vocab).total;
}

armt_status armt_lm_head_backward(const armt_config* cfg, const void* hidden, int64_t n_rows, const void* final_gain,
                                  const void* w_lm, int32_t vocab, const float* d_logits, float* d_hidden, float* d_final_gain,
                                  float* d_w_lm, void* workspace, size_t workspace_bytes, void* hip_stream) {
  Dims D;
  ARMT_TRY(check_config(cfg, &D));
  if (!hidden || !final_gain || !w_lm || !d_logits || !d_hidden || !d_final_gain || !d_w_lm) return ARMT_ERR_NULL;
  if (n_rows < 1 || n_rows > 0x7fffffff || vocab < 1) return ARMT_ERR_SHAPE;
  const HeadBwdLayout h = head_bwd_layout(D, n_rows, vocab);
  if (!workspace || ((uintptr_t)workspace % kAlign) != 0 || workspace_bytes < h.total) return ARMT_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)hip_stream;
  if (D.bf16)
    return lm_head_backward_typed<bf16>(D, h, hidden, n_rows, final_gain, w_lm, vocab, d_logits, d_hidden, d_final_gain, d_w_lm,
                                        (char*)workspace, st);
  return lm_head_backward_typed<float>(D, h, hidden, n_rows, final_gain, w_lm, vocab, d_logits, d_hidden, d_final_gain, d_w_lm,
                                       (char*)workspace, st);
}

armt_status armt_embed_tokens_backward(const armt_config* cfg, const float* dx, const int32_t* ids, int64_t n_tokens, int32_t vocab,
                                       float* d_emb_table, void* hip_stream) {
  Dims D;
  ARMT_TRY(check_config(cfg, &D));
  if (!dx || !ids || !d_emb_table) return ARMT_ERR_NULL;
  if (vocab < 1 || n_tokens < 1 || n_tokens > 0x7fffffff) return ARMT_ERR_SHAPE;
  embed_bwd_kernel<<<(unsigned)n_tokens, 256, 0, (hipStream_t)hip_stream>>>(dx, ids, vocab, D.d, d_emb_table);
  HIP_TRY(hipGetLastError());
  return ARMT_OK;
}

}  // extern "C"
