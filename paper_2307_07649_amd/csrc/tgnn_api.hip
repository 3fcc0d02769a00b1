// C-ABI entry points of libtgnn: argument validation, workspace layout, and the stream-ordered kernel
// sequence of each call.  See include/tgnn.h for the contract of every function.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <new>
#include <vector>

#include "tgnn_internal.h"

namespace tgnn {

static thread_local char g_err[512] = "";

int set_error(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

#define REQ_PTR(p)                                                                      \
  do {                                                                                  \
    if ((p) == nullptr) return tgnn::set_error(TGNN_E_NULL_PTR, "%s is NULL", #p);      \
    if (!tgnn::aligned16(p)) return tgnn::set_error(TGNN_E_MISALIGNED, "%s is not 16-byte aligned", #p); \
  } while (0)
#define OPT_PTR(p)                                                                      \
  do {                                                                                  \
    if ((p) != nullptr && !tgnn::aligned16(p))                                          \
      return tgnn::set_error(TGNN_E_MISALIGNED, "%s is not 16-byte aligned", #p);       \
  } while (0)

static int check_params(const tgnn_params* p, const char* what) {
  if (p == nullptr) return set_error(TGNN_E_NULL_PTR, "%s is NULL", what);
  const float* const* f = reinterpret_cast<const float* const*>(p);
  static const char* names[] = {"time_w", "time_b", "gru_wih", "gru_whh", "gru_bih", "gru_bhh", "wq", "bq", "wk", "bk",
                                "wv", "bv", "wo", "bo", "dec_ws", "dec_wd", "dec_b1", "dec_w2", "dec_b2"};
  for (int i = 0; i < 19; ++i) {
    if (f[i] == nullptr) return set_error(TGNN_E_NULL_PTR, "%s.%s is NULL", what, names[i]);
    if (!aligned16(f[i])) return set_error(TGNN_E_MISALIGNED, "%s.%s is not 16-byte aligned", what, names[i]);
  }
  return TGNN_OK;
}

static int check_graph(const tgnn_ctx* ctx, const tgnn_graph* g) {
  if (g == nullptr) return set_error(TGNN_E_NULL_PTR, "graph is NULL");
  REQ_PTR(g->indptr);
  REQ_PTR(g->nbr);
  REQ_PTR(g->eid);
  REQ_PTR(g->ts);
  if (ctx->d.de > 0) REQ_PTR(g->efeat);
  if (g->n_events < 0) return set_error(TGNN_E_INVALID_ARG, "graph.n_events < 0");
  return TGNN_OK;
}

static int check_state(const tgnn_ctx* ctx, const tgnn_state* st) {
  if (st == nullptr) return set_error(TGNN_E_NULL_PTR, "state is NULL");
  REQ_PTR(st->mem);
  REQ_PTR(st->mem_ts);
  REQ_PTR(st->mail);
  REQ_PTR(st->mail_ts);
  REQ_PTR(st->mail_eid);
  if (ctx->d.ds > 0) REQ_PTR(st->stat);
  return TGNN_OK;
}

// Bump allocator over the arena; first pass (base == nullptr) only measures.
struct Bump {
  char* base;
  size_t off = 0;
  template <typename T>
  T* take(size_t n) {
    off = (off + 255) & ~size_t(255);
    T* p = base ? reinterpret_cast<T*>(base + off) : nullptr;
    off += n * sizeof(T);
    return p;
  }
};

static void layout(const Dims& d, Ws& w, Bump& b) {
  const size_t R = d.maxR, RK = d.maxRK, S = d.maxS, B2 = (1 + (size_t)d.maxNeg) * d.maxEv;
  w.root_node = b.take<int32_t>(R);
  w.root_t = b.take<double>(R);
  w.nbr = b.take<int32_t>(RK); w.neid = b.take<int32_t>(RK); w.cnt = b.take<int32_t>(R); w.nts = b.take<double>(RK);
  w.slot_gid = b.take<int32_t>(S); w.slot_node = b.take<int32_t>(S); w.has = b.take<int32_t>(S);
  w.tau = b.take<double>(S); w.delta = b.take<double>(S); w.dtk = b.take<double>(RK);
  w.winkey = b.take<unsigned long long>((size_t)d.nrep * d.N);
  w.epoch = b.take<unsigned long long>(1);
  w.bad_ids = b.take<int32_t>(1);
  const size_t NG = (size_t)d.nrep * d.N, U = d.maxU;
  w.utag = b.take<unsigned long long>(NG); w.uidx = b.take<int32_t>(NG); w.ucount_pair = b.take<int32_t>(2); w.ucount = w.ucount_pair;
  w.ulist = b.take<int32_t>(U); w.slot_row = b.take<int32_t>(S); w.ucnt = b.take<int32_t>(U);
  w.rowptr = b.take<int32_t>(U + 1); w.cursor = b.take<int32_t>(U); w.sorted = b.take<int32_t>(S);
  w.sorted_row = b.take<int32_t>(S); w.sort_total = b.take<int32_t>(1);
  w.ds_row = b.take<float>(S * d.ldh);
  w.dstat = d.ds > 0 ? b.take<float>(S * d.ldst) : nullptr;
  w.adam_dev = b.take<AdamSet>(1); w.adam_t = b.take<int32_t>(1);
  w.bs_dev = b.take<BatchSet>(1);
  w.sgd_dev = b.take<SgdSet>(1);
  w.q_part = b.take<float>((size_t)QPHI_BLOCKS * d.dO);
  w.X = b.take<float>(S * d.ldx); w.Hm = b.take<float>(S * d.ldh);
  w.gi = b.take<float>(S * d.ld3); w.gh = b.take<float>(S * d.ld3);
  w.gates = b.take<float>(S * 4 * d.ldh); w.Xrow = b.take<float>(S * d.ldxr);
  w.dgi = b.take<float>(S * d.ld3); w.dgh = b.take<float>(S * d.ld3);
  // node rows of a standalone attention call are its slots, so P / dP hold S rows (a step uses far fewer)
  w.P = b.take<float>(S * d.ldp); w.dP = b.take<float>(S * d.ldp);
  w.Umat = b.take<float>(S * d.ldz);
  w.prob = b.take<float>(R * d.H * d.k); w.Onode = b.take<float>(R * d.ldh); w.Omat = b.take<float>(R * d.ldh);
  w.z = b.take<float>(R * d.ldh);
  w.dz = b.take<float>(R * d.ldh); w.dOmat = b.take<float>(R * d.ldh); w.dqn = b.take<float>(R * d.ldh);
  w.dq = b.take<float>(R * d.ldh); w.Gmat = b.take<float>(R * d.ldz);
  w.Zs = b.take<float>(R * d.ldz); w.Zp = b.take<float>(R * d.ldz); w.Qroot = b.take<float>(R * d.ldh);
  w.Yt = b.take<float>(R * d.ldy);
  w.dscore = b.take<float>(R * d.H * d.k);
  w.Pdec = b.take<float>(R * d.ldkv); w.dPdec = b.take<float>(R * d.ldkv);
  w.h1 = b.take<float>(B2 * d.ldh);
  w.logits = b.take<float>(std::max(B2, (size_t)d.maxEv * (size_t)d.nC));
  w.dlog = b.take<float>(d.nC > 0 ? (size_t)d.maxEv * d.ldc : 4);
  w.loss_acc = b.take<float>(TGNN_MAX_BATCHES);
  w.Wih_p = b.take<float>((size_t)3 * d.dm * d.ldx); w.Whh_p = b.take<float>((size_t)3 * d.dm * d.ldh);
  w.Wdec_p = b.take<float>((size_t)2 * d.dO * d.ldh);
  w.Wx = b.take<float>((size_t)d.ldp * d.ldxr); w.bias_x = b.take<float>((size_t)d.ldp);
  w.WkcT = b.take<float>((size_t)d.H * d.dcp * d.ldh + 32); w.WvcT = b.take<float>((size_t)d.H * d.dcp * d.ldh + 32);
  w.Wkc = b.take<float>((size_t)d.dO * d.ldz); w.Wvc = b.take<float>((size_t)d.dO * d.ldz);
  w.Wo_o = b.take<float>((size_t)d.dO * d.ldh);
  {
    const size_t ks = (size_t)(d.dO + 15) / 16;
    w.rc_pk = root_chain_fits(d) ? b.take<float>(6 * ks * ks * 256) : nullptr;
  }
  w.WdecT = b.take<float>((size_t)d.dO * d.ldkv); w.WihT_phi = b.take<float>((size_t)d.dt * d.ld3);
  w.WxT = b.take<float>((size_t)d.dx * d.ldp);
  w.WoT_o = b.take<float>((size_t)d.dO * d.ldh);
  b.take<char>(256);
}

static OutMap single_out(float* g, int ld, float* bias) {
  OutMap o;
  memset(&o, 0, sizeof(o));
  o.p[0][0] = g; o.ld[0][0] = ld;
  o.n_split = 1 << 30; o.k_split = 1 << 30;
  o.bias[0] = bias;
  return o;
}

// Fork/join between the caller's stream and the context's side stream.
struct Side {
  tgnn_ctx* c;
  hipStream_t main;
  bool on;
  hipStream_t stream() const { return on ? c->side : main; }
  hipEvent_t next() { hipEvent_t e = c->fork_ev[c->next_ev]; c->next_ev = (c->next_ev + 1) & 15; return e; }
  void fork() {   // side continues after everything queued on main so far
    if (!on) return;
    hipEvent_t e = next();
    (void)hipEventRecord(e, main);
    (void)hipStreamWaitEvent(c->side, e, 0);
  }
  void join() {   // main continues after everything queued on side so far
    if (!on) return;
    hipEvent_t e = next();
    (void)hipEventRecord(e, c->side);
    (void)hipStreamWaitEvent(main, e, 0);
  }
};

// Records a pair of events around a stage when its bit is set in the profiler mask.
struct StageTimer {
  tgnn_ctx* c;
  hipStream_t s;
  bool on(int st) const { return (c->prof.active >> st) & 1u && c->prof.count[st] < PROF_RING; }
  void begin(int st, hipStream_t on_stream) { hipStream_t keep = s; s = on_stream; begin(st); s = keep; }
  void end(int st, hipStream_t on_stream) { hipStream_t keep = s; s = on_stream; end(st); s = keep; }
  void begin(int st) {
    if (!on(st)) return;
    Profiler& pr = c->prof;
    for (int e = 0; e < 2; ++e)
      if (pr.ev[st][e] == nullptr) {
        pr.ev[st][e] = new hipEvent_t[PROF_RING];
        for (int i = 0; i < PROF_RING; ++i) (void)hipEventCreate(&pr.ev[st][e][i]);
      }
    (void)hipEventRecord(pr.ev[st][0][pr.count[st]], s);
  }
  void end(int st) {
    if (!on(st)) return;
    Profiler& pr = c->prof;
    (void)hipEventRecord(pr.ev[st][1][pr.count[st]], s);
    pr.count[st]++;
  }
};

// UPDT on n rows already staged in ws.X / ws.Hm / ws.has: projections (MFMA) + gates; s' goes to ws.Xrow.
static void gru_forward(tgnn_ctx* ctx, const tgnn_params* p, int n, hipStream_t s) {
  const Dims& d = ctx->d; Ws& w = ctx->w;
  const NtProblem pr[2] = {
      nt_live(nt_problem(w.X, d.ldx, w.Wih_p, d.ldx, p->gru_bih, w.gi, d.ld3, n, 3 * d.dm, d.ldx, d.ld3, false), d.d_in),
      nt_live(nt_problem(w.Hm, d.ldh, w.Whh_p, d.ldh, p->gru_bhh, w.gh, d.ld3, n, 3 * d.dm, d.ldh, d.ld3, false), d.dm)};
  gemm_nt_group(pr, 2, s);
  gru_gates_fwd(gru_gates_args(d, n, nullptr, w.gi, w.gh, w.Hm, w.has, w.gates, w.Xrow, d.ldxr, nullptr, nullptr, nullptr, 0), s);
}

// What the attention kernels need to know about a call.  slot_row maps root slot r and neighbour slot R + r k + j
// to node rows (NULL: slot = row).  efeat / neid / dt_in: see FusedAttn.
struct AttnIn {
  const int32_t* slot_row;
  const int32_t* cnt;
  const float* efeat;
  const int32_t* neid;
  const double* dt_in;
  const tgnn_params* p;
};

static FusedAttn fused_args(tgnn_ctx* ctx, int R, const AttnIn& in) {
  const Dims& d = ctx->d; Ws& w = ctx->w;
  FusedAttn a;
  memset(&a, 0, sizeof(a));
  a.R = R; a.k = d.k; a.H = d.H; a.dO = d.dO; a.dh = d.dO / d.H; a.de = d.de; a.dt = d.dt; a.dcp = d.dcp;
  a.ldz = d.ldz; a.ldh = d.ldh; a.ldp = d.ldp; a.ldy = d.ldy; a.off_q = d.ldkv; a.dt_source = d.dt_source;
  a.force_generic = (ctx->cfg.flags & TGNN_FLAG_GENERIC_ATTN) != 0;
  a.P = w.P; a.U = w.Umat; a.slot_row = in.slot_row; a.cnt = in.cnt; a.efeat = in.efeat; a.neid = in.neid;
  a.root_t = w.root_t; a.nts = w.nts; a.tau = w.tau; a.dt_in = in.dt_in;
  a.time_w = in.p->time_w; a.time_b = in.p->time_b; a.dtk = w.dtk; a.prob = w.prob;
  a.Onode = w.Onode; a.Zp = w.Zp; a.dOmat = w.dOmat; a.G = w.Gmat;
  a.dscore = w.dscore; a.dqn = w.dqn; a.Zs = w.Zs; a.Y = w.Yt; a.Qroot = w.Qroot;
  return a;
}

// Attention (Eq. 4-7) and the merge layer, from the node rows ws.Xrow [n_rows].  Every projection is linear in
// {x | e | Phi}, and x depends on the node only, so the x part of K, V, q and of the merge layer is one GEMM over the
// distinct node rows (ws.P).  The {e | Phi} part never becomes a key or value row (k_attn.hip): the scores need
// U = q (W_k^c) per head (a second GEMM over the node rows), the output is the kernel's node part plus Zp (W_v^c)^T
// (a GEMM over the roots).  n_rows_dev (may be NULL): device-side row count.
static void attn_forward(tgnn_ctx* ctx, const tgnn_params* p, int R, int n_rows, const int* n_rows_dev, const AttnIn& in,
                         StageTimer* tm, hipStream_t s, const SortArgs& fill = SortArgs(), bool with_merge = true) {
  const Dims& d = ctx->d; Ws& w = ctx->w;
  const bool slot_part = d.de + d.dt > 0;   // (always: d_t > 0)
  if (tm) tm->begin(9);
  const NtProblem node_part = nt_live(nt_problem(w.Xrow, d.ldxr, w.Wx, d.ldxr, w.bias_x, w.P, d.ldp, n_rows,
                                                 d.ldkv + 2 * d.dO, d.ldxr, d.ldp, false, n_rows_dev), d.dx);
  gemm_nt_group(&node_part, 1, s);
  if (tm) { tm->end(9); tm->begin(8); }
  if (slot_part) {   // U = q (W_k^c)_h per head: A is the q section of P (its pad columns meet zero columns of the weights)
    const NtProblem u = nt_blocks(nt_live(nt_problem(w.P + d.ldkv, d.ldp, w.WkcT, d.ldh, nullptr, w.Umat, d.ldz, n_rows,
                                                     d.H * d.dcp, d.ldh, d.ldz, false, n_rows_dev), d.dO),
                                  d.dcp, d.dO / d.H);
    gemm_nt_group(&u, 1, s);
  }
  if (tm) { tm->end(8); tm->begin(10); }
  FusedAttn fa = fused_args(ctx, R, in);
  fa.fill = fill;
  fattn_fwd(fa, s);
  if (tm) { tm->end(10); tm->begin(7); }
  {   // attention output = node part + Zp (W_v^c)^T
    RowAdd add;
    add.src = w.Onode; add.ld = d.ldh; add.index = nullptr; add.row0 = 0;
    const NtProblem o = nt_blocks(nt_live(nt_problem(w.Zp, d.ldz, w.Wvc, d.ldz, nullptr, w.Omat, d.ldh, R, d.dO, d.ldz, d.ldh,
                                                     false, nullptr, add), d.H * d.dcp),
                                  d.dO / d.H, d.dcp);
    gemm_nt_group(&o, 1, s);
  }
  if (tm) tm->end(7);
  if (!with_merge) return;   // the caller's next launch holds the merge layer
  if (tm) tm->begin(11);
  RowAdd m_add;
  m_add.src = w.P + d.ldkv + d.dO; m_add.ld = d.ldp; m_add.index = in.slot_row; m_add.row0 = 0;
  gemm_nt(w.Omat, d.ldh, w.Wo_o, d.ldh, nullptr, w.z, d.ldh, R, d.dO, d.ldh, d.ldh, true, s, nullptr, m_add);
  if (tm) tm->end(11);
}

// The query's time encoding: what turns ws.q_part (column sums of dq) into gradients of W_q and time_b.
static QPhi qphi_args(tgnn_ctx* ctx, const tgnn_params* p, tgnn_params* g) {
  const Dims& d = ctx->d; Ws& w = ctx->w;
  QPhi q;
  q.part = w.q_part; q.wq = p->wq; q.time_b = p->time_b; q.g_wq = g->wq; q.g_b = g->time_b;
  q.dO = d.dO; q.dq_w = d.dq; q.dx = d.dx; q.dt = d.dt;
  return q;
}

// From ws.dz (already masked by the merge ReLU) down to ws.dq, ws.dscore and the per-root sums; queues the
// weight-gradient GEMMs of W_o (attention-output columns) and of the {e | Phi} columns of W_k, W_v, and the column
// sums that give the gradients of the time-encoding parameters through the keys; adds the column sums of dq to
// ws.q_part, which the caller cleared (consumed by qphi_block in a later launch).
static void attn_backward(tgnn_ctx* ctx, tgnn_params* g, const tgnn_params* p, int R, const AttnIn& in, TnBatch& tn,
                          Side& side, hipStream_t s, StageTimer* tm, bool have_dOmat = false) {
  const Dims& d = ctx->d; Ws& w = ctx->w;
  tn.add(w.dz, d.ldh, w.Omat, d.ldh, R, d.dO, d.dO, single_out(g->wo, d.dO + d.dx, nullptr));
  if (!have_dOmat) gemm_nt(w.dz, d.ldh, w.WoT_o, d.ldh, nullptr, w.dOmat, d.ldh, R, d.dO, d.ldh, d.ldh, false, s);
  if (tm) tm->begin(19);
  {   // G = dO (W_v^c)_h per head
    const NtProblem gm = nt_blocks(nt_live(nt_problem(w.dOmat, d.ldh, w.WvcT, d.ldh, nullptr, w.Gmat, d.ldz, R, d.H * d.dcp,
                                                      d.ldh, d.ldz, false), d.dO),
                                   d.dcp, d.dO / d.H);
    gemm_nt_group(&gm, 1, s);
  }
  if (tm) { tm->end(19); tm->begin(14); }
  fattn_bwd(fused_args(ctx, R, in), s);
  if (tm) { tm->end(14); tm->begin(5); }
  {   // dq = node part + Zs (W_k^c)^T, with its column sums over the roots (for the query's Phi(0))
    RowAdd add;
    add.src = w.dqn; add.ld = d.ldh; add.index = nullptr; add.row0 = 0;
    NtProblem dq = nt_blocks(nt_live(nt_problem(w.Zs, d.ldz, w.Wkc, d.ldz, nullptr, w.dq, d.ldh, R, d.dO, d.ldz, d.ldh, false,
                                                nullptr, add), d.H * d.dcp),
                             d.dO / d.H, d.dcp);
    dq.colsum = w.q_part; dq.colsum_rows = QPHI_BLOCKS;
    gemm_nt_group(&dq, 1, s);
  }
  if (tm) tm->end(5);
  // Weight gradients of the {e | Phi} columns of W_k, W_v: per head, dK_j = ds_j q and dV_j = p_j dO, so
  // sum over slots of dK_j c_j^T = sum over roots of q Zs^T, and likewise dO Zp^T: products over R rows, not R k.
  OutMap m;
  memset(&m, 0, sizeof(m));
  m.n_split = 1 << 30; m.k_split = 1 << 30;
  m.head_n = d.dO / d.H; m.head_k = d.dcp; m.head_cols = d.de + d.dt;
  m.p[0][0] = g->wk + d.dx; m.ld[0][0] = d.dkv;
  tn.add(w.Qroot, d.ldh, w.Zs, d.ldz, R, d.dO, d.H * d.dcp, m);
  m.p[0][0] = g->wv + d.dx;
  tn.add(w.dOmat, d.ldh, w.Zp, d.ldz, R, d.dO, d.H * d.dcp, m);
  {   // gradients of the time-encoding parameters through the keys: column sums of the per-root sums Y = {d/dw | d/db}
    OutMap y;
    memset(&y, 0, sizeof(y));
    y.n_split = d.dt; y.k_split = 1 << 30;
    y.bias[0] = g->time_w; y.bias[1] = g->time_b;
    tn.add(w.Yt, d.ldy, w.Yt, d.ldy, R, 2 * d.dt, 0, y);
  }
  if (side.on) {   // the bulk of the weight-gradient work is known here: start it beside the rest of the chain
    side.fork();
    tn.launch(side.c->side);
  }
}

// After the per-row reduction into ws.dP: gradient reaching the node rows (ws.ds_row, dynamic columns) and
// the weight gradients of the node part of W_k, W_v, W_q, W_o with all four biases.
// through_gru: the gradient is not stored in ws.ds_row but carried on, in the same launch, to the gradients of
// the GRU gate pre-activations (ws.dgi, ws.dgh).  `with` (may be NULL): an independent product to run in the
// same launch.
static void node_proj_backward(tgnn_ctx* ctx, tgnn_params* g, int n_rows, const int* n_rows_dev, TnBatch& tn,
                               bool through_gru, hipStream_t s) {
  const Dims& d = ctx->d; Ws& w = ctx->w;
  GruBwdOut gb;
  if (through_gru) {
    gb.gates = w.gates; gb.Hm = w.Hm; gb.has = w.has; gb.dgi = w.dgi; gb.dgh = w.dgh;
    gb.dm = d.dm; gb.ldh = d.ldh; gb.ld3 = d.ld3;
  }
  const NtProblem mine = nt_live(nt_problem(w.dP, d.ldp, w.WxT, d.ldp, nullptr, w.ds_row, d.ldh, n_rows, d.dm, d.ldp, d.ldh,
                                            false, n_rows_dev, RowAdd(), TimeGradOut(), gb), d.ldkv + 2 * d.dO);
  if (ctx->train_static && through_gru && d.ds > 0) {
    // co-trained static memory (Sec. 3.1): the same product for the static columns of the node rows, stored per row;
    // the rows are scattered to the table by the step's last launch
    const NtProblem stat = nt_live(nt_problem(w.dP, d.ldp, w.WxT + (size_t)d.dm * d.ldp, d.ldp, nullptr, w.dstat, d.ldst, n_rows,
                                              d.ds, d.ldp, d.ldst, false, n_rows_dev), d.ldkv + 2 * d.dO);
    const NtProblem pr[2] = {mine, stat};
    gemm_nt_group(pr, 2, s);
  } else {
    gemm_nt_group(&mine, 1, s);
  }
  OutMap kv;
  memset(&kv, 0, sizeof(kv));
  kv.p[0][0] = g->wk; kv.p[1][0] = g->wv; kv.ld[0][0] = kv.ld[1][0] = d.dkv;
  kv.n_split = d.dO; kv.k_split = 1 << 30;
  kv.bias[0] = g->bk; kv.bias[1] = g->bv;
  tn.add(w.dP, d.ldp, w.Xrow, d.ldxr, n_rows, 2 * d.dO, d.dx, kv, n_rows_dev);
  OutMap qm;
  memset(&qm, 0, sizeof(qm));
  qm.p[0][0] = g->wq; qm.ld[0][0] = d.dq; qm.p[1][0] = g->wo + d.dO; qm.ld[1][0] = d.dO + d.dx;
  qm.n_split = d.dO; qm.k_split = 1 << 30;
  qm.bias[0] = g->bq; qm.bias[1] = g->bo;
  tn.add(w.dP + d.ldkv, d.ldp, w.Xrow, d.ldxr, n_rows, 2 * d.dO, d.dx, qm, n_rows_dev);
}

static hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }

static void fill_param_set(const Dims& d, const tgnn_params* p, const tgnn_params* g, int first, SgdSet& set) {
  memset(&set, 0, sizeof(set));
  float* const* pp = reinterpret_cast<float* const*>(p);
  float* const* gg = reinterpret_cast<float* const*>(g);
  const int sizes[19] = {d.dt, d.dt, 3 * d.dm * d.d_in, 3 * d.dm * d.dm, 3 * d.dm, 3 * d.dm, d.dO * d.dq, d.dO,
                         d.dO * d.dkv, d.dO, d.dO * d.dkv, d.dO, d.dO * (d.dO + d.dx), d.dO, d.dO * d.dO, d.dO * d.dO,
                         d.dO, d.nC > 0 ? d.nC * d.dO : d.dO, d.nC > 0 ? d.nC : 1};
  for (int i = first; i < 19; ++i) {
    set.p[set.cnt] = pp[i]; set.g[set.cnt] = gg ? gg[i] : nullptr; set.n[set.cnt] = sizes[i]; set.cnt++;
  }
}

}  // namespace tgnn

using namespace tgnn;

static int enqueue_step(tgnn_ctx* ctx, const tgnn_graph* g, tgnn_state* st, const tgnn_params* p, tgnn_params* grads,
                        const BatchSet& bs, float lr, float* out_loss, float* out_logits, int32_t* out_winner,
                        hipStream_t s);
static int replay_steps(tgnn_ctx* ctx, const tgnn_graph* g, tgnn_state* st, const tgnn_params* p, tgnn_params* grads,
                        const BatchSet* sets, int n_steps, int parity, float lr, float* out_loss, float* out_logits,
                        int32_t* out_winner, hipStream_t s);

extern "C" {

const char* tgnn_last_error(void) { return g_err; }

int32_t tgnn_create(const tgnn_config* cfg, tgnn_ctx** out) {
  if (cfg == nullptr || out == nullptr) return set_error(TGNN_E_NULL_PTR, "cfg or out is NULL");
  *out = nullptr;
  if (cfg->n_nodes <= 0 || cfg->max_batch <= 0 || cfg->n_replicas <= 0)
    return set_error(TGNN_E_INVALID_ARG, "n_nodes, max_batch and n_replicas must be positive");
  if (cfg->d_mem <= 0 || cfg->d_time <= 0 || cfg->d_edge < 0 || cfg->d_static < 0 || cfg->n_heads <= 0 || cfg->k <= 0)
    return set_error(TGNN_E_UNSUPPORTED_DIM, "d_mem, d_time, n_heads, k must be positive; d_edge, d_static >= 0");
  if (cfg->k > TGNN_MAX_K) return set_error(TGNN_E_UNSUPPORTED_DIM, "k = %d exceeds TGNN_MAX_K = %d", cfg->k, TGNN_MAX_K);
  if (cfg->n_heads > TGNN_MAX_HEADS)
    return set_error(TGNN_E_UNSUPPORTED_DIM, "n_heads = %d exceeds TGNN_MAX_HEADS = %d", cfg->n_heads, TGNN_MAX_HEADS);
  if (cfg->d_mem % cfg->n_heads != 0)
    return set_error(TGNN_E_UNSUPPORTED_DIM, "d_mem = %d is not a multiple of n_heads = %d", cfg->d_mem, cfg->n_heads);
  if (cfg->d_mem > 256 || cfg->d_time > 1024 || cfg->d_edge > 4096 || cfg->d_static > 4096)
    return set_error(TGNN_E_UNSUPPORTED_DIM, "width too large (d_mem <= 256, d_time <= 1024, d_edge, d_static <= 4096)");
  if (4LL * 4 * (cfg->d_mem + (long long)cfg->k * (cfg->d_mem + 1) + 2LL * cfg->n_heads * cfg->k) > 64 * 1024)
    return set_error(TGNN_E_UNSUPPORTED_DIM, "k * d_mem too large for the attention kernel's LDS staging");
  if (cfg->dt_source != 0 && cfg->dt_source != 1) return set_error(TGNN_E_INVALID_ARG, "dt_source must be 0 or 1");
  if (cfg->max_neg_sets < 0 || cfg->max_neg_sets > TGNN_MAX_NEG_SETS)
    return set_error(TGNN_E_OUT_OF_RANGE, "max_neg_sets = %d outside [0, %d]", cfg->max_neg_sets, TGNN_MAX_NEG_SETS);
  if ((long long)cfg->n_nodes * cfg->n_replicas > 0x7fffffffLL)
    return set_error(TGNN_E_OUT_OF_RANGE, "n_nodes * n_replicas exceeds int32");
  if (cfg->n_classes < 0 || cfg->n_classes > TGNN_MAX_CLASSES)
    return set_error(TGNN_E_OUT_OF_RANGE, "n_classes = %d outside [0, %d]", cfg->n_classes, TGNN_MAX_CLASSES);

  tgnn_ctx* ctx = new (std::nothrow) tgnn_ctx();
  if (ctx == nullptr) return set_error(TGNN_E_WORKSPACE, "out of host memory");
  ctx->cfg = *cfg;
  Dims& d = ctx->d;
  d.N = cfg->n_nodes; d.dm = cfg->d_mem; d.dt = cfg->d_time; d.de = cfg->d_edge; d.ds = cfg->d_static;
  d.H = cfg->n_heads; d.k = cfg->k; d.nrep = cfg->n_replicas; d.maxB = cfg->max_batch; d.dt_source = cfg->dt_source;
  d.d_in = 2 * d.dm + d.dt + d.de; d.dx = d.dm + d.ds; d.dq = d.dx + d.dt; d.dkv = d.dx + d.de + d.dt; d.dO = d.dm;
  d.ldx = padrow(d.d_in); d.ldh = padrow(d.dm); d.ld3 = padrow(3 * d.dm); d.ldxr = padrow(d.dx);
  d.ldkv = padrow(2 * d.dO); d.ldp = 2 * d.ldkv; d.ldt = padrow(d.dt);
  d.dcp = (d.de + d.dt + 3) & ~3; d.ldz = padrow(d.H * d.dcp); d.ldy = padrow(2 * d.dt); d.ldst = padrow(d.ds > 0 ? d.ds : 1);
  const int nb = d.nrep < TGNN_MAX_BATCHES ? d.nrep : TGNN_MAX_BATCHES;
  const long long maxEv = (long long)d.maxB * nb;
  d.maxNeg = cfg->max_neg_sets > 1 ? cfg->max_neg_sets : 1;
  d.nC = cfg->n_classes; d.ldc = padrow(d.nC > 0 ? d.nC : 1);
  if (maxEv * (2 + d.maxNeg) * (1 + d.k) > 0x3fffffffLL) {
    delete ctx;
    return set_error(TGNN_E_OUT_OF_RANGE, "max_batch * n_replicas * (2 + max_neg_sets) * (1 + k) exceeds the slot index range");
  }
  d.maxEv = (int)maxEv; d.maxR = (2 + d.maxNeg) * d.maxEv; d.maxRK = d.maxR * d.k; d.maxS = d.maxR + d.maxRK;
  {  // distinct (replica, node) rows a step can touch
    const long long ng = (long long)d.nrep * d.N;
    d.maxU = (int)(ng < d.maxS ? ng : d.maxS);
  }

  Bump measure{nullptr};
  layout(d, ctx->w, measure);
  ctx->arena_bytes = measure.off;
  hipError_t e = hipGetDevice(&ctx->device);
  if (e == hipSuccess) e = hipMalloc(&ctx->arena, ctx->arena_bytes);
  if (e != hipSuccess) {
    delete ctx;
    return set_error(e == hipErrorOutOfMemory ? TGNN_E_WORKSPACE : TGNN_E_HIP, "workspace allocation of %zu bytes failed: %s",
                     measure.off, hipGetErrorString(e));
  }
  e = hipMemset(ctx->arena, 0, ctx->arena_bytes);
  if (e != hipSuccess) {
    (void)hipFree(ctx->arena);
    delete ctx;
    return set_error(TGNN_E_HIP, "workspace clear failed: %s", hipGetErrorString(e));
  }
  Bump place{static_cast<char*>(ctx->arena)};
  layout(d, ctx->w, place);
  ctx->last_attn_roots = -1;
  e = hipStreamCreateWithFlags(&ctx->side, hipStreamNonBlocking);
  for (int i = 0; i < 16 && e == hipSuccess; ++i) e = hipEventCreateWithFlags(&ctx->fork_ev[i], hipEventDisableTiming);
  if (e != hipSuccess) {
    for (int i = 0; i < 16; ++i)
      if (ctx->fork_ev[i]) (void)hipEventDestroy(ctx->fork_ev[i]);
    if (ctx->side) (void)hipStreamDestroy(ctx->side);
    (void)hipFree(ctx->arena);
    delete ctx;
    return set_error(TGNN_E_HIP, "stream/event creation failed: %s", hipGetErrorString(e));
  }
  *out = ctx;
  return TGNN_OK;
}

int32_t tgnn_destroy(tgnn_ctx* ctx) {
  if (ctx == nullptr) return TGNN_OK;
  hipError_t e = hipDeviceSynchronize();
  hipError_t e2 = hipFree(ctx->arena);
  for (StepGraph& sg : ctx->graphs)
    if (sg.used) { (void)hipGraphExecDestroy(sg.exec); (void)hipGraphDestroy(sg.graph); }
  for (int i = 0; i < 16; ++i)
    if (ctx->fork_ev[i]) (void)hipEventDestroy(ctx->fork_ev[i]);
  if (ctx->side) (void)hipStreamDestroy(ctx->side);
  for (int st = 0; st < TGNN_N_STAGES; ++st)
    for (int k2 = 0; k2 < 2; ++k2)
      if (ctx->prof.ev[st][k2]) {
        for (int i = 0; i < PROF_RING; ++i) (void)hipEventDestroy(ctx->prof.ev[st][k2][i]);
        delete[] ctx->prof.ev[st][k2];
      }
  delete ctx;
  if (e != hipSuccess) return set_error(TGNN_E_HIP, "hipDeviceSynchronize: %s", hipGetErrorString(e));
  if (e2 != hipSuccess) return set_error(TGNN_E_HIP, "hipFree: %s", hipGetErrorString(e2));
  return TGNN_OK;
}

int64_t tgnn_workspace_bytes(const tgnn_ctx* ctx) { return ctx ? (int64_t)ctx->arena_bytes : 0; }

int32_t tgnn_build_tcsr(const int32_t* src, const int32_t* dst, const double* ts, int64_t n_events, int32_t n_nodes,
                        int64_t* indptr, int32_t* nbr, int32_t* eid, double* ts_out) {
  if (!src || !dst || !ts || !indptr || !nbr || !eid || !ts_out) return set_error(TGNN_E_NULL_PTR, "NULL argument");
  if (n_events < 0 || n_nodes <= 0 || n_events > 0x3fffffffLL) return set_error(TGNN_E_INVALID_ARG, "bad sizes");
  for (int64_t e = 0; e < n_events; ++e) {
    if (src[e] < 0 || src[e] >= n_nodes || dst[e] < 0 || dst[e] >= n_nodes)
      return set_error(TGNN_E_OUT_OF_RANGE, "event %lld has an endpoint outside [0, %d)", (long long)e, n_nodes);
    if (e > 0 && !(ts[e] >= ts[e - 1]))
      return set_error(TGNN_E_UNSORTED_TS, "timestamps decrease (or are NaN) at event %lld", (long long)e);
  }
  // counting sort by node; events are visited in (time, id) order, source entry before destination entry,
  // so every list ascends in (time, event id)
  for (int32_t v = 0; v <= n_nodes; ++v) indptr[v] = 0;
  for (int64_t e = 0; e < n_events; ++e) { indptr[src[e] + 1]++; indptr[dst[e] + 1]++; }
  for (int32_t v = 0; v < n_nodes; ++v) indptr[v + 1] += indptr[v];
  std::vector<int64_t> cur(indptr, indptr + n_nodes);
  for (int64_t e = 0; e < n_events; ++e) {
    int64_t a = cur[src[e]]++;
    nbr[a] = dst[e]; eid[a] = (int32_t)e; ts_out[a] = ts[e];
    int64_t b = cur[dst[e]]++;
    nbr[b] = src[e]; eid[b] = (int32_t)e; ts_out[b] = ts[e];
  }
  return TGNN_OK;
}

int32_t tgnn_state_reset(tgnn_ctx* ctx, tgnn_state* st, int32_t replica, void* stream) {
  if (ctx == nullptr) return set_error(TGNN_E_NULL_PTR, "ctx is NULL");
  if (int rc = check_state(ctx, st)) return rc;
  if (replica < -1 || replica >= ctx->d.nrep) return set_error(TGNN_E_OUT_OF_RANGE, "replica %d out of range", replica);
  fill_state(ctx, st, replica, as_stream(stream));
  TGNN_LAUNCH_CHECK();
  return TGNN_OK;
}

int32_t tgnn_sample_recent(tgnn_ctx* ctx, const tgnn_graph* g, const int32_t* node, const double* t, int32_t n_roots,
                           int32_t* out_nbr, int32_t* out_eid, double* out_ts, int32_t* out_cnt, void* stream) {
  if (ctx == nullptr) return set_error(TGNN_E_NULL_PTR, "ctx is NULL");
  if (int rc = check_graph(ctx, g)) return rc;
  if (n_roots < 0) return set_error(TGNN_E_INVALID_ARG, "n_roots < 0");
  if (n_roots == 0) return TGNN_OK;
  REQ_PTR(node); REQ_PTR(t); REQ_PTR(out_nbr); REQ_PTR(out_eid); REQ_PTR(out_ts); REQ_PTR(out_cnt);
  sample_recent(ctx->d, g, node, t, n_roots, out_nbr, out_eid, out_ts, out_cnt, as_stream(stream));
  TGNN_LAUNCH_CHECK();
  return TGNN_OK;
}

int32_t tgnn_gather_memory(tgnn_ctx* ctx, const tgnn_graph* g, const tgnn_state* st, int32_t replica,
                           const int32_t* slot_node, int32_t n_slots, float* out_mem, float* out_mail,
                           float* out_mail_efeat, double* out_mem_ts, double* out_mail_ts, int32_t* out_has_mail,
                           void* stream) {
  if (ctx == nullptr) return set_error(TGNN_E_NULL_PTR, "ctx is NULL");
  if (int rc = check_graph(ctx, g)) return rc;
  if (int rc = check_state(ctx, st)) return rc;
  const Dims& d = ctx->d;
  if (replica < 0 || replica >= d.nrep) return set_error(TGNN_E_OUT_OF_RANGE, "replica %d out of range", replica);
  if (n_slots < 0) return set_error(TGNN_E_INVALID_ARG, "n_slots < 0");
  if (n_slots == 0) return TGNN_OK;
  REQ_PTR(slot_node); REQ_PTR(out_mem); REQ_PTR(out_mail); REQ_PTR(out_mem_ts); REQ_PTR(out_mail_ts);
  REQ_PTR(out_has_mail);
  if (d.de > 0) REQ_PTR(out_mail_efeat);
  GatherArgs a;
  memset(&a, 0, sizeof(a));
  a.mem = st->mem; a.mail = st->mail; a.efeat = g->efeat; a.mem_ts = st->mem_ts; a.mail_ts = st->mail_ts;
  a.mail_eid = st->mail_eid; a.slot_gid = slot_node; a.gid_add = replica * d.N;
  a.o_mem = out_mem; a.p_mem = d.dm; a.o_mail = out_mail; a.p_mail = 2 * d.dm;
  a.o_ef = d.de > 0 ? out_mail_efeat : nullptr; a.p_ef = d.de;
  a.o_mem_ts = out_mem_ts; a.o_mail_ts = out_mail_ts; a.o_has = out_has_mail;
  a.n_slots = n_slots; a.dm = d.dm; a.dt = d.dt; a.de = d.de;
  gather_rows(a, as_stream(stream));
  TGNN_LAUNCH_CHECK();
  return TGNN_OK;
}

int32_t tgnn_gru_update(tgnn_ctx* ctx, const tgnn_params* p, int32_t n_slots, const float* mem, const float* mail,
                        const float* mail_efeat, const double* mem_ts, const double* mail_ts, const int32_t* has_mail,
                        float* out_s_new, double* out_tau, void* stream) {
  if (ctx == nullptr) return set_error(TGNN_E_NULL_PTR, "ctx is NULL");
  if (int rc = check_params(p, "params")) return rc;
  const Dims& d = ctx->d; Ws& w = ctx->w;
  if (n_slots < 0 || n_slots > d.maxS)
    return set_error(TGNN_E_WORKSPACE, "n_slots = %d outside [0, %d] (workspace row capacity)", n_slots, d.maxS);
  if (n_slots == 0) return TGNN_OK;
  REQ_PTR(mem); REQ_PTR(mail); REQ_PTR(mem_ts); REQ_PTR(mail_ts); REQ_PTR(has_mail); REQ_PTR(out_s_new); REQ_PTR(out_tau);
  if (d.de > 0) REQ_PTR(mail_efeat);
  hipStream_t s = as_stream(stream);
  prologue(ctx, p, nullptr, nullptr, nullptr, nullptr, s);
  GatherArgs a;
  memset(&a, 0, sizeof(a));
  a.mem = mem; a.mail = mail; a.efeat = mail_efeat; a.mem_ts = mem_ts; a.mail_ts = mail_ts;
  a.mail_eid = nullptr; a.has_in = has_mail; a.slot_gid = nullptr;
  a.o_mem = w.Hm; a.p_mem = d.ldh; a.z_mem = d.ldh - d.dm;
  a.o_mail = w.X; a.p_mail = d.ldx;
  a.o_phi = w.X + 2 * d.dm; a.p_phi = d.ldx;
  a.o_ef = w.X + 2 * d.dm + d.dt; a.p_ef = d.ldx; a.z_ef = d.ldx - d.d_in;
  a.o_tau = out_tau; a.o_delta = w.delta; a.o_has = w.has;
  a.time_w = p->time_w; a.time_b = p->time_b;
  a.n_slots = n_slots; a.dm = d.dm; a.dt = d.dt; a.de = d.de;
  gather_rows(a, s);
  gru_forward(ctx, p, n_slots, s);
  TGNN_HIP_CHECK(hipMemcpy2DAsync(out_s_new, (size_t)d.dm * 4, w.Xrow, (size_t)d.ldxr * 4, (size_t)d.dm * 4, n_slots,
                                  hipMemcpyDeviceToDevice, s));
  TGNN_LAUNCH_CHECK();
  return TGNN_OK;
}

int32_t tgnn_temporal_attn_fwd(tgnn_ctx* ctx, const tgnn_params* p, int32_t n_roots, const float* x_root,
                               const float* x_nbr, const float* e_nbr, const double* dt_nbr, const int32_t* cnt,
                               float* out_z, void* stream) {
  if (ctx == nullptr) return set_error(TGNN_E_NULL_PTR, "ctx is NULL");
  if (int rc = check_params(p, "params")) return rc;
  const Dims& d = ctx->d; Ws& w = ctx->w;
  if (n_roots < 0 || n_roots > d.maxR)
    return set_error(TGNN_E_WORKSPACE, "n_roots = %d outside [0, %d] (workspace root capacity)", n_roots, d.maxR);
  if (n_roots == 0) { ctx->last_attn_roots = 0; return TGNN_OK; }
  REQ_PTR(x_root); REQ_PTR(x_nbr); REQ_PTR(dt_nbr); REQ_PTR(cnt); REQ_PTR(out_z);
  if (d.de > 0) REQ_PTR(e_nbr);
  hipStream_t s = as_stream(stream);
  prologue(ctx, p, nullptr, nullptr, nullptr, nullptr, s);
  TGNN_HIP_CHECK(hipMemcpyAsync(w.cnt, cnt, sizeof(int32_t) * n_roots, hipMemcpyDeviceToDevice, s));
  stage_x_rows(n_roots, d.k, d.dx, x_root, x_nbr, cnt, w.Xrow, d.ldxr, s);
  // the caller's rows have to stay as they are until the backward call (the slots' inputs are read again there)
  ctx->last_attn = AttnCall{e_nbr, dt_nbr};
  const AttnIn in{nullptr, w.cnt, e_nbr, nullptr, dt_nbr, p};
  attn_forward(ctx, p, n_roots, n_roots * (1 + d.k), nullptr, in, nullptr, s);
  TGNN_HIP_CHECK(hipMemcpy2DAsync(out_z, (size_t)d.dO * 4, w.z, (size_t)d.ldh * 4, (size_t)d.dO * 4, n_roots,
                                  hipMemcpyDeviceToDevice, s));
  TGNN_LAUNCH_CHECK();
  ctx->last_attn_roots = n_roots;
  return TGNN_OK;
}

int32_t tgnn_temporal_attn_bwd(tgnn_ctx* ctx, const tgnn_params* p, int32_t n_roots, const float* dz, tgnn_params* grads,
                               float* d_x_root, float* d_x_nbr, void* stream) {
  if (ctx == nullptr) return set_error(TGNN_E_NULL_PTR, "ctx is NULL");
  if (int rc = check_params(p, "params")) return rc;
  if (int rc = check_params(grads, "grads")) return rc;
  const Dims& d = ctx->d; Ws& w = ctx->w;
  if (n_roots != ctx->last_attn_roots)
    return set_error(TGNN_E_INVALID_ARG, "n_roots = %d does not match the last tgnn_temporal_attn_fwd (%d)", n_roots,
                     ctx->last_attn_roots);
  if (n_roots == 0) return TGNN_OK;
  REQ_PTR(dz); REQ_PTR(d_x_root); REQ_PTR(d_x_nbr);
  hipStream_t s = as_stream(stream);
  mask_dz(n_roots, d.dO, dz, d.dO, w.z, d.ldh, w.dz, s);
  zero_f32(w.q_part, QPHI_BLOCKS * d.dO, s);
  TnBatch tn;
  Side side{ctx, s, false};
  const int RK = n_roots * d.k;
  const AttnIn in{nullptr, w.cnt, ctx->last_attn.e_nbr, nullptr, ctx->last_attn.dt_nbr, p};
  attn_backward(ctx, grads, p, n_roots, in, tn, side, s, nullptr);
  slots_to_dp(ctx, n_roots, RK, qphi_args(ctx, p, grads), s);
  node_proj_backward(ctx, grads, n_roots + RK, nullptr, tn, false, s);
  tn.launch(s);
  attn_dx_out(n_roots, RK, d.dm, w.ds_row, d.ldh, d_x_root, d_x_nbr, s);
  TGNN_LAUNCH_CHECK();
  return TGNN_OK;
}

static int make_batchset(const tgnn_ctx* ctx, const tgnn_batch* batches, int n_batches, BatchSet& bs, int nneg = 1) {
  const Dims& d = ctx->d;
  if (batches == nullptr) return set_error(TGNN_E_NULL_PTR, "batches is NULL");
  const int cap = d.nrep < TGNN_MAX_BATCHES ? d.nrep : TGNN_MAX_BATCHES;
  if (n_batches < 1 || n_batches > cap)
    return set_error(TGNN_E_INVALID_ARG, "n_batches = %d outside [1, %d]", n_batches, cap);
  memset(&bs, 0, sizeof(bs));
  int off = 0;
  for (int b = 0; b < n_batches; ++b) {
    const tgnn_batch& tb = batches[b];
    if (tb.n < 0 || tb.n > d.maxB) return set_error(TGNN_E_OUT_OF_RANGE, "batch %d: n = %d outside [0, %d]", b, tb.n, d.maxB);
    if (tb.replica < 0 || tb.replica >= d.nrep)
      return set_error(TGNN_E_OUT_OF_RANGE, "batch %d: replica %d outside [0, %d)", b, tb.replica, d.nrep);
    for (int b2 = 0; b2 < b; ++b2)
      if (batches[b2].replica == tb.replica)
        return set_error(TGNN_E_INVALID_ARG, "replica %d appears twice in one step", tb.replica);
    if (tb.n > 0) {
      REQ_PTR(tb.src); REQ_PTR(tb.dst); REQ_PTR(tb.eid); REQ_PTR(tb.t);
    }
    bs.b[b] = BatchDesc{tb.src, tb.dst, tb.neg, tb.eid, tb.t, tb.n, tb.replica, off};
    off += tb.n;
  }
  bs.nb = n_batches;
  bs.total = off;
  bs.nneg = nneg;
  return TGNN_OK;
}

int32_t tgnn_memory_writeback(tgnn_ctx* ctx, tgnn_state* st, int32_t replica, const int32_t* src, const int32_t* dst,
                              const int32_t* eid, const double* t, int32_t n_events, const float* s_new_src,
                              const float* s_new_dst, const double* tau_src, const double* tau_dst,
                              int32_t* out_winner, void* stream) {
  if (ctx == nullptr) return set_error(TGNN_E_NULL_PTR, "ctx is NULL");
  if (int rc = check_state(ctx, st)) return rc;
  const Dims& d = ctx->d;
  if (replica < 0 || replica >= d.nrep) return set_error(TGNN_E_OUT_OF_RANGE, "replica %d out of range", replica);
  if (n_events < 0 || n_events > d.maxB)
    return set_error(TGNN_E_OUT_OF_RANGE, "n_events = %d outside [0, %d]", n_events, d.maxB);
  if (n_events == 0) return TGNN_OK;
  REQ_PTR(src); REQ_PTR(dst); REQ_PTR(eid); REQ_PTR(t); REQ_PTR(s_new_src); REQ_PTR(s_new_dst); REQ_PTR(tau_src);
  REQ_PTR(tau_dst); OPT_PTR(out_winner);
  BatchSet bs;
  memset(&bs, 0, sizeof(bs));
  bs.b[0] = BatchDesc{src, dst, nullptr, eid, t, n_events, replica, 0};
  bs.nb = 1; bs.total = n_events; bs.nneg = 1;
  hipStream_t s = as_stream(stream);
  Ws& w = ctx->w;
  prologue(ctx, nullptr, &bs, nullptr, nullptr, nullptr, s);
  writeback_mark(d, w.bs_dev, n_events, w.winkey, w.epoch, s);
  writeback_scatter(d, w.bs_dev, n_events, st, w.winkey, w.epoch, nullptr, d.dm, nullptr, nullptr, s_new_src, s_new_dst,
                    tau_src, tau_dst, out_winner, s);
  TGNN_LAUNCH_CHECK();
  return TGNN_OK;
}

// loss_in_array: out_loss is an element of tgnn_train_steps' loss array (checked there; only 4-byte aligned)
static int train_step_impl(tgnn_ctx* ctx, const tgnn_graph* g, tgnn_state* st, const tgnn_params* p, tgnn_params* grads,
                           const tgnn_batch* batches, int32_t n_batches, float lr, float* out_loss, float* out_logits,
                           int32_t* out_winner, void* stream, bool loss_in_array, int nneg = 1,
                           const float* const* labels = nullptr);

int32_t tgnn_train_step_epoch_parallel(tgnn_ctx* ctx, const tgnn_graph* g, tgnn_state* st, const tgnn_params* p,
                                       tgnn_params* grads, const tgnn_batch* batches, int32_t n_batches,
                                       int32_t n_neg_sets, float lr, float* out_loss, float* out_logits,
                                       int32_t* out_winner, void* stream) {
  if (ctx == nullptr) return set_error(TGNN_E_NULL_PTR, "ctx is NULL");
  if (n_neg_sets < 1 || n_neg_sets > ctx->d.maxNeg)
    return set_error(TGNN_E_OUT_OF_RANGE, "n_neg_sets = %d outside [1, %d] (config.max_neg_sets)", n_neg_sets, ctx->d.maxNeg);
  return train_step_impl(ctx, g, st, p, grads, batches, n_batches, lr, out_loss, out_logits, out_winner, stream, false,
                         n_neg_sets);
}

int32_t tgnn_train_step(tgnn_ctx* ctx, const tgnn_graph* g, tgnn_state* st, const tgnn_params* p, tgnn_params* grads,
                        const tgnn_batch* batches, int32_t n_batches, float lr, float* out_loss, float* out_logits,
                        int32_t* out_winner, void* stream) {
  return train_step_impl(ctx, g, st, p, grads, batches, n_batches, lr, out_loss, out_logits, out_winner, stream, false);
}

int32_t tgnn_train_step_edge_class(tgnn_ctx* ctx, const tgnn_graph* g, tgnn_state* st, const tgnn_params* p,
                                   tgnn_params* grads, const tgnn_batch* batches, int32_t n_batches,
                                   const float* const* labels, float lr, float* out_loss, float* out_logits,
                                   int32_t* out_winner, void* stream) {
  if (ctx == nullptr) return set_error(TGNN_E_NULL_PTR, "ctx is NULL");
  if (labels == nullptr) return set_error(TGNN_E_NULL_PTR, "labels is NULL");
  return train_step_impl(ctx, g, st, p, grads, batches, n_batches, lr, out_loss, out_logits, out_winner, stream, false, 0,
                         labels);
}

int32_t tgnn_eval_step(tgnn_ctx* ctx, const tgnn_graph* g, tgnn_state* st, const tgnn_params* p,
                       const tgnn_batch* batches, int32_t n_batches, int32_t n_neg_sets, float* out_logits,
                       float* out_rank, float* out_rr_sum, int32_t* out_winner, void* stream) {
  if (ctx == nullptr) return set_error(TGNN_E_NULL_PTR, "ctx is NULL");
  if (n_neg_sets < 1 || n_neg_sets > ctx->d.maxNeg)
    return set_error(TGNN_E_OUT_OF_RANGE, "n_neg_sets = %d outside [1, %d] (config.max_neg_sets)", n_neg_sets, ctx->d.maxNeg);
  REQ_PTR(out_rank); REQ_PTR(out_rr_sum);
  tgnn_params no_grads;
  memset(&no_grads, 0, sizeof(no_grads));
  ctx->eval = true; ctx->out_rank = out_rank; ctx->out_rr = out_rr_sum;
  const int rc = train_step_impl(ctx, g, st, p, &no_grads, batches, n_batches, 0.0f, nullptr, out_logits, out_winner, stream,
                                 false, n_neg_sets);
  ctx->eval = false; ctx->out_rank = nullptr; ctx->out_rr = nullptr;
  return rc;
}

int32_t tgnn_eval_step_edge_class(tgnn_ctx* ctx, const tgnn_graph* g, tgnn_state* st, const tgnn_params* p,
                                  const tgnn_batch* batches, int32_t n_batches, const float* const* labels,
                                  float* out_logits, int32_t* out_counts, int32_t* out_winner, void* stream) {
  if (ctx == nullptr) return set_error(TGNN_E_NULL_PTR, "ctx is NULL");
  if (labels == nullptr) return set_error(TGNN_E_NULL_PTR, "labels is NULL");
  REQ_PTR(out_counts);
  tgnn_params no_grads;
  memset(&no_grads, 0, sizeof(no_grads));
  ctx->eval = true; ctx->out_counts = out_counts;
  const int rc = train_step_impl(ctx, g, st, p, &no_grads, batches, n_batches, 0.0f, nullptr, out_logits, out_winner, stream,
                                 false, 0, labels);
  ctx->eval = false; ctx->out_counts = nullptr;
  return rc;
}

static int train_step_impl(tgnn_ctx* ctx, const tgnn_graph* g, tgnn_state* st, const tgnn_params* p, tgnn_params* grads,
                           const tgnn_batch* batches, int32_t n_batches, float lr, float* out_loss, float* out_logits,
                           int32_t* out_winner, void* stream, bool loss_in_array, int nneg, const float* const* labels) {
  if (ctx == nullptr) return set_error(TGNN_E_NULL_PTR, "ctx is NULL");
  if ((ctx->d.nC > 0) != (labels != nullptr))
    return set_error(TGNN_E_INVALID_ARG, ctx->d.nC > 0 ? "this context has an edge-classification head (n_classes > 0): "
                                                         "use tgnn_train_step_edge_class"
                                                       : "tgnn_train_step_edge_class needs a context with n_classes > 0");
  if (int rc = check_graph(ctx, g)) return rc;
  if (int rc = check_state(ctx, st)) return rc;
  if (int rc = check_params(p, "params")) return rc;
  if (!ctx->eval)
    if (int rc = check_params(grads, "grads")) return rc;
  BatchSet bs;
  if (int rc = make_batchset(ctx, batches, n_batches, bs, nneg)) return rc;
  for (int b = 0; b < bs.nb; ++b) {
    if (labels != nullptr) {
      bs.b[b].neg = nullptr;
      bs.b[b].labels = labels[b];
      if (bs.b[b].n > 0) REQ_PTR(bs.b[b].labels);
    } else if (bs.b[b].n > 0) {
      REQ_PTR(bs.b[b].neg);
    }
  }
  bs.ncls = labels != nullptr ? ctx->d.nC : 0;
  if (!loss_in_array && !ctx->eval) REQ_PTR(out_loss);
  OPT_PTR(out_logits); OPT_PTR(out_winner);
  if (!(lr == lr)) return set_error(TGNN_E_INVALID_ARG, "lr is NaN");
  hipStream_t s = as_stream(stream);
  if (bs.total == 0) {
    if (out_loss != nullptr) zero_f32(out_loss, 1, s);
    TGNN_LAUNCH_CHECK();
    return TGNN_OK;
  }
  ctx->last_attn_roots = -1;

  // the legacy default stream (NULL) cannot be captured
  // Training steps alternate between two row counters: each clears the one the next step will use (nothing
  // else could do that before the first launch, which already counts rows).
  ctx->w.ucount = ctx->w.ucount_pair + ctx->step_parity;
  const int parity = ctx->step_parity;
  ctx->step_parity ^= 1;
  Profiler& pr = ctx->prof;
  pr.active = pr.mask != 0 && pr.calls++ % pr.every == 0 ? pr.mask : 0;
  bool use_graph = (ctx->cfg.flags & TGNN_FLAG_NO_GRAPH) == 0 && pr.active == 0 && s != nullptr;
  if (use_graph) {
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(s, &cs) != hipSuccess || cs != hipStreamCaptureStatusNone) use_graph = false;
  }
  if (!use_graph) return enqueue_step(ctx, g, st, p, grads, bs, lr, out_loss, out_logits, out_winner, s);

  return replay_steps(ctx, g, st, p, grads, &bs, 1, parity, lr, out_loss, out_logits, out_winner, s);
}

int32_t tgnn_train_steps(tgnn_ctx* ctx, const tgnn_graph* g, tgnn_state* st, const tgnn_params* p, tgnn_params* grads,
                         int32_t n_steps, const tgnn_batch* batches, int32_t n_batches, float lr, float* out_loss,
                         void* stream) {
  if (ctx == nullptr) return set_error(TGNN_E_NULL_PTR, "ctx is NULL");
  if (n_steps < 1 || n_steps > TGNN_MAX_STEPS_PER_CALL)
    return set_error(TGNN_E_OUT_OF_RANGE, "n_steps = %d outside [1, %d]", n_steps, TGNN_MAX_STEPS_PER_CALL);
  if (batches == nullptr) return set_error(TGNN_E_NULL_PTR, "batches is NULL");
  REQ_PTR(out_loss);
  // Runs of consecutive steps of one shape on which no stage timing is due are replayed as one recorded graph each
  // when nothing stands in the way of replaying (see tgnn_train_step); the other steps are issued one by one, with
  // the same result.
  bool can_replay = n_steps > 1 && (ctx->cfg.flags & (TGNN_FLAG_NO_GRAPH | TGNN_FLAG_SIDE_STREAM)) == 0 && stream != nullptr;
  if (can_replay) {
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(as_stream(stream), &cs) != hipSuccess || cs != hipStreamCaptureStatusNone) can_replay = false;
  }
  BatchSet sets[TGNN_MAX_STEPS_PER_CALL];
  if (can_replay) {
    if (int rc = check_graph(ctx, g)) return rc;
    if (int rc = check_state(ctx, st)) return rc;
    if (int rc = check_params(p, "params")) return rc;
    if (int rc = check_params(grads, "grads")) return rc;
    if (!(lr == lr)) return set_error(TGNN_E_INVALID_ARG, "lr is NaN");
    for (int i = 0; i < n_steps; ++i) {
      if (int rc = make_batchset(ctx, batches + (size_t)i * n_batches, n_batches, sets[i])) return rc;
      for (int b = 0; b < sets[i].nb; ++b)
        if (sets[i].b[b].n > 0) REQ_PTR(sets[i].b[b].neg);
    }
  }
  Profiler& pr = ctx->prof;
  auto same_shape = [&](int i, int j) {
    for (int b = 0; b < sets[i].nb; ++b)
      if (sets[i].b[b].n != sets[j].b[b].n || sets[i].b[b].replica != sets[j].b[b].replica) return false;
    return true;
  };
  for (int i = 0; i < n_steps;) {
    int run = 0;   // steps from i on that can share a graph: one shape, not empty, no stage timing due
    if (can_replay && sets[i].total > 0)
      while (i + run < n_steps && same_shape(i, i + run) && !(pr.mask != 0 && (pr.calls + run) % pr.every == 0)) ++run;
    if (run >= 2) {
      ctx->last_attn_roots = -1;
      if (pr.mask != 0) pr.calls += run;
      pr.active = 0;
      const int parity = ctx->step_parity;
      ctx->step_parity ^= run & 1;
      if (int rc = replay_steps(ctx, g, st, p, grads, sets + i, run, parity, lr, out_loss + i, nullptr, nullptr,
                                as_stream(stream)))
        return rc;
      i += run;
    } else {
      if (int rc = train_step_impl(ctx, g, st, p, grads, batches + (size_t)i * n_batches, n_batches, lr, out_loss + i,
                                   nullptr, nullptr, stream, true))
        return rc;
      i += 1;
    }
  }
  return TGNN_OK;
}

// Replays (recording it first if need be) the HIP graph of n_steps consecutive training steps of one shape; step i
// uses row counter (parity + i) & 1 and writes its loss to out_loss[i].
static int replay_steps(tgnn_ctx* ctx, const tgnn_graph* g, tgnn_state* st, const tgnn_params* p, tgnn_params* grads,
                        const BatchSet* sets, int n_steps, int parity, float lr, float* out_loss, float* out_logits,
                        int32_t* out_winner, hipStream_t s) {
  const BatchSet& bs = sets[0];
  // look the call signature up among the captured steps
  StepKey key;
  memset(&key, 0, sizeof(key));
  {
    int q = 0;
    key.ptr[q++] = g->indptr; key.ptr[q++] = g->nbr; key.ptr[q++] = g->eid; key.ptr[q++] = g->ts; key.ptr[q++] = g->efeat;
    key.ptr[q++] = st->mem; key.ptr[q++] = st->mem_ts; key.ptr[q++] = st->mail; key.ptr[q++] = st->mail_ts;
    key.ptr[q++] = st->mail_eid; key.ptr[q++] = st->stat;
    const float* const* pp = reinterpret_cast<const float* const*>(p);
    const float* const* gg = reinterpret_cast<const float* const*>(grads);
    for (int i = 0; i < 19; ++i) { key.ptr[q++] = pp[i]; key.ptr[q++] = gg[i]; }
    key.ptr[q++] = out_loss; key.ptr[q++] = out_logits; key.ptr[q++] = out_winner; key.ptr[q++] = s;
    key.ptr[q++] = ctx->out_rank; key.ptr[q++] = ctx->out_rr; key.ptr[q++] = ctx->out_counts;
    for (int b = 0; b < bs.nb; ++b) { key.n[b] = bs.b[b].n; key.rep[b] = bs.b[b].replica; }
    key.nb = bs.nb; key.lr = lr; key.parity = parity; key.n_steps = n_steps; key.nneg = bs.nneg;
    key.mode = (ctx->eval ? 2 : 0) + (bs.ncls > 0 ? 1 : 0);
  }
  StepGraph* hit = nullptr;
  StepGraph* victim = &ctx->graphs[0];
  for (StepGraph& sg : ctx->graphs) {
    if (sg.used && memcmp(&sg.key, &key, sizeof(key)) == 0) { hit = &sg; break; }
    if (!sg.used || (victim->used && sg.last_use < victim->last_use)) victim = &sg;
  }
  const Dims& d = ctx->d;
  if (hit == nullptr) {
    if (victim->used) {
      (void)hipGraphExecDestroy(victim->exec);
      (void)hipGraphDestroy(victim->graph);
      victim->used = false;
    }
    TGNN_HIP_CHECK(hipStreamBeginCapture(s, hipStreamCaptureModeThreadLocal));
    int rc = TGNN_OK;
    for (int i = 0; i < n_steps && rc == TGNN_OK; ++i) {
      ctx->w.ucount = ctx->w.ucount_pair + ((parity + i) & 1);
      rc = enqueue_step(ctx, g, st, p, grads, sets[i], lr, out_loss != nullptr ? out_loss + i : nullptr, out_logits,
                        out_winner, s);
    }
    hipGraph_t graph = nullptr;
    const hipError_t ce = hipStreamEndCapture(s, &graph);
    if (rc != TGNN_OK) { if (graph) (void)hipGraphDestroy(graph); return rc; }
    if (ce != hipSuccess) return set_error(TGNN_E_HIP, "hipStreamEndCapture failed: %s", hipGetErrorString(ce));
    // the recorded launches form a chain; the first launch of every step is found by its kernel
    hipGraphNode_t node = nullptr, heads[TGNN_MAX_STEPS_PER_CALL];
    int n_heads = 0;
    size_t n_next = 1;
    hipError_t e = hipGraphGetRootNodes(graph, &node, &n_next);
    bool chain = e == hipSuccess && n_next == 1;
    if (chain && n_steps == 1) {   // (with the side stream the graph forks further on: only its root is looked at)
      hipGraphNodeType ty = hipGraphNodeTypeEmpty;
      chain = hipGraphNodeGetType(node, &ty) == hipSuccess && ty == hipGraphNodeTypeKernel;
      heads[n_heads++] = node;
    }
    for (int guard = 0; n_steps > 1 && chain && node != nullptr && guard < 4096; ++guard) {
      hipGraphNodeType ty = hipGraphNodeTypeEmpty;
      if (hipGraphNodeGetType(node, &ty) != hipSuccess) { chain = false; break; }
      if (ty == hipGraphNodeTypeKernel) {
        hipKernelNodeParams kp;
        memset(&kp, 0, sizeof(kp));
        if (hipGraphKernelNodeGetParams(node, &kp) != hipSuccess) { chain = false; break; }
        if (kp.func == head_func()) {
          if (n_heads == TGNN_MAX_STEPS_PER_CALL) { chain = false; break; }
          heads[n_heads++] = node;
        }
      }
      size_t n_dep = 0;
      if (hipGraphNodeGetDependentNodes(node, nullptr, &n_dep) != hipSuccess || n_dep > 1) { chain = false; break; }
      if (n_dep == 0) break;
      hipGraphNode_t next = nullptr;
      n_dep = 1;
      if (hipGraphNodeGetDependentNodes(node, &next, &n_dep) != hipSuccess) { chain = false; break; }
      node = next;
    }
    if (!chain || n_heads != n_steps || heads[0] == nullptr) {
      (void)hipGraphDestroy(graph);
      return set_error(TGNN_E_HIP, "captured steps have an unexpected shape (%d first launches for %d steps)", n_heads,
                       n_steps);
    }
    hipGraphExec_t exec = nullptr;
    e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
    if (e != hipSuccess) {
      (void)hipGraphDestroy(graph);
      return set_error(TGNN_E_HIP, "hipGraphInstantiate failed: %s", hipGetErrorString(e));
    }
    victim->used = true; victim->key = key; victim->graph = graph; victim->exec = exec;
    for (int i = 0; i < n_steps; ++i) victim->head_node[i] = heads[i];
    hit = victim;
  } else {
    // same launches as the recorded steps; only the first launch's argument block (batch descriptors) of each is new
    SgdSet sgd_set, zero_set_;
    fill_param_set(d, p, grads, 2, sgd_set);
    fill_param_set(d, grads, nullptr, 0, zero_set_);
    const bool overwrite = (ctx->cfg.flags & TGNN_FLAG_OVERWRITE_GRADS) != 0;
    for (int i = 0; i < n_steps; ++i) {
      ctx->w.ucount = ctx->w.ucount_pair + ((parity + i) & 1);
      HeadArgs h;
      head_fill(ctx, g, (2 + sets[i].nneg) * sets[i].total, p, &sets[i], lr != 0.0f ? &sgd_set : nullptr,
                overwrite && !ctx->eval ? &zero_set_ : nullptr, out_loss != nullptr ? out_loss + i : nullptr, h);
      void* kargs[1] = {&h};
      hipKernelNodeParams np;
      memset(&np, 0, sizeof(np));
      np.func = head_func();
      np.gridDim = head_grid(h);
      np.blockDim = dim3(64 * SAMPLE_WAVES);
      np.kernelParams = kargs;
      TGNN_HIP_CHECK(hipGraphExecKernelNodeSetParams(hit->exec, hit->head_node[i], &np));
    }
  }
  hit->last_use = ++ctx->graph_clock;
  TGNN_HIP_CHECK(hipGraphLaunch(hit->exec, s));
  return TGNN_OK;
}

// Enqueues every launch of one training step on `s` (and the context's side stream).
static int enqueue_step(tgnn_ctx* ctx, const tgnn_graph* g, tgnn_state* st, const tgnn_params* p, tgnn_params* grads,
                        const BatchSet& bs, float lr, float* out_loss, float* out_logits, int32_t* out_winner,
                        hipStream_t s) {
  const Dims& d = ctx->d; Ws& w = ctx->w;
  const bool eval = ctx->eval, classes = bs.ncls > 0;
  const int R = (2 + bs.nneg) * bs.total, S = R * (1 + d.k);
  const int n_logits = classes ? bs.total * d.nC : (1 + bs.nneg) * bs.total;

  StageTimer tm{ctx, s};
  Side side{ctx, s, (ctx->cfg.flags & TGNN_FLAG_SIDE_STREAM) != 0};
  SgdSet sgd_set, zero_set_;
  fill_param_set(d, p, grads, 2, sgd_set);  // time_w, time_b stay frozen
  fill_param_set(d, grads, nullptr, 0, zero_set_);
  const bool overwrite = (ctx->cfg.flags & TGNN_FLAG_OVERWRITE_GRADS) != 0 && !eval;
  tm.begin(2);
  {  // first launch: the sampler's blocks, then the prologue's
    HeadArgs h;
    head_fill(ctx, g, R, p, &bs, lr != 0.0f ? &sgd_set : nullptr, overwrite ? &zero_set_ : nullptr, out_loss, h);
    step_head(h, s);
  }
  tm.end(2);
  // UPDT once per distinct (replica, node) among the root and supporting nodes, from the pre-batch state
  const int U = S < d.maxU ? S : d.maxU;   // launch bound; the actual row count is *w.ucount on the device
  // distinct node rows to expect: an eighth of the slots (a step's slots repeat nodes many times over on the
  // power-law graphs), but never more than there are nodes.  Kernels that stride over the rows are launched for it.
  const int U_est = std::min(U, std::max(S / 8, 64));
  GatherArgs a;
  memset(&a, 0, sizeof(a));
  a.mem = st->mem; a.mail = st->mail; a.efeat = g->efeat; a.mem_ts = st->mem_ts; a.mail_ts = st->mail_ts;
  a.mail_eid = st->mail_eid; a.slot_gid = w.ulist; a.gid_add = 0; a.n_dev = w.ucount;
  a.o_mem = w.Hm; a.p_mem = d.ldh; a.z_mem = d.ldh - d.dm;
  a.o_mail = w.X; a.p_mail = d.ldx;
  a.o_phi = w.X + 2 * d.dm; a.p_phi = d.ldx;
  a.o_ef = w.X + 2 * d.dm + d.dt; a.p_ef = d.ldx; a.z_ef = d.ldx - d.d_in;
  a.o_tau = w.tau; a.o_delta = w.delta; a.o_has = w.has;
  a.time_w = p->time_w; a.time_b = p->time_b;
  a.n_slots = U; a.dm = d.dm; a.dt = d.dt; a.de = d.de;
  a.launch_rows = U_est;
  a.map = sort_args(ctx, S);   // the slot -> row map rides along
  a.epoch_bump = w.epoch;      // the first launch worked with epoch + 1; from here on that is the epoch
  tm.begin(3);
  gather_rows(a, s);
  tm.end(3);
  tm.begin(4);
  {  // W_ih x and W_hh h are independent: one launch
    const NtProblem pr[2] = {
        nt_live(nt_problem(w.X, d.ldx, w.Wih_p, d.ldx, p->gru_bih, w.gi, d.ld3, U, 3 * d.dm, d.ldx, d.ld3, false, w.ucount),
                d.d_in),
        nt_live(nt_problem(w.Hm, d.ldh, w.Whh_p, d.ldh, p->gru_bhh, w.gh, d.ld3, U, 3 * d.dm, d.ldh, d.ld3, false, w.ucount),
                d.dm)};
    gemm_nt_group(pr, 2, s);
  }
  tm.end(4);
  // The GRU gates (with the scan of the slot sort) -> node rows x = {s' | static}
  tm.begin(6);
  gru_gates_fwd(gru_gates_args(d, U, w.ucount, w.gi, w.gh, w.Hm, w.has, w.gates, w.Xrow, d.ldxr, d.ds ? st->stat : nullptr,
                               w.ulist, w.dP, d.ldp, sort_args(ctx, S), U_est), s);
  tm.end(6);
  // (the fill pass of the slot sort, needed by the backward pass only, rides in the attention launch)
  // Merge layer, decoder + loss and their backward pass down to the attention output are local to an event's
  // three roots: one launch when the layer width allows it.
  // (the one-launch chain is laid out for three roots per event, the link decoder, and always runs its backward half)
  const bool chain = root_chain_fits(d) && bs.nneg == 1 && !eval && !classes;
  const AttnIn ain{w.slot_row, w.cnt, g->efeat, w.neid, nullptr, p};
  attn_forward(ctx, p, R, U, w.ucount, ain, &tm, s, sort_args(ctx, S), !chain);

  tm.begin(12);
  if (chain) {
    ChainArgs ca;
    ca.dO = d.dO; ca.ldh = d.ldh; ca.ldkv = d.ldkv; ca.ldp = d.ldp;
    ca.Omat = w.Omat; ca.P_o = w.P + d.ldkv + d.dO; ca.slot_row = w.slot_row;
    {
      const size_t ks = (size_t)(d.dO + 15) / 16, blk = ks * ks * 256;
      ca.Wo_pk = w.rc_pk; ca.Ws_pk = w.rc_pk + blk; ca.Wd_pk = w.rc_pk + 2 * blk; ca.WsT_pk = w.rc_pk + 3 * blk;
      ca.WdT_pk = w.rc_pk + 4 * blk; ca.WoT_pk = w.rc_pk + 5 * blk;
    }
    ca.b1 = p->dec_b1; ca.w2 = p->dec_w2; ca.b2 = p->dec_b2;
    ca.z = w.z; ca.h1 = w.h1; ca.logits = w.logits; ca.dPdec = w.dPdec; ca.dz = w.dz; ca.dOmat = w.dOmat;
    ca.loss = out_loss; ca.g_w2 = grads->dec_w2; ca.g_b2 = grads->dec_b2;
    root_chain(ca, bs, (ctx->cfg.flags & TGNN_FLAG_WIDE_ROOT_TILES) != 0, s);
  } else {   // decoder + loss (also produces d loss / d hidden)
    gemm_nt(w.z, d.ldh, w.Wdec_p, d.ldh, nullptr, w.Pdec, d.ldkv, R, 2 * d.dO, d.ldh, 2 * d.dO, false, s);
    if (classes)
      decoder_classes(d, w.bs_dev, bs.total, w.Pdec, d.ldkv, p->dec_b1, p->dec_w2, p->dec_b2, w.logits, out_loss, w.h1,
                      w.dPdec, w.dlog, s);
    else
      decoder_pairs(d, w.bs_dev, bs.total, w.Pdec, d.ldkv, p->dec_b1, p->dec_w2, p->dec_b2, w.logits, out_loss, w.h1, w.dPdec,
                    grads->dec_w2, grads->dec_b2, s);
  }
  tm.end(12);
  if (eval) {
    // Evaluation (Sec. 4: rank of the true destination among the sampled ones): no backward half; the write-back
    // scatter leaves in a launch of its own.
    if (classes) class_counts(w.bs_dev, bs.total, d.nC, w.logits, ctx->out_counts, s);
    else reciprocal_ranks(w.bs_dev, bs.total, w.logits, ctx->out_rank, ctx->out_rr, s);
    WbArgs wb = writeback_args(d, w.bs_dev, bs.total, st, w.winkey, w.epoch, w.Xrow, d.ldxr, w.tau, w.slot_row, nullptr,
                               nullptr, nullptr, nullptr, out_winner, nullptr, 0, 0.0f);
    gemm_nt_group(nullptr, 0, s, &wb);
    if (out_logits)
      TGNN_HIP_CHECK(hipMemcpyAsync(out_logits, w.logits, sizeof(float) * n_logits, hipMemcpyDeviceToDevice, s));
    TGNN_LAUNCH_CHECK();
    return TGNN_OK;
  }

  // Backward.  The data-gradient chain stays on the caller's stream; the weight-gradient GEMMs are queued and
  // leave in one launch at the end (side-stream mode: those known after the attention backward leave there,
  // on the side stream).
  if (!chain) tm.begin(13);
  OutMap dec;
  memset(&dec, 0, sizeof(dec));
  dec.p[0][0] = grads->dec_ws; dec.p[1][0] = grads->dec_wd; dec.ld[0][0] = dec.ld[1][0] = d.dO;
  dec.n_split = d.dO; dec.k_split = 1 << 30; dec.bias[1] = grads->dec_b1;   // every pair is in one W_d half
  TnBatch tn;
  tn.dev_rows_est = U_est;
  tn.add(w.dPdec, d.ldkv, w.z, d.ldh, R, 2 * d.dO, d.dO, dec);
  if (classes)   // output layer of the classification head: d logit^T hidden, column sums to its bias
    tn.add(w.dlog, d.ldc, w.h1, d.ldh, bs.total, d.nC, d.dO, single_out(grads->dec_w2, d.dO, grads->dec_b2));
  if (!chain) {  // dz, gated by the ReLU of the merge layer
    RowAdd gate;
    gate.gate = w.z; gate.ld_gate = d.ldh;
    gemm_nt(w.dPdec, d.ldkv, w.WdecT, d.ldkv, nullptr, w.dz, d.ldh, R, d.dO, d.ldkv, d.ldh, false, s, nullptr, gate);
    tm.end(13);
  }
  attn_backward(ctx, grads, p, R, ain, tn, side, s, &tm, chain);
  tm.begin(15);
  // per-row sum of the slot gradients reaching the per-node projections (the query's Phi(0) gradients ride along)
  seg_reduce(ctx, R, S, qphi_args(ctx, p, grads), s);
  node_proj_backward(ctx, grads, U, w.ucount, tn, true, s);
  tm.end(15);
  tn.add(w.dgi, d.ld3, w.X, d.ldx, U, 3 * d.dm, d.d_in, single_out(grads->gru_wih, d.d_in, grads->gru_bih), w.ucount);
  tn.add(w.dgh, d.ld3, w.Hm, d.ldh, U, 3 * d.dm, d.dm, single_out(grads->gru_whh, d.dm, grads->gru_bhh), w.ucount);
  tm.begin(16);
  tn.launch(s);
  tm.end(16);
  tm.begin(17);
  side.join();   // the weight gradients started beside the chain
  tm.begin(18);   // nothing in between: what a pair of event records costs by itself
  tm.end(18);
  tm.begin(17);
  {  // Last launch.  The gradient reaching the time encoding of the mails, reduced inside its GEMM (the keys'
     // went with the node projections' backward); and, as passengers (they depend on nothing in this launch:
     // the time-encoding parameters are not trained), the last-event-wins write-back of s', tau and the new
     // mails and the SGD update.
    TimeGradOut tg;
    tg.delta = w.delta; tg.w = p->time_w; tg.b = p->time_b; tg.g_w = grads->time_w; tg.g_b = grads->time_b;
    const NtProblem pr = nt_live(nt_problem(w.dgi, d.ld3, w.WihT_phi, d.ld3, nullptr, nullptr, d.ldt, U, d.dt, d.ld3, d.ldt,
                                            false, w.ucount, RowAdd(), tg), 3 * d.dm);
    WbArgs wb = writeback_args(d, w.bs_dev, bs.total, st, w.winkey, w.epoch, w.Xrow, d.ldxr, w.tau, w.slot_row, nullptr,
                               nullptr, nullptr, nullptr, out_winner, lr != 0.0f ? w.sgd_dev : nullptr, sgd_set.cnt, lr);
    if (ctx->adam && lr != 0.0f) wb.adam = w.adam_dev;
    if (ctx->train_static && d.ds > 0) {
      StatUpd& u = wb.stat;
      u.drow = w.dstat; u.ld = d.ldst; u.ds = d.ds; u.N = d.N; u.ulist = w.ulist; u.ucount = w.ucount;
      u.stat = const_cast<float*>(st->stat); u.gstat = ctx->grad_static; u.lr = ctx->lr_static;
      u.blocks = 64;
    }
    gemm_nt_group(&pr, 1, s, &wb);
  }
  tm.end(17);
  if (out_logits)
    TGNN_HIP_CHECK(hipMemcpyAsync(out_logits, w.logits, sizeof(float) * n_logits, hipMemcpyDeviceToDevice, s));
  TGNN_LAUNCH_CHECK();
  return TGNN_OK;
}

// captured steps hold the optimiser's launches: a change of optimiser or of static co-training drops them
static void drop_graphs(tgnn_ctx* ctx) {
  for (StepGraph& sg : ctx->graphs)
    if (sg.used) {
      (void)hipGraphExecDestroy(sg.exec);
      (void)hipGraphDestroy(sg.graph);
      sg.used = false;
    }
}

int32_t tgnn_set_optimizer(tgnn_ctx* ctx, int32_t kind, tgnn_params* m, tgnn_params* v, float beta1, float beta2, float eps) {
  if (ctx == nullptr) return set_error(TGNN_E_NULL_PTR, "ctx is NULL");
  if (kind != 0 && kind != 1) return set_error(TGNN_E_INVALID_ARG, "kind must be 0 (SGD) or 1 (Adam)");
  TGNN_HIP_CHECK(hipDeviceSynchronize());
  drop_graphs(ctx);
  if (kind == 0) { ctx->adam = false; return TGNN_OK; }
  if (int rc = check_params(m, "m")) return rc;
  if (int rc = check_params(v, "v")) return rc;
  if (!(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f) || !(eps > 0.f))
    return set_error(TGNN_E_INVALID_ARG, "Adam needs 0 <= beta1, beta2 < 1 and eps > 0");
  AdamSet a;
  memset(&a, 0, sizeof(a));
  float* const* mm = reinterpret_cast<float* const*>(m);
  float* const* vv = reinterpret_cast<float* const*>(v);
  for (int i = 2; i < 19; ++i) { a.m[i - 2] = mm[i]; a.v[i - 2] = vv[i]; }   // the table of the update skips time_w, time_b
  a.beta1 = beta1; a.beta2 = beta2; a.eps = eps; a.t = ctx->w.adam_t;
  TGNN_HIP_CHECK(hipMemcpy(ctx->w.adam_dev, &a, sizeof(a), hipMemcpyHostToDevice));
  TGNN_HIP_CHECK(hipMemset(ctx->w.adam_t, 0, sizeof(int32_t)));
  ctx->adam = true;
  return TGNN_OK;
}

int32_t tgnn_train_static(tgnn_ctx* ctx, int32_t enable, float* grad_static, float lr_static) {
  if (ctx == nullptr) return set_error(TGNN_E_NULL_PTR, "ctx is NULL");
  if (ctx->d.ds == 0) return set_error(TGNN_E_UNSUPPORTED_DIM, "the configuration has no static memory (d_static == 0)");
  OPT_PTR(grad_static);
  if (!(lr_static == lr_static)) return set_error(TGNN_E_INVALID_ARG, "lr_static is NaN");
  TGNN_HIP_CHECK(hipDeviceSynchronize());
  drop_graphs(ctx);
  ctx->train_static = enable != 0;
  ctx->grad_static = enable != 0 ? grad_static : nullptr;
  ctx->lr_static = enable != 0 ? lr_static : 0.f;
  return TGNN_OK;
}

int32_t tgnn_zero_params(tgnn_ctx* ctx, tgnn_params* g, void* stream) {
  if (ctx == nullptr) return set_error(TGNN_E_NULL_PTR, "ctx is NULL");
  if (int rc = check_params(g, "grads")) return rc;
  SgdSet set;
  fill_param_set(ctx->d, g, nullptr, 0, set);
  zero_set(set, as_stream(stream));
  TGNN_LAUNCH_CHECK();
  return TGNN_OK;
}

int32_t tgnn_debug_copy(void* dst, const void* src, int64_t n_bytes, void* stream) {
  REQ_PTR(dst); REQ_PTR(src);
  if (n_bytes < 0 || n_bytes % 16 != 0) return set_error(TGNN_E_INVALID_ARG, "n_bytes must be a non-negative multiple of 16");
  if (n_bytes == 0) return TGNN_OK;
  copy_f4(src, dst, (size_t)n_bytes / 16, as_stream(stream));
  TGNN_LAUNCH_CHECK();
  return TGNN_OK;
}

int32_t tgnn_profile_enable(tgnn_ctx* ctx, uint32_t stage_mask) {
  if (ctx == nullptr) return set_error(TGNN_E_NULL_PTR, "ctx is NULL");
  ctx->prof.mask = stage_mask;
  ctx->prof.active = 0;
  ctx->prof.calls = 0;
  for (int i = 0; i < TGNN_N_STAGES; ++i) ctx->prof.count[i] = 0;
  return TGNN_OK;
}

int32_t tgnn_profile_every(tgnn_ctx* ctx, int32_t n) {
  if (ctx == nullptr) return set_error(TGNN_E_NULL_PTR, "ctx is NULL");
  if (n < 1) return set_error(TGNN_E_INVALID_ARG, "n = %d must be at least 1", n);
  ctx->prof.every = n;
  ctx->prof.calls = 0;
  return TGNN_OK;
}

int32_t tgnn_profile_read(tgnn_ctx* ctx, int32_t stage, int32_t* out_count, double* out_total_ms) {
  if (ctx == nullptr || out_count == nullptr || out_total_ms == nullptr) return set_error(TGNN_E_NULL_PTR, "NULL argument");
  if (stage < 0 || stage >= TGNN_N_STAGES) return set_error(TGNN_E_OUT_OF_RANGE, "stage %d out of range", stage);
  Profiler& pr = ctx->prof;
  double total = 0.0;
  for (int i = 0; i < pr.count[stage]; ++i) {
    TGNN_HIP_CHECK(hipEventSynchronize(pr.ev[stage][1][i]));
    float ms = 0.f;
    TGNN_HIP_CHECK(hipEventElapsedTime(&ms, pr.ev[stage][0][i], pr.ev[stage][1][i]));
    total += ms;
  }
  *out_count = pr.count[stage];
  *out_total_ms = total;
  return TGNN_OK;
}

int32_t tgnn_debug_read(tgnn_ctx* ctx, int32_t what, void* dst, int64_t n_bytes, void* stream) {
  if (ctx == nullptr || dst == nullptr) return set_error(TGNN_E_NULL_PTR, "NULL argument");
  const Dims& d = ctx->d; Ws& w = ctx->w;
  const void* src = nullptr;
  size_t cap = 0;
  switch (what) {
    case 0: src = w.nbr; cap = sizeof(int32_t) * d.maxRK; break;
    case 1: src = w.neid; cap = sizeof(int32_t) * d.maxRK; break;
    case 2: src = w.nts; cap = sizeof(double) * d.maxRK; break;
    case 3: src = w.cnt; cap = sizeof(int32_t) * d.maxR; break;
    case 8: src = w.ucount; cap = sizeof(int32_t); break;
    case 9: src = w.bad_ids; cap = sizeof(int32_t); break;
    case 5: break;
    case 4: case 6: case 7: break;
    default: return set_error(TGNN_E_INVALID_ARG, "unknown item %d", what);
  }
  hipStream_t s = as_stream(stream);
  if (what == 4 || what == 5) {  // per-slot view of the per-row s' / tau of the last tgnn_train_step
    const size_t unit = what == 4 ? sizeof(float) * d.dm : sizeof(double);
    if (n_bytes < 0 || (size_t)n_bytes % unit != 0 || (size_t)n_bytes / unit > (size_t)d.maxS)
      return set_error(TGNN_E_OUT_OF_RANGE, "n_bytes is not a whole number of slots within capacity");
    const int n = (int)((size_t)n_bytes / unit);
    if (what == 4) expand_rows(ctx, n, w.Xrow, d.ldxr, nullptr, static_cast<float*>(dst), nullptr, s);
    else expand_rows(ctx, n, nullptr, 0, w.tau, nullptr, static_cast<double*>(dst), s);
    TGNN_LAUNCH_CHECK();
    return TGNN_OK;
  }
  if (what == 6 || what == 7) {  // pitched float rows -> dense [rows, d_m]
    const float* base = what == 6 ? w.z : w.h1;
    const size_t max_rows = what == 6 ? (size_t)d.maxR : (1 + (size_t)d.maxNeg) * d.maxEv;
    const size_t row_b = sizeof(float) * d.dm;
    if (n_bytes < 0 || (size_t)n_bytes % row_b != 0 || (size_t)n_bytes / row_b > max_rows)
      return set_error(TGNN_E_OUT_OF_RANGE, "n_bytes is not a whole number of rows within capacity");
    TGNN_HIP_CHECK(hipMemcpy2DAsync(dst, row_b, base, sizeof(float) * d.ldh, row_b, (size_t)n_bytes / row_b,
                                    hipMemcpyDeviceToDevice, s));
    return TGNN_OK;
  }
  if (n_bytes < 0 || (size_t)n_bytes > cap) return set_error(TGNN_E_OUT_OF_RANGE, "n_bytes exceeds the buffer");
  TGNN_HIP_CHECK(hipMemcpyAsync(dst, src, (size_t)n_bytes, hipMemcpyDeviceToDevice, s));
  return TGNN_OK;
}

}  // extern "C"
