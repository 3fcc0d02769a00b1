// Internal declarations shared by the HIP sources of libtgnn (not part of the public ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/tgnn.h"

namespace tgnn {

constexpr int WAVE = 64;

static inline int padrow(int x) { return (x + 31) & ~31; }  // row pitches are multiples of 32 floats

// Widths derived from the configuration, plus the row pitches (in floats, multiples of 32) of the
// workspace matrices.  Pad columns of every workspace matrix are kept at zero.
struct Dims {
  int N, dm, dt, de, ds, H, k, nrep, maxB, dt_source;
  int d_in, dx, dq, dkv, dO;
  int ldx;    // GRU input rows {mail | Phi | efeat}
  int ldh;    // rows of width d_m
  int ld3;    // rows of width 3 d_m
  int ldxr;   // node rows x = {s' | static}
  int ldkv;   // rows of width 2 d_o  (K | V), also decoder input {z_a | z_b}
  int ldp;    // per-node projections {K | V || q | merge}: two halves of pitch ldkv
  int ldt;    // rows of width d_t
  int dcp;    // d_e + d_t rounded up to 4: a head's block of a row of U / G / Zs / Zp
  int ldz;    // rows of width H * dcp
  int ldy;    // rows of width 2 d_t: a root's time-encoding gradient sums {d/dw | d/db}
  int ldst;   // rows of width d_s: gradient reaching a node row's static columns
  int maxNeg;   // negative sets a step may carry
  int nC, ldc;  // classes of the edge-classification head (0: link prediction) and the pitch of its [events, nC] rows
  int maxEv, maxR, maxRK, maxS, maxU;
};

struct BatchDesc {
  const int32_t *src, *dst, *neg, *eid;
  const double* t;
  int32_t n, replica, ev_off;
  const float* labels;   // [n, ncls] class targets of an edge-classification batch, else NULL
};
// Roots of batch b are [src | dst | neg set 0 | ... | neg set nneg-1], n each, starting at root (2 + nneg) * ev_off;
// its pairs are [true pairs | pairs with neg set 0 | ...], starting at pair (1 + nneg) * ev_off.
struct BatchSet {
  BatchDesc b[TGNN_MAX_BATCHES];
  int32_t nb, total;
  int32_t nneg;   // negative destinations per event (sets of the epoch-parallel step, Sec. 3.2.2); 1 in the plain step;
                  // 0 in an edge-classification step (roots [src | dst], one "pair" per event)
  int32_t ncls;   // classes of the edge-classification head; 0: link prediction
};

// Device workspace.  S slots = R roots followed by R*k neighbour slots (slot R + r*k + j).
struct Ws {
  // indices
  int32_t* root_node;                          // [R]
  double* root_t;                              // [R]
  int32_t *nbr, *neid, *cnt;                   // [R,k], [R,k], [R]
  double* nts;                                 // [R,k]
  int32_t *slot_gid, *slot_node, *has;         // [S]
  double *tau, *delta;                         // [S]
  double* dtk;                                 // [R*k] time difference in the keys (Eq. 5-6), kept for the backward pass
  unsigned long long* winkey;                  // [nrep*N] write-back arbitration: (epoch << 33) | occurrence key
  unsigned long long* epoch;                   // [1] bumped once per step, makes stale winkey entries lose
  int32_t* bad_ids;                            // [1] batch node ids outside [0, N) seen by the steps so far
  // distinct (replica, node) rows of the step
  unsigned long long* utag;                    // [nrep*N] epoch of the last step that claimed the node
  int32_t *uidx, *ucount, *ulist;              // [nrep*N] row of a claimed node; [1] number of rows; [maxU] row -> gid
  int32_t* ucount_pair;                        // [2] ucount points at one of them: training steps alternate, and
                                               // each clears the counter of the next one
  int32_t *slot_row, *ucnt, *rowptr, *cursor, *sorted;  // [S] slot -> row; [maxU] slots per row; CSR of slots by row
  int32_t *sorted_row, *sort_total;            // [S] row of every sorted slot; [1] number of sorted slots
  float* ds_row;                               // [maxS, ldh] gradient reaching s' per row
  float* dstat;                                // [maxS, ldst] gradient reaching the static columns per row (co-training)
  struct AdamSet* adam_dev;                    // device copy of the Adam moment pointers and constants
  int32_t* adam_t;                             // [1] Adam steps so far
  BatchSet* bs_dev;                            // device copy of the step's batch descriptors
  struct SgdSet* sgd_dev;                      // device copy of the parameter/gradient pointer table
  float* q_part;                               // [QPHI_BLOCKS, d_o] column sums of dq per block of roots
  // GRU
  float *X, *Hm, *gi, *gh, *gates;             // [S,ldx] [S,ldh] [S,ld3] [S,ld3] [S,4*ldh]
  float* Xrow;                                 // [S,ldxr] x = {s' | static} per distinct node (row)
  float *dgi, *dgh;                            // [S,ld3] [S,ld3]
  // attention.  The projections of x = {s' | static} are taken once per distinct node (P); the slots' own
  // inputs {e | Phi} never leave the attention kernels, which work with per-root vectors instead (k_attn.hip).
  float *P, *dP;                               // [S,ldp]
  float *Umat;                                 // [S,ldz] per node row and head: (W_k^c)_h^T q_h
  float *prob, *Onode, *Omat, *z;              // [R,H*k] [R,ldh] node part of the attention output [R,ldh] [R,ldh]
  float *dz, *dOmat, *dqn, *dq;                // [R,ldh] x 4 (dqn: node part of dq)
  float *Gmat;                                 // [R,ldz] per root and head: (W_v^c)_h^T dO_h
  float *Zs, *Zp, *Qroot;                      // [R,ldz] x 2 (per head: sums of the slots' {e | Phi} rows), [R,ldh]
  float *Yt;                                   // [R,ldy] per root: time-encoding gradient sums of its keys
  float *dscore;                               // [R,H*k] gradients of the attention scores
  // decoder
  float *Pdec, *dPdec, *h1, *logits;           // [R,ldkv] [R,ldkv] [pairs,ldh] [pairs] (classification: [B, nC])
  float* dlog;                                 // [B, ldc] d loss / d logit of the edge-classification head
  float* loss_acc;                                   // [TGNN_MAX_BATCHES] per-batch loss sums
  // packed weights
  float *Wih_p, *Whh_p, *Wdec_p;
  float *Wx, *bias_x;       // [ldkv + 2 d_o, ldxr] rows {W_k ; W_v ; 0 ; W_q ; W_o} restricted to the x columns; [ldp]
  // {e | Phi} columns of W_k, W_v, block-diagonal over the heads (off-diagonal blocks stay zero):
  float *WkcT, *WvcT;       // [H dcp, ldh]  row h dcp + c, column d of head h: W[d, d_x + c]   (U = q WkcT^T, G = dO WvcT^T)
  float *Wkc, *Wvc;         // [d_o, ldz]    row d of head h, column h dcp + c: W[d, d_x + c]   (dq += Zs Wkc^T, O += Zp Wvc^T)
  float *Wo_o;              // [d_o, ldh] W_o restricted to the attention-output columns
  float *rc_pk;             // six [d_o, d_o] blocks in MFMA B-operand order for the root chain (NULL: it does not fit)
  float *WdecT, *WihT_phi;
  float *WxT;               // [d_x, ldp]   transposed Wx (rows >= d_m: the static columns)
  float *WoT_o;             // [d_o, ldh]   transposed Wo_o
};

}  // namespace tgnn

namespace tgnn {
constexpr int PROF_RING = 4096;
struct Profiler {
  uint32_t mask = 0;     // stages to time
  uint32_t active = 0;   // the mask in effect for the tgnn_train_step being enqueued (0 between timed steps)
  int every = 1, calls = 0;
  hipEvent_t* ev[TGNN_N_STAGES][2] = {};  // lazily created rings
  int count[TGNN_N_STAGES] = {};
};
}  // namespace tgnn

namespace tgnn {
// A captured tgnn_train_step: every launch of the step recorded once into a HIP graph and replayed with one
// call; only the prologue node's arguments (the batch descriptors) change between replays.
constexpr int MAX_STEP_GRAPHS = 8;
// (tgnn_train_steps records several consecutive steps of the same shape into one graph: one first-launch node each)
struct StepKey {
  const void* ptr[64];
  int32_t n[TGNN_MAX_BATCHES], rep[TGNN_MAX_BATCHES];
  int32_t nb, parity, n_steps, nneg, mode;   // mode: 0 training, 1 edge classification, 2 evaluation
  float lr;
};
struct StepGraph {
  bool used = false;
  StepKey key;
  hipGraph_t graph = nullptr;
  hipGraphExec_t exec = nullptr;
  hipGraphNode_t head_node[TGNN_MAX_STEPS_PER_CALL] = {};   // the first launch of every recorded step
  unsigned long long last_use = 0;
};
}  // namespace tgnn

namespace tgnn {
// what the last tgnn_temporal_attn_fwd was given and tgnn_temporal_attn_bwd reads again
struct AttnCall {
  const float* e_nbr = nullptr;
  const double* dt_nbr = nullptr;
};
}  // namespace tgnn

struct tgnn_ctx {
  tgnn::Profiler prof;
  tgnn::AttnCall last_attn;
  hipStream_t side = nullptr;      // second stream for work that is off the critical path of a step
  hipEvent_t fork_ev[16] = {};     // fork/join events between the caller's stream and `side`
  int next_ev = 0;
  tgnn::StepGraph graphs[tgnn::MAX_STEP_GRAPHS];   // captured steps, one per distinct call signature
  unsigned long long graph_clock = 0;
  tgnn_config cfg;
  tgnn::Dims d;
  void* arena;
  size_t arena_bytes;
  tgnn::Ws w;
  int last_attn_roots;
  int device;
  int step_parity = 0;             // which of the two row counters the next training step uses
  // what the call in progress asks of its step beyond training (calls on one context are ordered by the caller)
  bool eval = false;               // tgnn_eval_step: forward half, ranks and write-back only
  float* out_rank = nullptr;       // ... its per-event ranks and the sum of their reciprocals
  float* out_rr = nullptr;
  int32_t* out_counts = nullptr;   // ... or, on a classification context, its tp / fp / fn counts
  bool adam = false;               // tgnn_set_optimizer: the in-step update is Adam's
  bool train_static = false;       // tgnn_train_static
  float* grad_static = nullptr;
  float lr_static = 0.f;
};

namespace tgnn {

int set_error(int code, const char* fmt, ...);
#define TGNN_HIP_CHECK(expr)                                                              \
  do {                                                                                    \
    hipError_t _e = (expr);                                                               \
    if (_e != hipSuccess)                                                                 \
      return tgnn::set_error(TGNN_E_HIP, "%s failed: %s", #expr, hipGetErrorString(_e));  \
  } while (0)
#define TGNN_LAUNCH_CHECK() TGNN_HIP_CHECK(hipGetLastError())

// Pointer table of the SGD update (and of "clear these tensors").
struct SgdSet {
  float* p[20];
  const float* g[20];
  int n[20];
  int cnt;
};

// Adam's moment tensors and constants (tgnn_set_optimizer), in the order of the SGD pointer table.
struct AdamSet {
  float* m[20];
  float* v[20];
  float beta1, beta2, eps;
  const int32_t* t;   // device step counter (already counting the step being applied)
};
// Sparse update of the co-trained static memory: row r of drow is the gradient of static[ulist[r] % N].
struct StatUpd {
  const float* drow = nullptr;    // NULL: off
  int ld = 0, ds = 0, N = 0;
  const int32_t* ulist = nullptr;
  const int32_t* ucount = nullptr;
  float* stat = nullptr;
  float* gstat = nullptr;         // may be NULL
  float lr = 0.f;
  int blocks = 0;
};

// Last-event-wins write-back (k_writeback.hip) as a record, so that it can ride in another launch.
struct WbPtrs {
  float *mem, *mail;
  double *mem_ts, *mail_ts;
  int32_t* mail_eid;
  const float *s_new, *s_src, *s_dst;
  const double *tau, *tau_src, *tau_dst;
  const int32_t* slot_row;
  int p_s;
};
struct WbArgs {
  const BatchSet* bs = nullptr;   // NULL: nothing to do
  int N = 0, dm = 0, vec = 1;     // vec: 4 when rows can be copied 16 bytes at a time
  WbPtrs w;
  const unsigned long long* winkey = nullptr;
  const unsigned long long* epoch = nullptr;
  int32_t* out_winner = nullptr;
  int wb_blocks = 0;              // blocks of 256 threads for the scatter ...
  const SgdSet* sgd = nullptr;    // ... followed by 64 per tensor for the update p -= lr * g (NULL: none)
  int sgd_cnt = 0;
  float lr = 0.f;
  const AdamSet* adam = nullptr;  // non-NULL: the update is Adam's
  StatUpd stat;                   // ... followed by stat.blocks for the static-memory rows
};
inline int wb_total_blocks(const WbArgs& a) {
  return a.bs != nullptr ? a.wb_blocks + (a.sgd != nullptr ? 64 * a.sgd_cnt : 0) + a.stat.blocks : 0;
}

// ---- k_gemm.hip ---------------------------------------------------------------------
// C[m, n] = sum_k A[m, k] * B[n, k] + bias[n]  (m < M, n < N), optional ReLU; columns [N, n_store) of C are
// set to zero.  Kp (multiple of 32) columns of A and B are read; B rows >= N and A rows >= M read as zero.
// m_dev (device pointer, may be NULL): the number of valid rows is min(M, *m_dev); the grid is sized for M.
// RowAdd (optional): row m of C additionally receives src[idx * ld + n] for n < N, with idx = index[m]
// (index[m] < 0: nothing is added) or, without an index array, idx = m + row0.  gate (optional, applied
// last): C[m, n] is set to zero where gate[m * ld_gate + n] is not positive (the ReLU gate of a stored output).
struct RowAdd {
  const float* src = nullptr;
  const int32_t* index = nullptr;
  int ld = 0, row0 = 0;
  const float* gate = nullptr;
  int ld_gate = 0;
};
// TimeGradOut (optional): C is not written.  Instead C[m, n] is taken as the gradient reaching the time encoding
// Phi(delta[m])_n = cos(w[n] delta[m] + b[n]) and each 64-row tile adds the column sums of its part of
//   dL/dw[n] = sum_m C[m, n] (-sin(w[n] delta[m] + b[n])) delta[m],   dL/db[n] = the same without the factor delta[m]
// to g_w[n] / g_b[n] (one float atomic each per tile and column).
constexpr int NT_BM = 64;
struct TimeGradOut {
  const double* delta = nullptr;
  const float *w = nullptr, *b = nullptr;
  float *g_w = nullptr, *g_b = nullptr;   // g_w != NULL switches the epilogue on
};
// GruBwdOut (optional): C is not written.  C[m, n] (n < d_m) is taken as the gradient reaching s' of node row m
// and turned into the gradients of the GRU gate pre-activations (Eq. 3), written to dgi / dgh [M, ld3] as
// {r | z | n} blocks of d_m columns; rows with has[m] == 0 (no mail: s' = s) get zeros.  gates holds
// {r | z | n | W_hn h + b_hn} per row in blocks of ldh columns, Hm the stored memory (pitch ldh).
struct GruBwdOut {
  const float* gates = nullptr;
  const float* Hm = nullptr;
  const int32_t* has = nullptr;
  float *dgi = nullptr, *dgh = nullptr;
  int dm = 0, ldh = 0, ld3 = 0;
};
void gemm_nt(const float* A, int lda, const float* B, int ldb, const float* bias, float* C, int ldc, int M,
             int N, int Kp, int n_store, bool relu, hipStream_t s, const int* m_dev = nullptr,
             const RowAdd& add = RowAdd(), const TimeGradOut& tg = TimeGradOut(),
             const GruBwdOut& gb = GruBwdOut());
// The same product as a record, so that two independent ones can share a launch (gemm_nt_group: the tile
// width is chosen for the first problem; col_tiles and wg_begin are filled in by the launcher).
struct NtProblem {
  const float *A, *B, *bias;
  float* C;
  int lda, ldb, ldc, M, N, Kp, n_store, relu;
  int k_live;   // columns >= k_live of A and B are padding (0: not stated); lets the last stage stop after 16 columns
  // bd_n > 0: B is block-diagonal, rows [h bd_n, (h + 1) bd_n) of it (output columns) are zero outside columns
  // [h bd_k, (h + 1) bd_k): a column tile then runs only the k stages its blocks reach into
  int bd_n, bd_k;
  const int* m_dev;
  int col_tiles, wg_begin;
  RowAdd add;
  TimeGradOut tg;
  GruBwdOut gb;
  // optional: the column sums of the stored tile are added to colsum[(tile & (colsum_rows - 1)) * N + n]
  // (colsum_rows partial rows, a power of two, keep the float atomics of different tiles apart)
  float* colsum;
  int colsum_rows;
};
struct NtGroup {
  NtProblem p[2];
  int n;
  int gemm_wgs;   // workgroups of the products; the ones after them run `tail`
  WbArgs tail;    // optional passenger: write-back scatter + SGD (wb_total_blocks(tail) blocks)
};
inline NtProblem nt_problem(const float* A, int lda, const float* B, int ldb, const float* bias, float* C, int ldc, int M,
                            int N, int Kp, int n_store, bool relu, const int* m_dev = nullptr,
                            const RowAdd& add = RowAdd(), const TimeGradOut& tg = TimeGradOut(),
                            const GruBwdOut& gb = GruBwdOut()) {
  NtProblem p;
  p.A = A; p.B = B; p.bias = bias; p.C = C; p.lda = lda; p.ldb = ldb; p.ldc = ldc; p.M = M; p.N = N; p.Kp = Kp;
  p.n_store = n_store; p.relu = relu ? 1 : 0; p.k_live = 0; p.m_dev = m_dev; p.col_tiles = 0; p.wg_begin = 0;
  p.add = add; p.tg = tg; p.gb = gb; p.colsum = nullptr; p.colsum_rows = 1; p.bd_n = 0; p.bd_k = 0;
  return p;
}
// the same problem with its live column count stated
inline NtProblem nt_live(NtProblem p, int k_live) { p.k_live = k_live; return p; }
// the same problem with B stated to be block-diagonal (see NtProblem::bd_n)
inline NtProblem nt_blocks(NtProblem p, int bd_n, int bd_k) { p.bd_n = bd_n; p.bd_k = bd_k; return p; }
void gemm_nt_group(const NtProblem* probs, int n, hipStream_t s, const WbArgs* tail = nullptr);

// Where the weight-gradient GEMM adds its result: element (n, k) goes to p[n >= n_split][k >= k_split]
// (indices taken relative to the split) with row pitch ld[..][..]; column sums of D go to bias[n >= n_split].
// head_k > 0 (then only p[0][0] is used): A holds one block of head_k columns per attention head and D's columns
// belong to heads of head_n columns each; element (n, k) is kept only where both heads agree, and goes to
// column k % head_k (dropped when >= head_cols) of row n.
struct OutMap {
  float* p[2][2];
  int ld[2][2];
  int n_split, k_split;
  float* bias[2];
  int head_n, head_k, head_cols;
};
// One weight-gradient problem G[n, k] += sum_m D[m, n] * A[m, k] and a group of them for one launch.
struct TnProblem {
  const float* D;
  const float* A;
  const int* m_dev;
  int ldd, lda, M, N, K;
  int m_chunk, tiles, chunks;   // tiles: workgroups per chunk of rows
  int heads;                    // out.head_k > 0: number of per-head blocks (N / head_n), else 1
  // Placement of the workgroups (one per chunk and tile).  Workgroup b of the launch runs on XCD b % 8; the
  // workgroups of XCD x form a queue of their own (position b / 8), in which this problem's start at
  // lane_begin[x].  XCD x works on the chunks v, v + 8, ... with v = (x + rot) % 8, all tiles of a chunk in a
  // row, so that the rows of a chunk are fetched into one L2 only.
  int rot, lane_begin[8];
  OutMap out;
};
constexpr int TN_MAX_GROUP = 10;
struct TnGroup {
  TnProblem p[TN_MAX_GROUP];
  int n;
  // The XCD queues once more, in the form a workgroup reads with two scalar loads: the problems in placement
  // order (qprob), and per XCD the queue position at which each of them starts, ascending, closed by the end of
  // the queue and padded with INT_MAX (qbegin).
  int qbegin[8][16];
  unsigned char qprob[16];
};
struct TnBatch {
  TnGroup g;
  // rows to expect of a problem whose row count lives on the device (the chunking is laid out for it; any count
  // works, a poor guess only costs time).  0: an eighth of the problem's bound.
  int dev_rows_est = 0;
  TnBatch() { g.n = 0; }
  void add(const float* D, int ldd, const float* A, int lda, int M, int N, int K, const OutMap& out,
           const int* m_dev = nullptr);
  void launch(hipStream_t s);   // one kernel for all added problems; empties the batch
};
// G[n, k] += sum_m D[m, n] * A[m, k]  (n < N, k < K), bias[n] += sum_m D[m, n]; float atomics.
void gemm_tn_acc(const float* D, int ldd, const float* A, int lda, int M, int N, int K, const OutMap& out,
                 hipStream_t s, const int* m_dev = nullptr);

// ---- k_misc.hip ---------------------------------------------------------------------
struct PackDesc {
  const float* src;
  float* dst;
  int rows, cols, zero_to, ldd;  // dst[r*ldd + c] = src[r*srs + c*scs] for c < cols, 0 for cols <= c < zero_to
  int srs, scs;
  // mfma_ks > 0: MFMA B-operand order instead (zero_to, ldd unused).  For column block cb (16 rows), k slab s < mfma_ks
  // (16 columns), lane (li, lg) and c < 4:  dst[((cb * mfma_ks + s) * 64 + lg * 16 + li) * 4 + c] =
  // src[(16 cb + li) * srs + (16 s + 4 lg + c) * scs], zero beyond rows / cols: a wavefront then reads the operand
  // of one MFMA slab as 1 KB of contiguous memory.
  int mfma_ks;
  // nblk > 0: block-diagonal instead (zero_to, mfma_ks unused).  For block h < nblk, r < rows, c < cols:
  // dst[(h * brd + r) * ldd + h * bcd + c] = src[h * bsrc + r * srs + c * scs]; nothing else is written.
  int nblk, brd, bcd, bsrc;
};
constexpr int MAX_PACK = 32;
struct PrologueArgs {
  PackDesc d[MAX_PACK];
  int n_pack;
  SgdSet zero;          // tensors to clear (cnt = 0: none)
  BatchSet bs;          // copied to *bs_dev when bs_dev != NULL
  BatchSet* bs_dev;
  SgdSet sgd;           // copied to *sgd_dev when sgd_dev != NULL
  SgdSet* sgd_dev;
  float* loss;
  unsigned long long* epoch;
  int32_t* ucount;
  // bq_out[n] = bq[n] + sum_c wq[n, dx + c] * cos(time_b[c]): the query's time encoding Phi(0) is a constant
  const float *bq, *wq, *time_b;
  float* bq_out;
  int dO, dq, dx, dt;
  float* q_part;        // cleared (q_part_n floats)
  int q_part_n;
  // head_of_step: this runs inside the first launch of a training step, beside the sampler.  The sampler then
  // works with epoch + 1 and with a row counter that is already zero, so neither is touched here; instead the
  // row counter of the next step (ucount_next) is cleared.  Otherwise: epoch += 1, *ucount = 0.
  int head_of_step;
  int32_t* ucount_next;
  int32_t* adam_t;      // non-NULL: *adam_t += 1 (one Adam step is about to be applied)
};
void prologue_fill(tgnn_ctx* ctx, const tgnn_params* p, const BatchSet* bs, const SgdSet* sgd, const SgdSet* zero,
                   float* loss, PrologueArgs& pa);
dim3 prologue_grid(const PrologueArgs& pa);
void* prologue_func();
// One launch at the start of a call: packs the weights, optionally zeroes the gradient tensors in `zero`,
// copies the batch descriptors and the SGD pointer table to the device, zeroes *loss, bumps the epoch.
// bs / sgd / zero / loss may be NULL.
void prologue(tgnn_ctx* ctx, const tgnn_params* p, const BatchSet* bs, const struct SgdSet* sgd,
              const struct SgdSet* zero, float* loss, hipStream_t s);
void fill_state(tgnn_ctx* ctx, tgnn_state* st, int replica, hipStream_t s);
void sgd_update(const SgdSet* set_dev, int cnt, float lr, hipStream_t s);
void zero_set(const SgdSet& set, hipStream_t s);
void copy_f4(const void* src, void* dst, size_t n_float4, hipStream_t s);

// ---- k_sample.hip -------------------------------------------------------------------
struct UniqPtrs {
  unsigned long long* utag;
  const unsigned long long* epoch;
  int32_t *uidx, *ucount, *ulist, *ucnt;
};
// The first launch of a training step: roots of every batch (node, time, slot ids), write-back arbitration marks,
// neighbour sampling and row claims (blocks 0 .. sample_blocks - 1, a lane group of 16 or 64 per root, 64 * SAMPLE_WAVES threads per
// block), and, in the blocks after those, everything the prologue does (it depends on nothing the sampler does
// and the other way round: the sampler takes the batch descriptors from the argument block and uses epoch + 1,
// which a later launch makes official).
struct SampleArgs {
  const int64_t* indptr;
  const int32_t *g_nbr, *g_eid;
  const double* g_ts;
  int N, n_roots, k;
  const int32_t* q_node;   // caller's queries (plain sampling only)
  const double* q_t;
  int32_t *out_nbr, *out_eid;
  double* out_ts;
  int32_t* out_cnt;
  int32_t* root_node;
  double* root_t;
  int32_t *slot_gid, *slot_node;
  unsigned long long* winkey;
  int32_t* bad_ids;        // counter of batch node ids outside [0, N) (fused form only)
  UniqPtrs uq;
};
struct HeadArgs {
  SampleArgs sa;
  int sample_blocks, pro_bx;   // pro_bx: prologue blocks per grid row
  PrologueArgs pa;
};
#ifndef TGNN_SAMPLE_WAVES
#define TGNN_SAMPLE_WAVES 8
#endif
constexpr int SAMPLE_WAVES = TGNN_SAMPLE_WAVES;   // wavefronts per block in the first launch of a step (four roots each when k < 16)
void head_fill(tgnn_ctx* ctx, const tgnn_graph* g, int n_roots, const tgnn_params* p, const BatchSet* bs,
               const struct SgdSet* sgd, const struct SgdSet* zero, float* loss, HeadArgs& h);
dim3 head_grid(const HeadArgs& h);
void* head_func();
void step_head(const HeadArgs& h, hipStream_t s);
// Plain sampling of caller-provided queries.
void sample_recent(const Dims& d, const tgnn_graph* g, const int32_t* node, const double* t, int n_roots,
                   int32_t* out_nbr, int32_t* out_eid, double* out_ts, int32_t* out_cnt, hipStream_t s);

// ---- k_unique.hip -------------------------------------------------------------------
// Gradients through the query's time encoding Phi(0) = cos(time_b), from the column sums of dq [R, ld]:
// g_b[c] += -sin(time_b[c]) sum_n colsum[n] wq[n, dx + c] and g_wq[n, dx + c] += colsum[n] cos(time_b[c]).
// The attention backward kernel adds them to q_part [QPHI_BLOCKS, d_o]; qphi_block (qphi_device.h), run as the
// first qphi_blocks() blocks of a later 256-thread launch, turns them into the two gradients.
constexpr int QPHI_BLOCKS = 64;
struct QPhi {
  const float* part = nullptr;   // NULL: no query part
  const float *wq = nullptr, *time_b = nullptr;
  float *g_wq = nullptr, *g_b = nullptr;
  int dO = 0, dq_w = 0, dx = 0, dt = 0;
};
__host__ __device__ inline int qphi_blocks(const QPhi& q) { return q.part != nullptr ? (q.dO * q.dt + 255) / 256 : 0; }
// Slot -> row map and the row-sorted slot list (the latter needed by seg_reduce only).  Three small passes:
// map (slot_row[s] = uidx[slot_gid[s]], slots counted per row), an exclusive scan of the counts, and the fill
// (every slot takes the next free position of its row).  None gets a launch of its own in the training
// step: they ride as extra blocks in the state-gather, GRU-gates and softmax-attention launches
// (unique_device.h).  ucnt == NULL: nothing to do.
struct SortArgs {
  const int32_t* ucount = nullptr;   // device row count
  int32_t* ucnt = nullptr;           // slots per row
  int32_t *rowptr = nullptr, *cursor = nullptr;
  int S = 0;
  const int32_t *slot_gid = nullptr, *uidx = nullptr;
  int32_t* slot_row = nullptr;
  int32_t *sorted = nullptr, *sorted_row = nullptr;   // the sorted slots and, beside them, their rows
  int32_t* total = nullptr;                           // number of sorted slots (= rowptr[*ucount])
};
SortArgs sort_args(tgnn_ctx* ctx, int S);
// Per-row sums of the slot gradients that reach the per-node projections: for a neighbour slot (r, j) the gradient
// of its key / value rows is formed on the fly, dK = ds[r, h, j] q[r], dV = p[r, h, j] dO[r] per head h.
struct SlotGrads {
  const float *dscore, *prob;     // [R, H k]
  const float *Qroot, *dOmat;     // [R, ldh]
  const float *dq, *dz;           // [R, ldh] gradients of the root's own query row and of its merge-layer row
  int R, k, H, dO, dh, ldh;
};
// qphi: rides along in the first blocks (see QPhi)
void seg_reduce(tgnn_ctx* ctx, int R, int S, const QPhi& qphi, hipStream_t s);
// the same with slot = row (standalone attention call): plain stores, every row of dP written
void slots_to_dp(tgnn_ctx* ctx, int R, int RK, const QPhi& qphi, hipStream_t s);
void expand_rows(tgnn_ctx* ctx, int S, const float* src, int ld, const double* src_d, float* dst, double* dst_d,
                 hipStream_t s);

// ---- k_gru.hip ----------------------------------------------------------------------
// GRU gates (Eq. 3) from the two projections gi = W_ih x + b_ih, gh = W_hh h + b_hh, as a record: blocks of 256
// threads, gru_total_blocks() of them.  n_dev (device, may be NULL) caps the row count.  s' goes to
// x_out [n, ld_x]; with stat != NULL the node's static row stat[gid[row] % N] is appended (columns d_m ..
// d_m + d_s).  zero_buf (may be NULL) [n, zero_w] is cleared for the backward pass.  scan.ucnt != NULL: block 0
// runs the scan of the slot sort instead.
struct GruFwdArgs {
  int n_max = 0;
  const int* n_dev = nullptr;
  int dm = 0, ldh = 0, ld3 = 0;
  const float *gi = nullptr, *gh = nullptr, *Hm = nullptr;   // gi == NULL: nothing to do
  const int32_t* has = nullptr;
  float *gates = nullptr, *x_out = nullptr;
  int ld_x = 0;
  const float* stat = nullptr;
  int ds = 0;
  const int32_t* gid = nullptr;
  int N = 0;
  float* zero_buf = nullptr;
  int zero_w = 0, gru_blocks = 0;
  SortArgs scan;
};
__host__ __device__ inline int gru_total_blocks(const GruFwdArgs& a) {
  return a.gi != nullptr ? a.gru_blocks + (a.scan.ucnt != nullptr ? 1 : 0) : 0;
}
GruFwdArgs gru_gates_args(const Dims& d, int n, const int* n_dev, const float* gi, const float* gh, const float* Hm,
                          const int32_t* has, float* gates, float* x_out, int ld_x, const float* stat, const int32_t* gid,
                          float* zero_buf, int zero_w, const SortArgs& scan = SortArgs(), int launch_rows = 0);
void gru_gates_fwd(const GruFwdArgs& a, hipStream_t s);

// ---- k_gather.hip -------------------------------------------------------------------
struct GatherArgs {
  // sources
  const float *mem, *mail, *efeat;
  const double *mem_ts, *mail_ts;
  const int32_t* mail_eid;  // NULL: the staged layout of tgnn_gru_update (row index = slot, has_in given)
  const int32_t* has_in;
  const int32_t* n_dev;     // device row count (NULL: n_slots)
  int launch_rows;          // with n_dev: rows to launch for (0: a quarter of n_slots); the waves stride over the rest
  const int32_t* slot_gid;  // NULL: identity
  int gid_add;              // added to every non-negative slot_gid entry (replica offset)
  // destinations (pitches in floats)
  float *o_mem, *o_mail, *o_ef, *o_phi;  // o_phi NULL: no time encoding
  int p_mem, p_mail, p_ef, p_phi;
  int z_mem, z_mail, z_ef, z_phi;  // number of zero floats to append after each segment (row padding)
  double *o_mem_ts, *o_mail_ts, *o_tau, *o_delta;
  int32_t* o_has;
  const float *time_w, *time_b;
  int n_slots, dm, dt, de;
  SortArgs map;             // map.ucnt != NULL: the first blocks of the launch run the slot -> row map instead
  unsigned long long* epoch_bump;   // may be NULL: *epoch_bump += 1 (the step's epoch becomes official here)
};
void gather_rows(const GatherArgs& a, hipStream_t s);

// Standalone attention call: node rows from the caller's x_root / x_nbr (rows of absent neighbours zeroed).
void stage_x_rows(int R, int k, int dx, const float* x_root, const float* x_nbr, const int32_t* cnt, float* Xrow,
                  int ldxr, hipStream_t s);

// ---- k_attn.hip ---------------------------------------------------------------------
// Arguments of the attention kernels (Eq. 4-7 forward and backward; see k_attn.hip).  Root r's node row is
// slot_row[r], neighbour slot (r, j)'s is slot_row[R + r k + j] (slot_row == NULL: row = slot).
struct FusedAttn {
  int R, k, H, dO, dh, de, dt, dcp, ldz, ldh, ldp, ldy, off_q, dt_source, force_generic;
  const float* P;            // node rows {K | V || q | merge}, pitch ldp; q at column off_q
  const float* U;            // [rows, ldz]
  const int32_t *slot_row, *cnt;
  const float* efeat;        // [E, d_e]; or [R k, d_e] when neid == NULL
  const int32_t* neid;       // [R, k] edge-feature row of every slot
  const double *root_t, *nts, *tau;   // query times [R], edge times [R, k], update times per node row
  const double* dt_in;       // non-NULL: time differences given directly [R k]
  const float *time_w, *time_b;
  double* dtk;               // [R k] time differences: written by the forward pass, read by the backward pass
  float* prob;               // [R, H k] softmax weights
  float *Onode, *Zp;         // forward out: node part of the attention output [R, ldh], per-head sums [R, ldz]
  const float *dOmat, *G;    // backward in: gradient of the attention output [R, ldh], G [R, ldz]
  float *dscore, *dqn, *Zs, *Y, *Qroot;   // backward out
  SortArgs fill;             // forward only, fill.ucnt != NULL: the first blocks run the fill pass of the slot sort
};
void fattn_fwd(const FusedAttn& a, hipStream_t s);
void fattn_bwd(const FusedAttn& a, hipStream_t s);

// ---- k_decoder.hip ------------------------------------------------------------------
void decoder_pairs(const Dims& d, const BatchSet* bs, int total, const float* Pdec, int ldp, const float* b1,
                   const float* w2, const float* b2, float* logits, float* out_loss, float* h1, float* dPdec,
                   float* g_w2, float* g_b2, hipStream_t s);
// Edge-classification head (nC outputs, targets in the batch descriptors): hidden layer, logits [total, nC], loss,
// d loss / d logit (dlog, pitch ldc), and per root the gradient of its Pdec row.
void decoder_classes(const Dims& d, const BatchSet* bs, int total, const float* Pdec, int ldp, const float* b1,
                     const float* w2, const float* b2, float* logits, float* out_loss, float* h1, float* dPdec,
                     float* dlog, hipStream_t s);
// rank[ev] = 1 + #(negative pairs of the event scoring above its true pair) + 0.5 #(scoring the same); rr_sum += sum 1/rank
void reciprocal_ranks(const BatchSet* bs, int total, const float* logits, float* rank, float* rr_sum, hipStream_t s);
// counts[0..2] += tp, fp, fn of the predictions logit > 0 against the batches' class targets (logits [total, C])
void class_counts(const BatchSet* bs, int total, int C, const float* logits, int32_t* counts, hipStream_t s);
void mask_dz(int R, int dO, const float* dz_in, int p_in, const float* z, int ldz, float* dz_out, hipStream_t s);
// d_x_root[r, c] = ds_row[r, c];  d_x_nbr[j, c] = ds_row[R + j, c]   (c < dm, outputs pitch dm)
void attn_dx_out(int R, int RK, int dm, const float* ds_row, int ldh, float* d_x_root, float* d_x_nbr, hipStream_t s);
void zero_f32(float* p, int n, hipStream_t s);

// ---- k_rootchain.hip ----------------------------------------------------------------
// Merge layer, decoder with loss, and their backward pass down to the gradient of the attention output, for
// the roots of a step in one launch.
struct ChainArgs {
  int nb, n[TGNN_MAX_BATCHES];   // batch sizes (events of batch b follow those of the batches before it); set by root_chain
  int dO, ldh, ldkv, ldp;
  const float* Omat;          // [R, ldh] attention output
  const float* P_o;           // node part of the merge layer (bias included), row pitch ldp
  const int32_t* slot_row;    // root slot -> node row (NULL: identity)
  // weight blocks in MFMA B-operand order (see PackDesc): merge layer (attention-output columns), W_s, W_d, and
  // their transposes
  const float *Wo_pk, *Ws_pk, *Wd_pk, *WsT_pk, *WdT_pk, *WoT_pk;
  const float *b1, *w2, *b2;
  float *z, *h1, *logits, *dPdec, *dz, *dOmat;
  float *loss, *g_w2, *g_b2;
};
bool root_chain_fits(const Dims& d);
// force_wide: 16 events per workgroup whatever the size of the step (otherwise 5 when there are few events)
void root_chain(ChainArgs a, const BatchSet& bs_host, bool force_wide, hipStream_t s);

// ---- k_writeback.hip ----------------------------------------------------------------
void writeback_mark(const Dims& d, const BatchSet* bs, int total, unsigned long long* winkey,
                    const unsigned long long* epoch, hipStream_t s);
// Fused layout: s_new/tau indexed by root slot.  Standalone layout: separate src/dst arrays.
void writeback_scatter(const Dims& d, const BatchSet* bs, int total, const tgnn_state* st,
                       const unsigned long long* winkey, const unsigned long long* epoch, const float* s_new, int p_s,
                       const double* tau, const int32_t* slot_row, const float* s_src, const float* s_dst, const double* tau_src,
                       const double* tau_dst, int32_t* out_winner, hipStream_t s,
                       const SgdSet* sgd_dev = nullptr, int sgd_cnt = 0, float lr = 0.f);
// The same as a record (for a launch that carries it as a passenger); blocks of 256 threads.
WbArgs writeback_args(const Dims& d, const BatchSet* bs, int total, const tgnn_state* st, const unsigned long long* winkey,
                      const unsigned long long* epoch, const float* s_new, int p_s, const double* tau,
                      const int32_t* slot_row, const float* s_src, const float* s_dst, const double* tau_src,
                      const double* tau_dst, int32_t* out_winner, const SgdSet* sgd_dev, int sgd_cnt, float lr);
// key of occurrence (event e = ev_off + i, role) in the step with epoch counter `epoch`
__host__ __device__ inline unsigned long long wb_key(unsigned long long epoch, int e, int role) {
  return (epoch << 33) | (1ull + 2ull * (unsigned long long)e + (unsigned long long)role);
}

}  // namespace tgnn
