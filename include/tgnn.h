/*
 * libtgnn -- the per-mini-batch training step of a memory-based temporal graph neural network
 * (TGN-attn with static node memory, as trained by DistTGL, arXiv 2307.07649) on one AMD MI355X.
 *
 * Conventions
 *   - plain C ABI; every call returns 0 (TGNN_OK) or a negative TGNN_E_* code, and leaves a message
 *     that tgnn_last_error() returns (thread-local, valid until the next failing call on the thread);
 *   - unless marked HOST, every pointer is a DEVICE pointer owned by the caller, row-major,
 *     contiguous, 16-byte aligned; the library never frees or reallocates caller memory;
 *   - the structs themselves (tgnn_config, tgnn_graph, ...) are host structs passed by pointer;
 *   - node and event ids are int32, CSR offsets int64, timestamps double, everything else float;
 *   - `stream` is a hipStream_t (NULL = the default stream); calls are asynchronous on it and never
 *     synchronise the device, except tgnn_destroy;
 *   - a context owns a device workspace sized at tgnn_create; two calls that use one context must
 *     be ordered on one stream;
 *   - padding: nbr = eid = -1 for a missing neighbour, mail_eid = -1 for "no cached mail".
 *
 * Notation: B events in a batch; roots R = 3B in the order [sources | destinations | negative
 * destinations]; k most recent neighbours per root; d_m memory width, d_t time-encoding width,
 * d_e edge-feature width, d_s static-memory width (0 = none), H heads;
 *   d_in = 2 d_m + d_t + d_e,  d_x = d_m + d_s,  d_q = d_x + d_t,  d_kv = d_x + d_e + d_t,  d_o = d_m.
 */
#ifndef TGNN_H
#define TGNN_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TGNN_OK 0
#define TGNN_E_INVALID_ARG (-1)
#define TGNN_E_NULL_PTR (-2)
#define TGNN_E_MISALIGNED (-3)
#define TGNN_E_OUT_OF_RANGE (-4)
#define TGNN_E_UNSORTED_TS (-5)
#define TGNN_E_UNSUPPORTED_DIM (-6)
#define TGNN_E_WORKSPACE (-7)
#define TGNN_E_HIP (-8)

#define TGNN_FLAG_OVERWRITE_GRADS 1 /* tgnn_train_step clears `grads` first instead of adding to them */
#define TGNN_FLAG_NO_GRAPH 4        /* tgnn_train_step enqueues its launches (16 on the main path) one by one; by default it records
                                       them once per call signature (same pointers, batch sizes, lr, stream) into a
                                       HIP graph and replays that with one launch, updating only the batch
                                       descriptors.  Not used on the NULL (legacy default) stream, while the caller's stream is itself being captured
                                       or while stage timing is enabled. */
#define TGNN_FLAG_WIDE_ROOT_TILES 8  /* tgnn_train_step's root chain (merge layer, decoder, loss and their backward
                                       pass in one launch) takes 16 events per workgroup whatever the size of the
                                       step; by default steps of at most 1,280 events take 5 per workgroup.  Same
                                       results up to the order of the sums over workgroups; for tests. */
#define TGNN_FLAG_GENERIC_ATTN 16    /* the attention kernels take their generic code path (any k, widths and number of
                                       heads) also where the shape fits the register-resident one; for tests */
#define TGNN_FLAG_SIDE_STREAM 2     /* tgnn_train_step starts the bulk of the weight-gradient GEMMs (decoder, merge
                                       layer, {e | Phi} columns of W_k / W_v) on a second stream of the context as
                                       soon as their operands exist, beside the remaining chain of small backward
                                       kernels; forked from and joined back into the caller's stream with one
                                       event each inside the call.  Off by default: measured on MI355X the two
                                       streams get in each other's way and the step takes a few per cent longer,
                                       launched one by one and as a captured graph alike. */

#define TGNN_MAX_K 32        /* neighbours per root */
#define TGNN_MAX_BATCHES 16  /* mini-batches (memory replicas) per tgnn_train_step call */
#define TGNN_MAX_STEPS_PER_CALL 8 /* consecutive training steps per tgnn_train_steps call */
#define TGNN_MAX_HEADS 8
#define TGNN_MAX_NEG_SETS 64 /* negative-destination sets per event (tgnn_train_step_epoch_parallel, tgnn_eval_step) */
#define TGNN_MAX_CLASSES 256 /* outputs of the edge-classification head (tgnn_train_step_edge_class) */
#define TGNN_NOALLOC_MAX_NODES 262144   /* tgnn_memory_writeback_noalloc: nodes its static scratch array covers (2 MiB) */
#define TGNN_NOALLOC_MAX_EVENTS 1048576 /* ... and events per call */

typedef struct tgnn_ctx tgnn_ctx;

typedef struct {
  int32_t n_nodes, d_mem, d_time, d_edge, d_static, n_heads, k;
  int32_t max_batch;  /* largest number of events in one mini-batch */
  int32_t n_replicas; /* independent memory/mailbox copies (memory parallelism, Sec. 3.2.3); >= 1 */
  int32_t dt_source;  /* time difference in the attention keys (Eq. 5-6): 0 = query time minus the update
                         time of the neighbour's memory as used (the paper's wording), 1 = minus the edge time */
  int32_t flags;      /* TGNN_FLAG_* bits */
  int32_t max_neg_sets; /* largest number of negative-destination sets a step carries (tgnn_train_step_epoch_parallel,
                           tgnn_eval_step); 0 or 1: one, the plain step.  The workspace grows with it. */
  int32_t n_classes;    /* 0: link prediction (dec_w2 [d_o], dec_b2 [1]).  C > 0: the decoder is an edge-classification
                           head with C outputs (dec_w2 [C, d_o], dec_b2 [C]); such a context trains with
                           tgnn_train_step_edge_class only.  C <= TGNN_MAX_CLASSES. */
} tgnn_config;

/* Temporal CSR: node v's incident events (both directions) are entries indptr[v] .. indptr[v+1]-1 of
 * nbr/eid/ts, ascending in (time, event id).  efeat is [n_events, d_edge]. */
typedef struct {
  const int64_t* indptr; /* [n_nodes + 1] */
  const int32_t* nbr;    /* [2 n_events] other endpoint */
  const int32_t* eid;    /* [2 n_events] event id */
  const double* ts;      /* [2 n_events] event time */
  const float* efeat;    /* [n_events, d_edge], may be NULL when d_edge == 0 */
  int64_t n_events;
} tgnn_graph;

/* Node state; every array has leading dimension n_replicas (replica r, node v -> row r*n_nodes + v).
 * Sec. 2.1: memory s_v (zero-initialised), its last-update time t_v^-, and the cached mail. */
typedef struct {
  float* mem;        /* [n_replicas * n_nodes, d_mem] */
  double* mem_ts;    /* [n_replicas * n_nodes] */
  float* mail;       /* [n_replicas * n_nodes, 2 d_mem]  {s'_self || s'_other} of the last event */
  double* mail_ts;   /* [n_replicas * n_nodes] time of that event */
  int32_t* mail_eid; /* [n_replicas * n_nodes] id of that event (its edge feature is looked up), -1 = none */
  const float* stat; /* [n_nodes, d_static] frozen static node memory (Sec. 3.1), NULL when d_static == 0 */
} tgnn_state;

/* Parameters; the same struct carries gradients.  Matrices are [out, in] row-major.
 *   time_w, time_b [d_t]                         Phi(dt)_c = cos(time_w[c] * dt + time_b[c])
 *   gru_wih [3 d_m, d_in], gru_whh [3 d_m, d_m], gru_bih, gru_bhh [3 d_m]    gate order r, z, n;
 *           input columns ordered {mail (2 d_m) || Phi (d_t) || edge feature (d_e)}  (Eq. 1-2)
 *   wq [d_o, d_q], wk, wv [d_o, d_kv], biases [d_o]; key/value input {x_w || e_vw || Phi} (Eq. 4-6)
 *   wo [d_o, d_o + d_x], bo [d_o]                merge layer on {h_v || x_v}
 *   dec_ws, dec_wd [d_o, d_o], dec_b1 [d_o], dec_w2 [d_o], dec_b2 [1]        link decoder
 *           (config.n_classes = C > 0: dec_w2 [C, d_o], dec_b2 [C], the edge-classification head) */
typedef struct {
  float *time_w, *time_b, *gru_wih, *gru_whh, *gru_bih, *gru_bhh, *wq, *bq, *wk, *bk, *wv, *bv, *wo, *bo,
      *dec_ws, *dec_wd, *dec_b1, *dec_w2, *dec_b2;
} tgnn_params;

/* One chronological mini-batch of events (u_i, v_i, e_i, t_i) with one sampled negative destination
 * n_i per event, advancing memory replica `replica`. */
typedef struct {
  const int32_t *src, *dst, *neg, *eid; /* [n] */
  const double* t;                      /* [n] */
  int32_t n;
  int32_t replica;
} tgnn_batch;

const char* tgnn_last_error(void);

/* Validates the configuration (TGNN_E_UNSUPPORTED_DIM: d_mem % n_heads != 0, k > TGNN_MAX_K, n_heads >
 * TGNN_MAX_HEADS, a width that is not positive, d_edge or d_static negative) and allocates the workspace
 * on the current HIP device (TGNN_E_WORKSPACE / TGNN_E_HIP on failure). */
int32_t tgnn_create(const tgnn_config* cfg, tgnn_ctx** out);
/* Synchronises the device and frees the workspace.  NULL is accepted. */
int32_t tgnn_destroy(tgnn_ctx* ctx);
/* Bytes of device workspace the context holds. */
int64_t tgnn_workspace_bytes(const tgnn_ctx* ctx);

/* HOST.  Builds the temporal CSR from a chronological event list (src, dst, ts: HOST arrays [n_events],
 * ts non-decreasing -> else TGNN_E_UNSORTED_TS; ids in [0, n_nodes) -> else TGNN_E_OUT_OF_RANGE) into
 * caller-allocated HOST arrays indptr [n_nodes+1], nbr/eid/ts_out [2 n_events].  Every event is listed
 * under both endpoints; each list ascends in (time, event id).  (Sec. 2.1, "most recent neighbors".) */
int32_t tgnn_build_tcsr(const int32_t* src, const int32_t* dst, const double* ts, int64_t n_events,
                        int32_t n_nodes, int64_t* indptr, int32_t* nbr, int32_t* eid, double* ts_out);

/* Epoch start (Alg. 1 "reset memory and mail"): zero memory, mails and both time arrays and set
 * mail_eid = -1 for one replica (replica = -1: all replicas). */
int32_t tgnn_state_reset(tgnn_ctx* ctx, tgnn_state* st, int32_t replica, void* stream);

/* Sec. 2.1 "most recent neighbors", k = 10 in Sec. 4.  For each query (node[r], t[r]), r < n_roots: the
 * min(k, #) incident events with time strictly below t[r] that are last in (time, event id) order, most
 * recent first.  out_nbr, out_eid [n_roots, k] int32 (-1 padded), out_ts [n_roots, k] double (0 padded),
 * out_cnt [n_roots].  n_roots <= 3 * max_batch * n_replicas.  Node ids must lie in [0, n_nodes)
 * (not checked on the device: rows of out-of-range nodes are reported as empty). */
int32_t tgnn_sample_recent(tgnn_ctx* ctx, const tgnn_graph* g, const int32_t* node, const double* t,
                           int32_t n_roots, int32_t* out_nbr, int32_t* out_eid, double* out_ts,
                           int32_t* out_cnt, void* stream);

/* Sec. 3.2.1: fetch the node memory and cached mails of root and supporting nodes.  For each slot
 * s < n_slots with node w = slot_node[s] of replica `replica` (w = -1: padding, the row is zero-filled):
 * out_mem [n_slots, d_m] = mem[w]; out_mail [n_slots, 2 d_m] = mail[w]; out_mail_efeat [n_slots, d_e] =
 * efeat[mail_eid[w]] (zeros when there is no mail); out_mem_ts, out_mail_ts [n_slots]; out_has_mail
 * [n_slots] = 1 if mail_eid[w] >= 0.  n_slots <= workspace slot capacity (3 B (1+k) per batch). */
int32_t tgnn_gather_memory(tgnn_ctx* ctx, const tgnn_graph* g, const tgnn_state* st, int32_t replica,
                           const int32_t* slot_node, int32_t n_slots, float* out_mem, float* out_mail,
                           float* out_mail_efeat, double* out_mem_ts, double* out_mail_ts,
                           int32_t* out_has_mail, void* stream);

/* Eq. 3 with the mail of Eq. 1-2: for each staged row s (the outputs of tgnn_gather_memory):
 * has_mail ? s' = GRU({mail || Phi(mail_ts - mem_ts) || mail_efeat}, mem), tau = mail_ts
 *          : s' = mem, tau = mem_ts.    out_s_new [n_slots, d_m], out_tau [n_slots]. */
int32_t tgnn_gru_update(tgnn_ctx* ctx, const tgnn_params* p, int32_t n_slots, const float* mem,
                        const float* mail, const float* mail_efeat, const double* mem_ts,
                        const double* mail_ts, const int32_t* has_mail, float* out_s_new, double* out_tau,
                        void* stream);

/* Eq. 4-7 plus the merge layer.  x_root [n_roots, d_x] = {s'_v || static_v}; x_nbr [n_roots*k, d_x];
 * e_nbr [n_roots*k, d_e]; dt_nbr [n_roots*k] double (time difference of Eq. 5-6); cnt [n_roots] valid
 * neighbours per root (the first cnt of each k).  q = W_q{x_v || Phi(0)} + b_q; K, V from
 * {x_w || e_vw || Phi(dt)}; per head softmax(q K^T / sqrt(cnt)) V; out_z [n_roots, d_o] =
 * ReLU(W_o{h_v || x_v} + b_o).  Activations are kept in the context for tgnn_temporal_attn_bwd, which also reads
 * e_nbr again: it must stay unchanged until then. */
int32_t tgnn_temporal_attn_fwd(tgnn_ctx* ctx, const tgnn_params* p, int32_t n_roots, const float* x_root,
                               const float* x_nbr, const float* e_nbr, const double* dt_nbr,
                               const int32_t* cnt, float* out_z, void* stream);

/* Reverse mode through the most recent tgnn_temporal_attn_fwd on this context (same n_roots, same p).
 * dz [n_roots, d_o].  Adds the gradients of wq,bq,wk,bk,wv,bv,wo,bo,time_w,time_b into `grads` (+=) and
 * writes d_x_root [n_roots, d_m] and d_x_nbr [n_roots*k, d_m]: the gradient with respect to the dynamic
 * (first d_m) columns of x_root / x_nbr.  Static memory and edge features are constants. */
int32_t tgnn_temporal_attn_bwd(tgnn_ctx* ctx, const tgnn_params* p, int32_t n_roots, const float* dz,
                               tgnn_params* grads, float* d_x_root, float* d_x_nbr, void* stream);

/* COMB = most recent mail (Eq. 8, Sec. 2.1.1) and "only root nodes are written" (Sec. 3.2.1).  Occurrence
 * (i, role) with role 0 = source, 1 = destination has key 2i+role; for every distinct node among the 2n
 * endpoints the occurrence with the largest key wins and writes mem = s'_self, mem_ts = tau_self,
 * mail = {s'_self || s'_other}, mail_eid = eid[i], mail_ts = t[i].  s_new_src/dst [n, d_m], tau_src/dst [n].
 * out_winner [2n] (may be NULL): 1 where occurrence role*n+i won, else 0. */
int32_t tgnn_memory_writeback(tgnn_ctx* ctx, tgnn_state* st, int32_t replica, const int32_t* src,
                              const int32_t* dst, const int32_t* eid, const double* t, int32_t n_events,
                              const float* s_new_src, const float* s_new_dst, const double* tau_src,
                              const double* tau_dst, int32_t* out_winner, void* stream);

/* For callers that cannot allocate device memory -- code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc: tgnn_memory_writeback for ONE memory replica without a context.  It allocates nothing
 * (no hipMalloc / hipFree, no allocating library call): the arbitration words live in a static device array of the
 * library, 8 bytes per node, 2 MiB + 1 KiB per GPU, held until the process ends.  `st` describes the replica to write
 * (arrays of n_nodes rows; st->stat is not used); all other arguments, the results and out_winner are as in
 * tgnn_memory_writeback, bit for bit.  Three kernel launches on `stream`, no memset, no synchronisation.
 * TGNN_E_OUT_OF_RANGE: n_nodes > TGNN_NOALLOC_MAX_NODES, n_events > TGNN_NOALLOC_MAX_EVENTS or a device ordinal >= 64.
 * Every call on a GPU shares that GPU's array (it keeps the last call's contents; each call clears the words of its
 * node range first): calls that overlap in time on one GPU, also from different streams or threads, race -- order them. */
int32_t tgnn_memory_writeback_noalloc(int32_t n_nodes, int32_t d_mem, tgnn_state* st, const int32_t* src,
                                      const int32_t* dst, const int32_t* eid, const double* t, int32_t n_events,
                                      const float* s_new_src, const float* s_new_dst, const double* tau_src,
                                      const double* tau_dst, int32_t* out_winner, void* stream);

/* The whole step for n_batches mini-batches (one per memory replica, distinct replicas) that share one
 * weight set: sample -> gather -> UPDT for root and supporting nodes -> attention -> decoder ->
 * loss = mean binary cross-entropy over each batch's n positive and n negative pairs -> backward (the
 * stored memory and mails are constants: no back-propagation through time) -> last-event-wins write-back.
 *   grads      gradients of sum_b loss_b are ADDED (+=) to these tensors (with TGNN_FLAG_OVERWRITE_GRADS in the
 *              configuration they are cleared first, inside the step);
 *   lr         if nonzero, plain SGD p -= lr * grads on every tensor except time_w/time_b after the
 *              backward pass (grads must then hold only this step's gradients, i.e. be zero on entry);
 *   out_loss   device scalar, mean over the batches of loss_b;
 *   out_logits [2 * sum n] or NULL; batch b at offset 2 * (events before b): n positive then n negative;
 *   out_winner [2 * sum n] or NULL; as in tgnn_memory_writeback, per batch.
 * Each batches[b].n <= max_batch, n_batches <= min(n_replicas, TGNN_MAX_BATCHES).
 * Node ids in the batch arrays live on the device and cannot be validated by the host: an id outside [0, n_nodes) is
 * computed as node 0 (no access leaves the arrays), is never written back, and is counted; the running count is item 9
 * of tgnn_debug_read.  Event ids must lie in [0, graph.n_events), and the temporal CSR must be the one
 * tgnn_build_tcsr produces for these n_nodes (not checked). */
int32_t tgnn_train_step(tgnn_ctx* ctx, const tgnn_graph* g, tgnn_state* st, const tgnn_params* p,
                        tgnn_params* grads, const tgnn_batch* batches, int32_t n_batches, float lr,
                        float* out_loss, float* out_logits, int32_t* out_winner, void* stream);

/* Epoch parallelism on one GPU (Sec. 3.2.2): the work of n_neg_sets trainers that train the SAME positive mini-batch
 * with different sampled negative destinations, in one step.  The inputs of the positive roots (memory, mails,
 * neighbours) are fetched, updated (UPDT) and embedded once and shared by all sets; every set adds its n negative roots
 * and its n pairs (src_i, neg_{g,i}); memory and mails are written once (the paper: only the first trainer writes).
 * batches[b].neg holds the sets one after the other, [n_neg_sets, n].  Roots per batch: [src | dst | neg set 0 | ... ].
 *   loss       mean over the sets of each set's loss (1 / 2n) (sum softplus(-logit+) + sum softplus(logit-_g));
 *   grads      gradient of the SUM of the sets' losses (what the trainers' gradient all-reduce would deliver), +=;
 *   out_logits [(1 + n_neg_sets) * sum n] or NULL; per batch: n true pairs, then n pairs per set.
 * n_neg_sets = 1 is tgnn_train_step.  1 <= n_neg_sets <= config.max_neg_sets <= TGNN_MAX_NEG_SETS, else
 * TGNN_E_OUT_OF_RANGE.  The multi-GPU schedule staggers the sets over consecutive iterations (each trainer then sees
 * weights one update newer); running them in one step is the same work at the same shapes with one weight set. */
int32_t tgnn_train_step_epoch_parallel(tgnn_ctx* ctx, const tgnn_graph* g, tgnn_state* st, const tgnn_params* p,
                                       tgnn_params* grads, const tgnn_batch* batches, int32_t n_batches,
                                       int32_t n_neg_sets, float lr, float* out_loss, float* out_logits,
                                       int32_t* out_winner, void* stream);

/* Dynamic edge classification (Sec. 4 "Datasets": the 56-class task with several true classes per event).  The step of
 * tgnn_train_step with another head and no negative destinations: roots per batch are [src | dst] (batches[b].neg is
 * not read), logit_{i,c} = dec_w2[c] . ReLU(W_s z_src_i + W_d z_dst_i + b1) + dec_b2[c] for the C = config.n_classes
 * classes, and the loss is the mean over the events of a batch and the classes of the binary cross-entropy
 * softplus(logit) - y logit, averaged over the batches.  Memory and mails are written back as in tgnn_train_step.
 *   labels     HOST array of n_batches DEVICE pointers; labels[b] is [batches[b].n, C] float, 1 = class is true;
 *   out_logits [sum n, C] or NULL;  out_winner [2 * sum n] or NULL.
 * TGNN_E_INVALID_ARG on a context with n_classes == 0 (and the link-prediction steps refuse one with n_classes > 0). */
int32_t tgnn_train_step_edge_class(tgnn_ctx* ctx, const tgnn_graph* g, tgnn_state* st, const tgnn_params* p,
                                   tgnn_params* grads, const tgnn_batch* batches, int32_t n_batches,
                                   const float* const* labels, float lr, float* out_loss, float* out_logits,
                                   int32_t* out_winner, void* stream);

/* Evaluation pass of temporal link prediction (Sec. 4: the rank of the true destination among itself and 49 sampled
 * negative destinations, mean reciprocal rank reported).  The forward half of tgnn_train_step_epoch_parallel with
 * n_neg_sets negative destinations per event (batches[b].neg is [n_neg_sets, n]), then per event
 * rank = 1 + #(negatives scoring strictly higher than the true destination) + 0.5 #(negatives scoring the same),
 * and the write-back of memory and mails (evaluation events advance the memory like training events).  No gradients, no
 * optimiser step, parameters untouched.
 *   out_logits [(1 + n_neg_sets) * sum n] or NULL, laid out as in tgnn_train_step_epoch_parallel;
 *   out_rank   [sum n] float;   out_rr_sum [1] float: the sum over the events of 1 / rank is ADDED to it;
 *   out_winner [2 * sum n] or NULL.
 * 1 <= n_neg_sets <= config.max_neg_sets. */
int32_t tgnn_eval_step(tgnn_ctx* ctx, const tgnn_graph* g, tgnn_state* st, const tgnn_params* p,
                       const tgnn_batch* batches, int32_t n_batches, int32_t n_neg_sets, float* out_logits,
                       float* out_rank, float* out_rr_sum, int32_t* out_winner, void* stream);

/* Evaluation pass of the edge-classification task (Sec. 4: micro-averaged F1 reported).  The forward half of
 * tgnn_train_step_edge_class, then over all events and classes the counts tp (logit > 0 and label set), fp (logit > 0,
 * label not set) and fn (logit <= 0, label set), and the write-back of memory and mails.  No gradients, no optimiser
 * step.  F1-micro = 2 tp / (2 tp + fp + fn) is left to the caller (counts of several calls add up).
 *   labels      as in tgnn_train_step_edge_class;   out_logits [sum n, C] or NULL;
 *   out_counts  [3] int32: tp, fp, fn are ADDED to it;   out_winner [2 * sum n] or NULL. */
int32_t tgnn_eval_step_edge_class(tgnn_ctx* ctx, const tgnn_graph* g, tgnn_state* st, const tgnn_params* p,
                                  const tgnn_batch* batches, int32_t n_batches, const float* const* labels,
                                  float* out_logits, int32_t* out_counts, int32_t* out_winner, void* stream);

/* Optimiser of the in-step update that tgnn_train_step (and its variants) apply when lr != 0.
 *   kind 0  plain SGD, p -= lr g (the default);
 *   kind 1  Adam: m = beta1 m + (1 - beta1) g, v = beta2 v + (1 - beta2) g^2, p -= lr (m / (1 - beta1^t)) /
 *           (sqrt(v / (1 - beta2^t)) + eps), t = number of Adam steps so far on this context (kept on the device, starts
 *           at 0 with this call).  m, v: moment tensors laid out like the parameters, caller-owned, zero on entry.
 * The time-encoding parameters time_w, time_b stay frozen under both.  The learning rate is the `lr` of every step (the
 * paper scales it linearly with the global batch size, Sec. 4: the caller's choice).  Takes effect from the next step;
 * synchronises the device. */
int32_t tgnn_set_optimizer(tgnn_ctx* ctx, int32_t kind, tgnn_params* m, tgnn_params* v, float beta1, float beta2, float eps);

/* Co-trained static node memory (Sec. 3.1: the static memory as a learnable embedding table trained with the model
 * instead of a frozen pre-trained one).  From the next step on, every training step also back-propagates into the
 * static rows {static_w} of the nodes it touches (roots and supporting nodes):
 *   grad_static [n_nodes, d_static] or NULL: the rows' gradients (of the sum of the batches' losses) are ADDED here;
 *   lr_static: if nonzero, the touched rows of state.stat are updated in the step, stat[w] -= lr_static * g[w] (plain
 *              sparse SGD on the table: no moments are kept for rows, whatever tgnn_set_optimizer selects).
 * state.stat is then written by the library although the struct declares it const.  enable = 0 switches it off.
 * TGNN_E_UNSUPPORTED_DIM when d_static == 0.  Synchronises the device. */
int32_t tgnn_train_static(tgnn_ctx* ctx, int32_t enable, float* grad_static, float lr_static);

/* n_steps consecutive training steps (Sec. 3.2.1: mini-batches are trained in chronological order, each step
 * reading the memory the step before it wrote) in one call: the same sequence of launches, with the same results
 * (up to the order of floating-point sums), as n_steps calls of tgnn_train_step with out_logits = out_winner = NULL.
 * For callers that have the next mini-batches at hand: every run of consecutive steps with the same batch sizes
 * and replicas is one recorded HIP graph and one launch, which saves the idle time between two graph launches
 * (about 8 us each on MI355X).  Steps on which stage timing is due, and all steps on the NULL stream or with
 * TGNN_FLAG_NO_GRAPH or TGNN_FLAG_SIDE_STREAM, are issued one by one.
 *   batches    host array [n_steps * n_batches]: step i uses batches[i * n_batches .. (i + 1) * n_batches);
 *   out_loss   device array [n_steps]: the loss of every step;
 *   grads, lr  as in tgnn_train_step, per step (without TGNN_FLAG_OVERWRITE_GRADS and with lr == 0 the gradients
 *              of all steps add up).
 * 1 <= n_steps <= TGNN_MAX_STEPS_PER_CALL, else TGNN_E_OUT_OF_RANGE; other errors as tgnn_train_step. */
int32_t tgnn_train_steps(tgnn_ctx* ctx, const tgnn_graph* g, tgnn_state* st, const tgnn_params* p,
                         tgnn_params* grads, int32_t n_steps, const tgnn_batch* batches, int32_t n_batches,
                         float lr, float* out_loss, void* stream);

/* Sets every tensor of `g` (a gradient set laid out like the parameters) to zero with one kernel. */
int32_t tgnn_zero_params(tgnn_ctx* ctx, tgnn_params* g, void* stream);

/* Stage timing with HIP events on the call's own stream.  Stages of tgnn_train_step (launches, in step order):
 *  2 first launch: roots + sample + distinct-node rows, and the prologue (pack weights, clear loss/grads, batch
 *    descriptors)   3 state gather + time-encode (GRU input; with the slot -> row map)   4 GRU input and hidden
 *    projections (MFMA, one launch)   6 GRU gates (with the scan of the slot sort)
 *  9 per-node projections K, V, q, merge (MFMA)   8 per-node score vectors U = q W_k^c (MFMA)
 *  10 attention forward: gathers the slots' edge features, time encoding, scores, softmax, weighted sums (with the fill
 *    pass of the slot sort)   7 attention output = node part + Zp (W_v^c)^T (MFMA)
 *  12 root chain: merge layer, decoder + loss and their backward pass down to the gradient of the attention output,
 *    one launch (d_mem a multiple of 4 and <= 128; otherwise 11 merge layer, 12 decoder forward + loss, 13 decoder
 *    backward, and the attention-output gradient GEMM)
 *  19 G = dO W_v^c per root (MFMA)   14 attention backward   5 dq = node part + Zs (W_k^c)^T (MFMA)
 *  15 per-node gradient sums (with the gradients through the query's Phi(0)) + node projections backward with GRU
 *    gates backward
 *  16 all weight gradients and the time-encoding gradients of the keys (one grouped MFMA GEMM)   17 time-encoding
 *    gradient of the mails (GEMM with the reduction in its epilogue) + write-back scatter + SGD, one launch
 *  18 nothing (two event records back to back: the cost of a bracket by itself)   0, 1 unused
 * tgnn_profile_enable: time the stages whose bit is set in `stage_mask` in every following tgnn_train_step
 * (0 = off); each timed stage costs two event records per step.  At most 4096 steps are kept per stage;
 * enabling resets the record.  tgnn_profile_read: synchronises the recorded events and returns the number
 * of recorded launches of `stage` and their total duration in milliseconds.  HOST pointers.
 * tgnn_profile_every: with a non-zero mask, only every `n`-th tgnn_train_step (the first one after this call,
 * then every n-th; n >= 1, default 1) is timed; the steps between run as if the mask were zero, i.e. they may
 * replay the captured graph.  Keeps the mask and the record. */
#define TGNN_N_STAGES 20
int32_t tgnn_profile_enable(tgnn_ctx* ctx, uint32_t stage_mask);
int32_t tgnn_profile_every(tgnn_ctx* ctx, int32_t n);
int32_t tgnn_profile_read(tgnn_ctx* ctx, int32_t stage, int32_t* out_count, double* out_total_ms);

/* A plain streaming copy kernel (dst[i] = src[i], 16-byte words; n_bytes % 16 == 0; buffers must not overlap).
 * It moves a known number of bytes, which calibrates hardware HBM-traffic counters. */
int32_t tgnn_debug_copy(void* dst, const void* src, int64_t n_bytes, void* stream);

/* Debug/parity access to what the last tgnn_train_step left in the workspace.  `what`:
 * 0 nbr [R,k] i32, 1 eid [R,k] i32, 2 nts [R,k] f64, 3 cnt [R] i32, 4 s_new [R(1+k), d_m] f32,
 * 5 tau [R(1+k)] f64, 6 z [R, d_o] f32, 7 decoder hidden layer [2 sum n, d_o] f32, 8 the number of distinct
 * (replica, node) rows of the step [1] i32, 9 the number of batch node ids outside [0, n_nodes) seen by all training
 * steps of the context so far [1] i32.  Copies n_bytes (device to device) into dst on `stream`. */
int32_t tgnn_debug_read(tgnn_ctx* ctx, int32_t what, void* dst, int64_t n_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif
