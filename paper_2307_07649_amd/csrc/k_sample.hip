// Root construction and most-recent-neighbour sampling (Sec. 2.1 "most recent neighbors"; k = 10 in Sec. 4)
// on the temporal CSR: a group of 64 or 16 lanes per query, a search over the node's ascending time array with as
// many probes per level as the group has lanes, followed by one k-wide read of the newest entries below the query
// time.
#include <string.h>

#include "tgnn_internal.h"
#include "prologue_device.h"

namespace tgnn {

// FUSED: the query of lane group r is root r of the step's batches ([src | dst | neg] per batch); the group also
// records the root (node, time, slot ids), marks the write-back arbitration word of a positive endpoint
// (last-event-wins: largest key survives) and claims rows for the root and its neighbours.  `bs` are the batch
// descriptors (read from the kernel's argument block), `ep` the epoch of the step.
// Otherwise the queries are the caller's (node, t) arrays.
// `block` is the calling block's number among the sampling blocks.
// G lanes per query (64 or 16): a query is a chain of eight to ten dependent memory round trips (batch arrays,
// list bounds, G-ary search, the k newest entries, row claim) during which most lanes have nothing to do, and a
// compute unit holds at most 32 wavefronts: with a wavefront per query a 12,000-root step needs one and a half
// rounds of them.  Four queries per wavefront (G = 16, k < 16) put all roots of such a step in flight at once; the
// search takes one level more on lists of a few thousand entries.
template <bool FUSED, int G>
__device__ __forceinline__ void sample_block(const SampleArgs& a, const BatchSet& bs, unsigned long long ep, int block) {
  __shared__ int blk_count, blk_base;
  constexpr int QW = 64 / G;   // queries per wavefront
  const UniqPtrs& uq = a.uq;
  const int N = a.N, n_roots = a.n_roots, k = a.k;
  const int lane = threadIdx.x & 63;
  const int grp = lane / G, gl = lane - grp * G;        // lane group and lane in it
  const unsigned long long gmask = G == 64 ? ~0ull : ((1ull << (G & 63)) - 1ull) << (grp * G);
  const int r = (block * (blockDim.x >> 6) + (int)(threadIdx.x >> 6)) * QW + grp;
  const bool active = r < n_roots;   // per group; in the fused form idle groups still join the block barriers
  if (!FUSED && G == 64 && !active) return;
  if (FUSED) {
    if (threadIdx.x == 0) blk_count = 0;
    __syncthreads();
  }
  int claim = -1;   // (replica, node) this lane wants a row for
  {
    int node = -1, rep_base = 0, root_gid = -1;
    double t = 0.0;
    if (active) {
      if (FUSED) {
        int b = 0;
        const int n_roles = 2 + bs.nneg;
        while (b + 1 < bs.nb && r >= n_roles * bs.b[b + 1].ev_off) ++b;
        const int ev_off = bs.b[b].ev_off, n = bs.b[b].n;
        const int local = r - n_roles * ev_off;
        const int role = local / n, i = local - role * n;
        const int32_t* nodes = role == 0 ? bs.b[b].src : role == 1 ? bs.b[b].dst : bs.b[b].neg + (size_t)(role - 2) * n;
        node = nodes[i];
        t = bs.b[b].t[i];
        // an id outside [0, N) in the caller's batch arrays: the root is computed as node 0 (every index stays in
        // range), takes no part in the write-back, and is counted for the caller to see
        const bool bad = node < 0 || node >= N;
        if (bad) node = 0;
        rep_base = bs.b[b].replica * N;
        root_gid = rep_base + node;
        if (gl == 0) {
          a.root_node[r] = node;
          a.root_t[r] = t;
          a.slot_gid[r] = root_gid;
          a.slot_node[r] = node;
          if (bad) atomicAdd(a.bad_ids, 1);
          else if (role < 2) atomicMax(a.winkey + root_gid, wb_key(ep, ev_off + i, role));
        }
      } else {
        node = a.q_node[r];
        t = a.q_t[r];
      }
    }
    long long base = 0, lo = 0, hi = 0;
    if (active && node >= 0 && node < N) {
      base = a.indptr[node];
      lo = base;
      hi = a.indptr[node + 1];
    }
    // invariant: entries before lo are < t; entry hi (if inside the list) is >= t; answer in [lo, hi]
    // (the loop runs while any group of the wavefront still has more than G candidates; a group that is done idles)
    while (__any(hi - lo > G)) {
      const bool more = hi - lo > G;
      const long long step = (hi - lo + G - 1) / G;
      const long long idx = lo + (long long)(gl + 1) * step - 1;
      const bool below = more && idx < hi && a.g_ts[idx] < t;
      const int nb = __popcll(__ballot(below) & gmask);
      if (more) {
        const long long nlo = lo + (long long)nb * step;
        const long long nhi = lo + (long long)(nb + 1) * step - 1;
        lo = nlo;
        hi = nhi < hi ? nhi : hi;
      }
    }
    {
      const long long idx = lo + gl;
      const bool below = idx < hi && a.g_ts[idx] < t;
      lo += __popcll(__ballot(below) & gmask);
    }
    const long long pos = lo;  // first entry with time >= t
    const long long avail = pos - base;
    const int cnt = avail < k ? (int)avail : k;
    if (active && gl == 0) a.out_cnt[r] = cnt;
    int nb = -1, ei = -1;
    double ts = 0.0;
    if (active && gl < cnt) {
      const long long idx = pos - 1 - gl;
      nb = a.g_nbr[idx];
      ei = a.g_eid[idx];
      ts = a.g_ts[idx];
    }
    if (active && gl < k) {
      const size_t o = (size_t)r * k + gl;
      a.out_nbr[o] = nb;
      a.out_eid[o] = ei;
      a.out_ts[o] = ts;
      if (FUSED) {
        a.slot_gid[(size_t)n_roots + o] = nb >= 0 ? rep_base + nb : -1;
        a.slot_node[(size_t)n_roots + o] = nb;
      }
    }
    // lanes 0 .. k-1 of the group claim their neighbour, lane k (k < G) the root itself
    if (FUSED && active) claim = gl < k ? (nb >= 0 ? rep_base + nb : -1) : (gl == k ? root_gid : -1);
  }
  if (FUSED) {
    // Row numbers for the nodes claimed first by this block: winners are counted per wave (ballot), per block
    // (LDS) and only then on the device-wide row counter, whose atomics serialise in the L2.
    bool won = false;
    if (claim >= 0 && __atomic_load_n(uq.utag + claim, __ATOMIC_RELAXED) < ep)   // popular nodes: look first
      won = atomicMax(uq.utag + claim, ep) < ep;
    const unsigned long long winners = __ballot(won);
    int wave_base = 0;
    if (winners != 0ull && lane == 0) wave_base = atomicAdd(&blk_count, __popcll(winners));
    __syncthreads();
    if (threadIdx.x == 0) blk_base = blk_count > 0 ? atomicAdd(uq.ucount, blk_count) : 0;
    __syncthreads();
    wave_base = __shfl(wave_base, 0);   // all lanes take part: lane 0 need not be a winner itself
    if (won) {
      const int row = blk_base + wave_base + __popcll(winners & ((1ull << lane) - 1ull));
      uq.uidx[claim] = row;
      uq.ulist[row] = claim;
      uq.ucnt[row] = 0;
    }
  }
}

// plain sampling of the caller's queries
__global__ __launch_bounds__(256) void sample_kernel(SampleArgs a, BatchSet none) { sample_block<false, 64>(a, none, 0ull, blockIdx.x); }

// The first launch of a training step: sampling blocks, then the prologue's blocks (see HeadArgs).
__global__ __launch_bounds__(64 * SAMPLE_WAVES) void step_head_kernel(HeadArgs h) {
  if ((int)blockIdx.x < h.sample_blocks) {
    // the epoch counter still holds the previous step's value: nothing writes it during this launch
    if (h.sa.k < 16) sample_block<true, 16>(h.sa, h.pa.bs, *h.sa.uq.epoch + 1ull, blockIdx.x);
    else sample_block<true, 64>(h.sa, h.pa.bs, *h.sa.uq.epoch + 1ull, blockIdx.x);
    return;
  }
  const int pb = blockIdx.x - h.sample_blocks;
  const int y = pb / h.pro_bx;
  prologue_block(h.pa, pb - y * h.pro_bx, h.pro_bx, y);
}

static SampleArgs sample_args(const Dims& d, const tgnn_graph* g, int n_roots) {
  SampleArgs a;
  memset(&a, 0, sizeof(a));
  a.indptr = g->indptr; a.g_nbr = g->nbr; a.g_eid = g->eid; a.g_ts = g->ts;
  a.N = d.N; a.n_roots = n_roots; a.k = d.k;
  return a;
}

void head_fill(tgnn_ctx* ctx, const tgnn_graph* g, int n_roots, const tgnn_params* p, const BatchSet* bs,
               const SgdSet* sgd, const SgdSet* zero, float* loss, HeadArgs& h) {
  const Dims& d = ctx->d;
  Ws& w = ctx->w;
  h.sa = sample_args(d, g, n_roots);
  h.sa.out_nbr = w.nbr; h.sa.out_eid = w.neid; h.sa.out_ts = w.nts; h.sa.out_cnt = w.cnt;
  h.sa.root_node = w.root_node; h.sa.root_t = w.root_t; h.sa.slot_gid = w.slot_gid; h.sa.slot_node = w.slot_node;
  h.sa.winkey = w.winkey; h.sa.bad_ids = w.bad_ids;
  h.sa.uq = UniqPtrs{w.utag, w.epoch, w.uidx, w.ucount, w.ulist, w.ucnt};
  const int per_block = SAMPLE_WAVES * (d.k < 16 ? 4 : 1);   // four roots per wavefront when a lane group of 16 holds k + 1 claims
  h.sample_blocks = (n_roots + per_block - 1) / per_block;
  h.pro_bx = 12 * 16 / SAMPLE_WAVES;   // blocks of 1024 threads per grid row of the prologue (C1: 12 measured best of 2 .. 48; 24: +1.6 us per step)
  prologue_fill(ctx, p, bs, sgd, zero, loss, h.pa);
  h.pa.head_of_step = 1;
  h.pa.ucount_next = w.ucount_pair + (w.ucount == w.ucount_pair ? 1 : 0);
}

dim3 head_grid(const HeadArgs& h) { return dim3(h.sample_blocks + h.pro_bx * (h.pa.n_pack + h.pa.zero.cnt + 1)); }
void* head_func() { return reinterpret_cast<void*>(step_head_kernel); }

void step_head(const HeadArgs& h, hipStream_t s) {
  hipLaunchKernelGGL(step_head_kernel, head_grid(h), dim3(64 * SAMPLE_WAVES), 0, s, h);
}

void sample_recent(const Dims& d, const tgnn_graph* g, const int32_t* node, const double* t, int n_roots,
                   int32_t* out_nbr, int32_t* out_eid, double* out_ts, int32_t* out_cnt, hipStream_t s) {
  if (n_roots <= 0) return;
  SampleArgs a = sample_args(d, g, n_roots);
  a.q_node = node; a.q_t = t;
  a.out_nbr = out_nbr; a.out_eid = out_eid; a.out_ts = out_ts; a.out_cnt = out_cnt;
  BatchSet none;
  memset(&none, 0, sizeof(none));
  hipLaunchKernelGGL(sample_kernel, dim3((n_roots + 3) / 4), dim3(256), 0, s, a, none);
}

}  // namespace tgnn
