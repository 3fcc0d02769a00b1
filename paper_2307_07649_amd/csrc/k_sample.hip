// Root construction and most-recent-neighbour sampling (Sec. 2.1 "most recent neighbors"; k = 10 in Sec. 4)
// on the temporal CSR: one wavefront per query, a 64-ary search over the node's ascending time array
// followed by one k-wide read of the newest entries below the query time.
#include "tgnn_internal.h"

namespace tgnn {

// FUSED: the query of wave r is root r of the step's batches ([src | dst | neg] per batch); the wave also
// records the root (node, time, slot ids), marks the write-back arbitration word of a positive endpoint
// (last-event-wins: largest key survives) and claims rows for the root and its neighbours.
// Otherwise the queries are the caller's (node, t) arrays.
template <bool FUSED>
__global__ __launch_bounds__(1024) void sample_kernel(const int64_t* __restrict__ indptr,
                                                      const int32_t* __restrict__ g_nbr,
                                                      const int32_t* __restrict__ g_eid,
                                                      const double* __restrict__ g_ts, int N,
                                                      const int32_t* __restrict__ q_node,
                                                      const double* __restrict__ q_t, int n_roots, int k,
                                                      int32_t* __restrict__ out_nbr, int32_t* __restrict__ out_eid,
                                                      double* __restrict__ out_ts, int32_t* __restrict__ out_cnt,
                                                      const BatchSet* __restrict__ bsp, int32_t* __restrict__ root_node,
                                                      double* __restrict__ root_t, int32_t* __restrict__ slot_gid,
                                                      int32_t* __restrict__ slot_node, unsigned long long* winkey,
                                                      UniqPtrs uq) {
  __shared__ int blk_count, blk_base;
  const int lane = threadIdx.x & 63;
  const int r = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  const bool active = r < n_roots;   // per wave; in the fused form idle waves still join the block barriers
  if (!FUSED && !active) return;
  if (FUSED) {
    if (threadIdx.x == 0) blk_count = 0;
    __syncthreads();
  }
  int claim = -1;   // (replica, node) this lane wants a row for
  unsigned long long ep = 0ull;
  if (active) {
    int node, rep_base = 0, root_gid = -1;
    double t;
    if (FUSED) {
      const BatchSet& bs = *bsp;
      int b = 0;
      while (b + 1 < bs.nb && r >= 3 * bs.b[b + 1].ev_off) ++b;
      const BatchDesc bd = bs.b[b];
      const int local = r - 3 * bd.ev_off;
      const int role = local / bd.n, i = local - role * bd.n;
      node = (role == 0 ? bd.src : role == 1 ? bd.dst : bd.neg)[i];
      t = bd.t[i];
      rep_base = bd.replica * N;
      ep = *uq.epoch;
      root_gid = rep_base + node;
      if (lane == 0) {
        root_node[r] = node;
        root_t[r] = t;
        slot_gid[r] = root_gid;
        slot_node[r] = node;
        if (role < 2) atomicMax(winkey + root_gid, wb_key(ep, bd.ev_off + i, role));
      }
    } else {
      node = q_node[r];
      t = q_t[r];
    }
    long long base = 0, lo = 0, hi = 0;
    if (node >= 0 && node < N) {
      base = indptr[node];
      lo = base;
      hi = indptr[node + 1];
    }
    // invariant: entries before lo are < t; entry hi (if inside the list) is >= t; answer in [lo, hi]
    while (hi - lo > 64) {
      const long long step = (hi - lo + 63) / 64;
      const long long idx = lo + (long long)(lane + 1) * step - 1;
      const bool below = idx < hi && g_ts[idx] < t;
      const int nb = __popcll(__ballot(below));
      const long long nlo = lo + (long long)nb * step;
      const long long nhi = lo + (long long)(nb + 1) * step - 1;
      lo = nlo;
      hi = nhi < hi ? nhi : hi;
    }
    {
      const long long idx = lo + lane;
      const bool below = idx < hi && g_ts[idx] < t;
      lo += __popcll(__ballot(below));
    }
    const long long pos = lo;  // first entry with time >= t
    const long long avail = pos - base;
    const int cnt = avail < k ? (int)avail : k;
    if (lane == 0) out_cnt[r] = cnt;
    int nb = -1, ei = -1;
    double ts = 0.0;
    if (lane < cnt) {
      const long long idx = pos - 1 - lane;
      nb = g_nbr[idx];
      ei = g_eid[idx];
      ts = g_ts[idx];
    }
    if (lane < k) {
      const size_t o = (size_t)r * k + lane;
      out_nbr[o] = nb;
      out_eid[o] = ei;
      out_ts[o] = ts;
      if (FUSED) {
        slot_gid[(size_t)n_roots + o] = nb >= 0 ? rep_base + nb : -1;
        slot_node[(size_t)n_roots + o] = nb;
      }
    }
    // lanes 0 .. k-1 claim their neighbour, lane k (k < 64) the root itself
    if (FUSED) claim = lane < k ? (nb >= 0 ? rep_base + nb : -1) : (lane == k ? root_gid : -1);
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

constexpr int SAMPLE_WAVES = 16;   // roots per block

void sample_roots(tgnn_ctx* ctx, const tgnn_graph* g, int n_roots, hipStream_t s) {
  if (n_roots <= 0) return;
  const Dims& d = ctx->d;
  Ws& w = ctx->w;
  UniqPtrs uq{w.utag, w.epoch, w.uidx, w.ucount, w.ulist, w.ucnt};
  hipLaunchKernelGGL(sample_kernel<true>, dim3((n_roots + SAMPLE_WAVES - 1) / SAMPLE_WAVES), dim3(64 * SAMPLE_WAVES), 0, s, g->indptr, g->nbr, g->eid, g->ts, d.N,
                     nullptr, nullptr, n_roots, d.k, w.nbr, w.neid, w.nts, w.cnt, w.bs_dev, w.root_node, w.root_t,
                     w.slot_gid, w.slot_node, w.winkey, uq);
}

void sample_recent(const Dims& d, const tgnn_graph* g, const int32_t* node, const double* t, int n_roots,
                   int32_t* out_nbr, int32_t* out_eid, double* out_ts, int32_t* out_cnt, hipStream_t s) {
  if (n_roots <= 0) return;
  UniqPtrs uq{};
  hipLaunchKernelGGL(sample_kernel<false>, dim3((n_roots + 3) / 4), dim3(256), 0, s, g->indptr, g->nbr, g->eid, g->ts, d.N,
                     node, t, n_roots, d.k, out_nbr, out_eid, out_ts, out_cnt, nullptr, nullptr, nullptr, nullptr, nullptr,
                     nullptr, uq);
}

}  // namespace tgnn
