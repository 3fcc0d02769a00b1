// Root construction and most-recent-neighbour sampling (Sec. 2.1 "most recent neighbors"; k = 10 in Sec. 4)
// on the temporal CSR: one wavefront per query, a 64-ary search over the node's ascending time array
// followed by one k-wide read of the newest entries below the query time.
#include "tgnn_internal.h"

namespace tgnn {

__global__ void roots_kernel(const BatchSet* __restrict__ bsp, int N, int32_t* root_node, int32_t* root_gid,
                             int32_t* root_batch, double* root_t, int32_t* slot_gid, int32_t* slot_node,
                             unsigned long long* winkey, const unsigned long long* __restrict__ epoch,
                             unsigned long long* utag, int32_t* uidx, int32_t* ucount, int32_t* ulist, int32_t* ucnt) {
  const BatchSet& bs = *bsp;
  const int e = blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= bs.total) return;
  int b = 0;
  while (b + 1 < bs.nb && e >= bs.b[b + 1].ev_off) ++b;
  const BatchDesc bd = bs.b[b];
  const int i = e - bd.ev_off;
  const double t = bd.t[i];
  const int nodes[3] = {bd.src[i], bd.dst[i], bd.neg[i]};
  const unsigned long long ep = *epoch;
#pragma unroll
  for (int role = 0; role < 3; ++role) {
    const int r = 3 * bd.ev_off + role * bd.n + i;
    const int gid = bd.replica * N + nodes[role];
    root_node[r] = nodes[role];
    root_gid[r] = gid;
    root_batch[r] = b;
    root_t[r] = t;
    slot_gid[r] = gid;
    slot_node[r] = nodes[role];
    if (role < 2) atomicMax(winkey + gid, wb_key(ep, e, role));   // last-event-wins arbitration
    uniq_claim(utag, uidx, ucount, ulist, ucnt, gid, ep);
  }
}

void build_roots(tgnn_ctx* ctx, int total, hipStream_t s) {
  Ws& w = ctx->w;
  hipLaunchKernelGGL(roots_kernel, dim3((total + 255) / 256), dim3(256), 0, s, w.bs_dev, ctx->d.N, w.root_node,
                     w.root_gid, w.root_batch, w.root_t, w.slot_gid, w.slot_node, w.winkey, w.epoch, w.utag, w.uidx,
                     w.ucount, w.ulist, w.ucnt);
}

// gid = replica * N + node for roots of the fused step (root_gid given), plain node ids otherwise.
__global__ __launch_bounds__(256) void sample_kernel(const int64_t* __restrict__ indptr,
                                                     const int32_t* __restrict__ g_nbr,
                                                     const int32_t* __restrict__ g_eid,
                                                     const double* __restrict__ g_ts, int N,
                                                     const int32_t* __restrict__ q_node,
                                                     const double* __restrict__ q_t,
                                                     const int32_t* __restrict__ root_gid, int n_roots, int k,
                                                     int32_t* __restrict__ out_nbr, int32_t* __restrict__ out_eid,
                                                     double* __restrict__ out_ts, int32_t* __restrict__ out_cnt,
                                                     int32_t* __restrict__ slot_gid, int32_t* __restrict__ slot_node,
                                                     UniqPtrs uq) {
  const int lane = threadIdx.x & 63;
  const int r = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (r >= n_roots) return;  // whole wave leaves together
  const int node = q_node[r];
  const double t = q_t[r];
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
  if (lane < k) {
    int nb = -1, ei = -1;
    double ts = 0.0;
    if (lane < cnt) {
      const long long idx = pos - 1 - lane;
      nb = g_nbr[idx];
      ei = g_eid[idx];
      ts = g_ts[idx];
    }
    const size_t o = (size_t)r * k + lane;
    out_nbr[o] = nb;
    out_eid[o] = ei;
    out_ts[o] = ts;
    if (slot_gid != nullptr) {
      const int rep_base = root_gid[r] - node;
      slot_gid[(size_t)n_roots + o] = nb >= 0 ? rep_base + nb : -1;
      slot_node[(size_t)n_roots + o] = nb;
      if (nb >= 0 && uq.utag != nullptr)
        uniq_claim(uq.utag, uq.uidx, uq.ucount, uq.ulist, uq.ucnt, rep_base + nb, *uq.epoch);
    }
  }
}

void sample_recent(const Dims& d, const tgnn_graph* g, const int32_t* node, const double* t, const int32_t* root_gid,
                   int n_roots, int32_t* out_nbr, int32_t* out_eid, double* out_ts, int32_t* out_cnt,
                   int32_t* slot_gid, int32_t* slot_node, const UniqPtrs* uq, hipStream_t s) {
  if (n_roots <= 0) return;
  UniqPtrs u{};
  if (uq) u = *uq;
  hipLaunchKernelGGL(sample_kernel, dim3((n_roots + 3) / 4), dim3(256), 0, s, g->indptr, g->nbr, g->eid, g->ts, d.N,
                     node, t, root_gid, n_roots, d.k, out_nbr, out_eid, out_ts, out_cnt, slot_gid, slot_node, u);
}

}  // namespace tgnn
