// Device side of the last-event-wins write-back (see k_writeback.hip) and of the SGD update, callable from any
// kernel with blocks of 256 threads: block b < wb_blocks scatters four occurrences, the blocks after that update
// the parameters (64 blocks per tensor).
#pragma once
#include "tgnn_internal.h"
#include "device_math.h"

namespace tgnn {

__device__ __forceinline__ bool occ_decode(const BatchSet& bs, int o, int& b, int& i, int& role) {
  if (o >= 2 * bs.total) return false;
  b = 0;
  while (b + 1 < bs.nb && o >= 2 * bs.b[b + 1].ev_off) ++b;
  const int local = o - 2 * bs.b[b].ev_off;
  role = local >= bs.b[b].n ? 1 : 0;
  i = local - role * bs.b[b].n;
  return true;
}

template <int VEC>
__device__ __forceinline__ void wb_scatter_block(const WbArgs& a, int block) {
  const BatchSet& bs = *a.bs;
  const WbPtrs& w = a.w;
  const int lane = threadIdx.x & 63;
  int b, i, role;
  const int o = block * 4 + (threadIdx.x >> 6);
  if (!occ_decode(bs, o, b, i, role)) return;
  const BatchDesc& bd = bs.b[b];
  const int node = role ? bd.dst[i] : bd.src[i];
  const bool in_range = node >= 0 && node < a.N;   // an id outside the node range is never written
  const size_t gid = (size_t)bd.replica * a.N + (in_range ? node : 0);
  const bool win = in_range && a.winkey[gid] == wb_key(*a.epoch, bd.ev_off + i, role);
  if (lane == 0 && a.out_winner) a.out_winner[o] = win ? 1 : 0;
  if (!win) return;
  const float *self_row, *other_row;
  double tau;
  if (w.s_new) {  // fused layout: rows indexed by root slot [src | dst | neg] of the batch
    size_t rs = (size_t)((2 + bs.nneg) * bd.ev_off + i), rd = rs + (size_t)bd.n;
    if (w.slot_row) { rs = (size_t)w.slot_row[rs]; rd = (size_t)w.slot_row[rd]; }
    self_row = w.s_new + (role ? rd : rs) * w.p_s;
    other_row = w.s_new + (role ? rs : rd) * w.p_s;
    tau = w.tau[role ? rd : rs];
  } else {
    self_row = (role ? w.s_dst : w.s_src) + (size_t)i * w.p_s;
    other_row = (role ? w.s_src : w.s_dst) + (size_t)i * w.p_s;
    tau = role ? w.tau_dst[i] : w.tau_src[i];
  }
  const int dm = a.dm;
  wave_copy<VEC>(w.mem + gid * dm, self_row, dm, 0, lane);
  wave_copy<VEC>(w.mail + gid * 2 * dm, self_row, dm, 0, lane);
  wave_copy<VEC>(w.mail + gid * 2 * dm + dm, other_row, dm, 0, lane);
  if (lane == 0) {
    w.mem_ts[gid] = tau;
    w.mail_ts[gid] = bd.t[i];
    w.mail_eid[gid] = bd.eid[i];
  }
}

// Co-trained static memory (Sec. 3.1): row r of the step's distinct node rows carries the gradient of the static row of
// node ulist[r] % N.  Rows of different memory replicas may be the same node, so the table is updated with atomics.
__device__ __forceinline__ void stat_update_block(const StatUpd& u, int block) {
  const int rows = *u.ucount;
  const long long total = (long long)rows * u.ds;
  for (long long i = block * 256LL + threadIdx.x; i < total; i += (long long)u.blocks * 256) {
    const int r = (int)(i / u.ds), c = (int)(i - (long long)r * u.ds);
    const float g = u.drow[(size_t)r * u.ld + c];
    const size_t o = (size_t)(u.ulist[r] % u.N) * u.ds + c;
    if (u.gstat != nullptr) atomicAdd(u.gstat + o, g);
    if (u.lr != 0.f) atomicAdd(u.stat + o, -u.lr * g);
  }
}

// block: 0 .. wb_total_blocks(a) - 1
__device__ __forceinline__ void wb_sgd_block(const WbArgs& a, int block) {
  if (block >= a.wb_blocks) {
    const int extra = block - a.wb_blocks;
    const int n_sgd = a.sgd != nullptr ? 64 * a.sgd_cnt : 0;
    if (extra >= n_sgd) {
      if (a.stat.drow != nullptr && extra - n_sgd < a.stat.blocks) stat_update_block(a.stat, extra - n_sgd);
      return;
    }
    const int t = extra >> 6, x = extra & 63;
    float* p = a.sgd->p[t];
    const float* g = a.sgd->g[t];
    const int n = a.sgd->n[t];
    if (a.adam != nullptr) {   // Adam with bias correction; the step count and the corrections in double
      const AdamSet& ad = *a.adam;
      float* m = ad.m[t];
      float* v = ad.v[t];
      const double steps = (double)*ad.t;
      const float c1 = (float)(1.0 / (1.0 - pow((double)ad.beta1, steps)));
      const float c2 = (float)(1.0 / (1.0 - pow((double)ad.beta2, steps)));
      for (int i = x * 256 + threadIdx.x; i < n; i += 64 * 256) {
        const float gi = g[i];
        const float mi = ad.beta1 * m[i] + (1.0f - ad.beta1) * gi;
        const float vi = ad.beta2 * v[i] + (1.0f - ad.beta2) * gi * gi;
        m[i] = mi;
        v[i] = vi;
        p[i] -= a.lr * (mi * c1) / (sqrtf(vi * c2) + ad.eps);
      }
      return;
    }
    for (int i = x * 256 + threadIdx.x; i < n; i += 64 * 256) p[i] -= a.lr * g[i];
    return;
  }
  if (a.vec == 4) wb_scatter_block<4>(a, block);
  else wb_scatter_block<1>(a, block);
}

}  // namespace tgnn
