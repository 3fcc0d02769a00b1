// Last-event-wins write-back: COMB keeps the most recent mail of a batch (Eq. 8, Sec. 2.1.1) and only
// root nodes are written (Sec. 3.2.1).  Arbitration is a segmented maximum over occurrence keys, taken
// with a 64-bit atomic max on a per-(replica, node) scratch word; maximum is order-independent, so the
// winners are deterministic.  Occurrence (event e = off + i, role) has key 1 + 2e + role, prefixed by a
// per-step epoch counter so that the words never need clearing: entries of earlier steps always lose.
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

__global__ void wb_mark_kernel(const BatchSet* __restrict__ bsp, int N, unsigned long long* winkey,
                               const unsigned long long* __restrict__ epoch) {
  const BatchSet& bs = *bsp;
  int b, i, role;
  if (!occ_decode(bs, blockIdx.x * blockDim.x + threadIdx.x, b, i, role)) return;
  const BatchDesc& bd = bs.b[b];
  const int node = role ? bd.dst[i] : bd.src[i];
  atomicMax(winkey + (size_t)bd.replica * N + node, wb_key(*epoch, bd.ev_off + i, role));
}

void writeback_mark(const Dims& d, const BatchSet* bs, int total, unsigned long long* winkey,
                    const unsigned long long* epoch, hipStream_t s) {
  if (total <= 0) return;
  hipLaunchKernelGGL(wb_mark_kernel, dim3((2 * total + 255) / 256), dim3(256), 0, s, bs, d.N, winkey, epoch);
}

struct WbPtrs {
  float *mem, *mail;
  double *mem_ts, *mail_ts;
  int32_t* mail_eid;
  const float *s_new, *s_src, *s_dst;
  const double *tau, *tau_src, *tau_dst;
  const int32_t* slot_row;
  int p_s;
};

template <int VEC>
__global__ __launch_bounds__(256) void wb_scatter_kernel(const BatchSet* __restrict__ bsp, int N, int dm, WbPtrs w,
                                                         const unsigned long long* __restrict__ winkey,
                                                         const unsigned long long* __restrict__ epoch,
                                                         int32_t* __restrict__ out_winner, int wb_blocks,
                                                         const SgdSet* __restrict__ sgd, float lr) {
  if ((int)blockIdx.x >= wb_blocks) {
    // The SGD update of the step shares the launch (it touches parameters and gradients only): 64 blocks per
    // tensor, p -= lr * g.
    const int extra = blockIdx.x - wb_blocks;
    const int t = extra >> 6, x = extra & 63;
    float* p = sgd->p[t];
    const float* g = sgd->g[t];
    const int n = sgd->n[t];
    for (int i = x * 256 + threadIdx.x; i < n; i += 64 * 256) p[i] -= lr * g[i];
    return;
  }
  const BatchSet& bs = *bsp;
  const int lane = threadIdx.x & 63;
  int b, i, role;
  const int o = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (!occ_decode(bs, o, b, i, role)) return;
  const BatchDesc& bd = bs.b[b];
  const int node = role ? bd.dst[i] : bd.src[i];
  const size_t gid = (size_t)bd.replica * N + node;
  const bool win = winkey[gid] == wb_key(*epoch, bd.ev_off + i, role);
  if (lane == 0 && out_winner) out_winner[o] = win ? 1 : 0;
  if (!win) return;
  const float *self_row, *other_row;
  double tau;
  if (w.s_new) {  // fused layout: rows indexed by root slot [src | dst | neg] of the batch
    size_t rs = (size_t)(3 * bd.ev_off + i), rd = (size_t)(3 * bd.ev_off + bd.n + i);
    if (w.slot_row) { rs = (size_t)w.slot_row[rs]; rd = (size_t)w.slot_row[rd]; }
    self_row = w.s_new + (role ? rd : rs) * w.p_s;
    other_row = w.s_new + (role ? rs : rd) * w.p_s;
    tau = w.tau[role ? rd : rs];
  } else {
    self_row = (role ? w.s_dst : w.s_src) + (size_t)i * w.p_s;
    other_row = (role ? w.s_src : w.s_dst) + (size_t)i * w.p_s;
    tau = role ? w.tau_dst[i] : w.tau_src[i];
  }
  wave_copy<VEC>(w.mem + gid * dm, self_row, dm, 0, lane);
  wave_copy<VEC>(w.mail + gid * 2 * dm, self_row, dm, 0, lane);
  wave_copy<VEC>(w.mail + gid * 2 * dm + dm, other_row, dm, 0, lane);
  if (lane == 0) {
    w.mem_ts[gid] = tau;
    w.mail_ts[gid] = bd.t[i];
    w.mail_eid[gid] = bd.eid[i];
  }
}

void writeback_scatter(const Dims& d, const BatchSet* bs, int total, const tgnn_state* st,
                       const unsigned long long* winkey, const unsigned long long* epoch, const float* s_new, int p_s,
                       const double* tau, const int32_t* slot_row, const float* s_src, const float* s_dst,
                       const double* tau_src, const double* tau_dst, int32_t* out_winner, hipStream_t s,
                       const SgdSet* sgd_dev, int sgd_cnt, float lr) {
  if (total <= 0) {
    if (sgd_dev != nullptr && sgd_cnt > 0) sgd_update(sgd_dev, sgd_cnt, lr, s);
    return;
  }
  WbPtrs w{st->mem, st->mail, st->mem_ts, st->mail_ts, st->mail_eid, s_new, s_src, s_dst, tau, tau_src, tau_dst,
           slot_row, p_s};
  const int blocks = (2 * total + 3) / 4;
  const int grid = blocks + (sgd_dev != nullptr ? 64 * sgd_cnt : 0);
  if (d.dm % 4 == 0 && p_s % 4 == 0)
    hipLaunchKernelGGL(wb_scatter_kernel<4>, dim3(grid), dim3(256), 0, s, bs, d.N, d.dm, w, winkey, epoch, out_winner,
                       blocks, sgd_dev, lr);
  else
    hipLaunchKernelGGL(wb_scatter_kernel<1>, dim3(grid), dim3(256), 0, s, bs, d.N, d.dm, w, winkey, epoch, out_winner,
                       blocks, sgd_dev, lr);
}

}  // namespace tgnn
