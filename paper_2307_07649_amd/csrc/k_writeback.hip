// Last-event-wins write-back: COMB keeps the most recent mail of a batch (Eq. 8, Sec. 2.1.1) and only
// root nodes are written (Sec. 3.2.1).  Arbitration is a segmented maximum over occurrence keys, taken
// with a 64-bit atomic max on a per-(replica, node) scratch word; maximum is order-independent, so the
// winners are deterministic.  Occurrence (event e = off + i, role) has key 1 + 2e + role, prefixed by a
// per-step epoch counter so that the words never need clearing: entries of earlier steps always lose.
#include "tgnn_internal.h"
#include "device_math.h"
#include "writeback_device.h"

namespace tgnn {

__global__ void wb_mark_kernel(const BatchSet* __restrict__ bsp, int N, unsigned long long* winkey,
                               const unsigned long long* __restrict__ epoch) {
  const BatchSet& bs = *bsp;
  int b, i, role;
  if (!occ_decode(bs, blockIdx.x * blockDim.x + threadIdx.x, b, i, role)) return;
  const BatchDesc& bd = bs.b[b];
  const int node = role ? bd.dst[i] : bd.src[i];
  if (node < 0 || node >= N) return;   // an id outside the node range takes no part in the write-back
  atomicMax(winkey + (size_t)bd.replica * N + node, wb_key(*epoch, bd.ev_off + i, role));
}

void writeback_mark(const Dims& d, const BatchSet* bs, int total, unsigned long long* winkey,
                    const unsigned long long* epoch, hipStream_t s) {
  if (total <= 0) return;
  hipLaunchKernelGGL(wb_mark_kernel, dim3((2 * total + 255) / 256), dim3(256), 0, s, bs, d.N, winkey, epoch);
}

__global__ __launch_bounds__(256) void wb_scatter_kernel(WbArgs a) { wb_sgd_block(a, blockIdx.x); }

WbArgs writeback_args(const Dims& d, const BatchSet* bs, int total, const tgnn_state* st, const unsigned long long* winkey,
                      const unsigned long long* epoch, const float* s_new, int p_s, const double* tau,
                      const int32_t* slot_row, const float* s_src, const float* s_dst, const double* tau_src,
                      const double* tau_dst, int32_t* out_winner, const SgdSet* sgd_dev, int sgd_cnt, float lr) {
  WbArgs a;
  a.bs = bs; a.N = d.N; a.dm = d.dm;
  a.vec = (d.dm % 4 == 0 && p_s % 4 == 0) ? 4 : 1;
  a.w = WbPtrs{st->mem, st->mail, st->mem_ts, st->mail_ts, st->mail_eid, s_new, s_src, s_dst, tau, tau_src, tau_dst,
               slot_row, p_s};
  a.winkey = winkey; a.epoch = epoch; a.out_winner = out_winner;
  a.wb_blocks = total > 0 ? (2 * total + 3) / 4 : 0;
  a.sgd = sgd_dev; a.sgd_cnt = sgd_dev != nullptr ? sgd_cnt : 0; a.lr = lr;
  return a;
}

void writeback_scatter(const Dims& d, const BatchSet* bs, int total, const tgnn_state* st,
                       const unsigned long long* winkey, const unsigned long long* epoch, const float* s_new, int p_s,
                       const double* tau, const int32_t* slot_row, const float* s_src, const float* s_dst,
                       const double* tau_src, const double* tau_dst, int32_t* out_winner, hipStream_t s,
                       const SgdSet* sgd_dev, int sgd_cnt, float lr) {
  const WbArgs a = writeback_args(d, bs, total, st, winkey, epoch, s_new, p_s, tau, slot_row, s_src, s_dst, tau_src, tau_dst,
                                  out_winner, sgd_dev, sgd_cnt, lr);
  const int blocks = wb_total_blocks(a);
  if (blocks > 0) hipLaunchKernelGGL(wb_scatter_kernel, dim3(blocks), dim3(256), 0, s, a);
}

}  // namespace tgnn
