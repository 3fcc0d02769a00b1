// Small utility kernels: weight packing into padded / transposed workspace copies, state reset, SGD.
#include <string.h>

#include "tgnn_internal.h"
#include "device_math.h"
#include "prologue_device.h"

namespace tgnn {

__global__ void prologue_kernel(PrologueArgs a) { prologue_block(a, blockIdx.x, gridDim.x, blockIdx.y); }

// Padded copies of the weights (row pitch = the pitch of the activation matrix they multiply), split into
// the blocks that multiply the node rows, the per-slot rows and the attention output, and the transposed
// copies that the data-gradient GEMMs read.
void prologue_fill(tgnn_ctx* ctx, const tgnn_params* p, const BatchSet* bs, const SgdSet* sgd, const SgdSet* zero,
                   float* loss, PrologueArgs& pa) {
  const Dims& d = ctx->d;
  Ws& w = ctx->w;
  static_assert(sizeof(PrologueArgs) <= 4096, "kernel argument block too large");
  memset(&pa, 0, sizeof(pa));
  int n = 0;
  auto add = [&](const float* src, float* dst, int rows, int cols, int zero_to, int ldd, int srs, int scs) {
    pa.d[n++] = PackDesc{src, dst, rows, cols, zero_to, ldd, srs, scs, 0, 0, 0, 0, 0};
  };
  // block-diagonal over the heads: block h of `rows` x `cols` lands at rows h * brd, columns h * bcd of dst
  auto add_bd = [&](const float* src, float* dst, int rows, int cols, int ldd, int srs, int scs, int brd, int bcd, int bsrc) {
    pa.d[n++] = PackDesc{src, dst, rows, cols, 0, ldd, srs, scs, 0, d.H, brd, bcd, bsrc};
  };
  if (p != nullptr) {
    const int dO = d.dO, dm = d.dm, dx = d.dx, dkv = d.dkv, dmrg = d.dO + d.dx, half = d.ldkv;
    add(p->gru_wih, w.Wih_p, 3 * dm, d.d_in, d.ldx, d.ldx, d.d_in, 1);
    add(p->gru_whh, w.Whh_p, 3 * dm, dm, d.ldh, d.ldh, dm, 1);
    // node part of every projection of x = {s' | static}: rows {W_k ; W_v} then, from row `half`, {W_q ; W_o}
    // (rows 2 d_o .. half stay zero); row pitch = the pitch of the node rows
    add(p->wk, w.Wx, dO, dx, d.ldxr, d.ldxr, dkv, 1);
    add(p->wv, w.Wx + (size_t)dO * d.ldxr, dO, dx, d.ldxr, d.ldxr, dkv, 1);
    add(p->wq, w.Wx + (size_t)half * d.ldxr, dO, dx, d.ldxr, d.ldxr, d.dq, 1);
    add(p->wo + dO, w.Wx + (size_t)(half + dO) * d.ldxr, dO, dx, d.ldxr, d.ldxr, dmrg, 1);
    // its transpose, dynamic columns only: WxT[c, j] = Wx[j, c], c < d_m
    // (rows c >= d_m, the static columns, are read only when the static memory is co-trained)
    add(p->wk, w.WxT, dx, dO, dO, d.ldp, 1, dkv);
    add(p->wv, w.WxT + dO, dx, dO, dO, d.ldp, 1, dkv);
    add(p->wq, w.WxT + half, dx, dO, dO, d.ldp, 1, d.dq);
    add(p->wo + dO, w.WxT + half + dO, dx, dO, dO, d.ldp, 1, dmrg);
    // {e | Phi} columns of W_k, W_v (the slots' own inputs), per head: head h owns output rows [h dh, (h + 1) dh)
    if (d.de + d.dt > 0) {
      const int dh = dO / d.H, dc = d.de + d.dt;
      // row h dcp + c, column h dh + dd  <-  W[h dh + dd, d_x + c]
      add_bd(p->wk + dx, w.WkcT, dc, dh, d.ldh, 1, dkv, d.dcp, dh, dh * dkv);
      add_bd(p->wv + dx, w.WvcT, dc, dh, d.ldh, 1, dkv, d.dcp, dh, dh * dkv);
      // row h dh + dd, column h dcp + c  <-  W[h dh + dd, d_x + c]
      add_bd(p->wk + dx, w.Wkc, dh, dc, d.ldz, dkv, 1, dh, d.dcp, dh * dkv);
      add_bd(p->wv + dx, w.Wvc, dh, dc, d.ldz, dkv, 1, dh, d.dcp, dh * dkv);
    }
    // merge layer, attention-output columns, and their transpose
    add(p->wo, w.Wo_o, dO, dO, d.ldh, d.ldh, dmrg, 1);
    add(p->wo, w.WoT_o, dO, dO, d.ldh, d.ldh, 1, dmrg);
    // decoder hidden layer per root: rows {W_s ; W_d}; and for the way back, side by side and transposed:
    // WdecT[c, j] = W_s[j, c], WdecT[c, d_o + j] = W_d[j, c]
    add(p->dec_ws, w.Wdec_p, dO, dO, d.ldh, d.ldh, dO, 1);
    add(p->dec_wd, w.Wdec_p + (size_t)dO * d.ldh, dO, dO, d.ldh, d.ldh, dO, 1);
    add(p->dec_ws, w.WdecT, dO, dO, dO, d.ldkv, 1, dO);
    add(p->dec_wd, w.WdecT + dO, dO, dO, d.ldkv - dO, d.ldkv, 1, dO);
    add(p->gru_wih + 2 * dm, w.WihT_phi, d.dt, 3 * dm, d.ld3, d.ld3, 1, d.d_in);
    if (w.rc_pk != nullptr) {   // the root chain's copies, in MFMA B-operand order: [out column][k]
      const int ks = (dO + 15) / 16;
      const size_t blk = (size_t)ks * ks * 256;
      auto add_mfma = [&](const float* src, int which, int srs, int scs) {
        pa.d[n++] = PackDesc{src, w.rc_pk + which * blk, dO, dO, 0, 0, srs, scs, ks, 0, 0, 0, 0};
      };
      add_mfma(p->wo, 0, dmrg, 1);       // z column n      <- h columns k:      W_o[n, k]
      add_mfma(p->dec_ws, 1, dO, 1);     // hidden column j <- z columns k:      W_s[j, k]
      add_mfma(p->dec_wd, 2, dO, 1);
      add_mfma(p->dec_ws, 3, 1, dO);     // dz column c     <- hidden gradient j: W_s[j, c]
      add_mfma(p->dec_wd, 4, 1, dO);
      add_mfma(p->wo, 5, 1, dmrg);       // dh column c     <- dz columns n:     W_o[n, c]
    }
    // biases of the per-node projections: {b_k | b_v || b_q + W_q Phi(0) | b_o}
    add(p->bk, w.bias_x, 1, dO, dO, d.ldp, 0, 1);
    add(p->bv, w.bias_x + dO, 1, dO, dO, d.ldp, 0, 1);
    add(p->bo, w.bias_x + half + dO, 1, dO, dO, d.ldp, 0, 1);
    pa.bq = p->bq; pa.wq = p->wq; pa.time_b = p->time_b; pa.bq_out = w.bias_x + half;
    pa.dO = dO; pa.dq = d.dq; pa.dx = dx; pa.dt = d.dt;
  }
  pa.n_pack = n;
  if (zero) pa.zero = *zero;
  if (bs) { pa.bs = *bs; pa.bs_dev = w.bs_dev; }
  if (sgd) { pa.sgd = *sgd; pa.sgd_dev = w.sgd_dev; }
  pa.loss = loss;
  pa.epoch = w.epoch;
  pa.ucount = w.ucount;
  pa.q_part = w.q_part; pa.q_part_n = QPHI_BLOCKS * d.dO;
  pa.adam_t = (sgd != nullptr && ctx->adam) ? w.adam_t : nullptr;   // a step that updates the weights is one Adam step
}

dim3 prologue_grid(const PrologueArgs& pa) { return dim3(96, pa.n_pack + pa.zero.cnt + 1); }
void* prologue_func() { return reinterpret_cast<void*>(prologue_kernel); }

void prologue(tgnn_ctx* ctx, const tgnn_params* p, const BatchSet* bs, const SgdSet* sgd, const SgdSet* zero,
              float* loss, hipStream_t s) {
  PrologueArgs pa;
  prologue_fill(ctx, p, bs, sgd, zero, loss, pa);
  hipLaunchKernelGGL(prologue_kernel, prologue_grid(pa), dim3(256), 0, s, pa);
}

__global__ void fill_state_kernel(float* mem, double* mem_ts, float* mail, double* mail_ts, int32_t* mail_eid,
                                  long long row0, long long rows, int dm) {
  const long long total = rows * dm;
  const long long stride = (long long)gridDim.x * blockDim.x;
  for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < 2 * total; i += stride) {
    if (i < total) mem[row0 * dm + i] = 0.f;
    mail[row0 * 2 * dm + i] = 0.f;
    if (i < rows) {
      mem_ts[row0 + i] = 0.0;
      mail_ts[row0 + i] = 0.0;
      mail_eid[row0 + i] = -1;
    }
  }
}

void fill_state(tgnn_ctx* ctx, tgnn_state* st, int replica, hipStream_t s) {
  const Dims& d = ctx->d;
  long long row0 = replica < 0 ? 0 : (long long)replica * d.N;
  long long rows = replica < 0 ? (long long)d.nrep * d.N : d.N;
  hipLaunchKernelGGL(fill_state_kernel, dim3(1024), dim3(256), 0, s, st->mem, st->mem_ts, st->mail, st->mail_ts,
                     st->mail_eid, row0, rows, d.dm);
}

__global__ void sgd_kernel(const SgdSet* __restrict__ set, float lr) {
  const int t = blockIdx.y;
  float* p = set->p[t];
  const float* g = set->g[t];
  const int n = set->n[t];
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) p[i] -= lr * g[i];
}

void sgd_update(const SgdSet* set_dev, int cnt, float lr, hipStream_t s) {
  hipLaunchKernelGGL(sgd_kernel, dim3(64, cnt), dim3(256), 0, s, set_dev, lr);
}

// plain streaming copy: the reference point for HBM-traffic counters (known bytes in, known bytes out)
__global__ void copy_kernel(const float4* __restrict__ src, float4* __restrict__ dst, size_t n) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}
void copy_f4(const void* src, void* dst, size_t n_float4, hipStream_t s) {
  hipLaunchKernelGGL(copy_kernel, dim3(8192), dim3(256), 0, s, static_cast<const float4*>(src),
                     static_cast<float4*>(dst), n_float4);
}

__global__ void zero_set_kernel(SgdSet set) {
  const int t = blockIdx.y;
  float* p = set.p[t];
  const int n = set.n[t];
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) p[i] = 0.f;
}

void zero_set(const SgdSet& set, hipStream_t s) {
  hipLaunchKernelGGL(zero_set_kernel, dim3(64, set.cnt), dim3(256), 0, s, set);
}

}  // namespace tgnn
