// Distinct-node bookkeeping of a step.  UPDT (Eq. 3) depends only on a node's stored state, so every slot
// that refers to the same (replica, node) gets the same s'.  The step therefore evaluates the GRU once per
// distinct node ("row") and lets slots point at rows; this is an exact shortcut of the per-reference
// re-computation of Sec. 3.2.1.  The attention projections are linear in their input, so their node part
// is taken per row as well.  The backward pass needs, per row, the sum of the gradients of its slots:
// slots are counting-sorted by row and reduced in fixed chunks, so a node referenced thousands of times
// (power-law graphs) costs a few dozen atomic row updates instead of thousands.
#include "tgnn_internal.h"
#include "unique_device.h"
#include "qphi_device.h"

namespace tgnn {

SortArgs sort_args(tgnn_ctx* ctx, int S) {
  Ws& w = ctx->w;
  SortArgs a;
  a.ucount = w.ucount; a.ucnt = w.ucnt; a.rowptr = w.rowptr; a.cursor = w.cursor;
  a.S = S; a.slot_gid = w.slot_gid; a.uidx = w.uidx; a.slot_row = w.slot_row; a.sorted = w.sorted;
  a.sorted_row = w.sorted_row; a.total = w.sort_total;
  return a;
}

// Per-row sums of the slot gradients that reach the per-node projections P = {K | V || q | merge}:
//   neighbour slot (r, j) : dP[row, 0 .. 2 d_o)          += {ds[r, h, j] q[r] | p[r, h, j] dO[r]}   (per head h: the
//                           gradients of the slot's key and value rows, formed here instead of being stored)
//   root slot r           : dP[row, half .. half + 2 d_o) += {dq[r] | dz[r]}          (half = the pitch of {K | V})
// One wavefront owns SEG_CHUNK consecutive entries of the row-sorted slot list; runs of one row are summed
// in registers and leave as one atomic row update per half.
// element c < 2 d_o of the gradient of neighbour slot `sl` (= r k + j)
__device__ __forceinline__ float slot_grad(const SlotGrads& g, int sl, int c) {
  const int r = sl / g.k, j = sl - r * g.k;
  if (c < g.dO) return g.dscore[(size_t)r * g.H * g.k + (c / g.dh) * g.k + j] * g.Qroot[(size_t)r * g.ldh + c];
  const int cc = c - g.dO;
  return g.prob[(size_t)r * g.H * g.k + (cc / g.dh) * g.k + j] * g.dOmat[(size_t)r * g.ldh + cc];
}

#ifndef TGNN_SEG_CHUNK
#define TGNN_SEG_CHUNK 16
#endif
constexpr int SEG_CHUNK = TGNN_SEG_CHUNK;
// SPAN: consecutive chunks per wavefront (1, 2 or 4).  The accumulators of a run of equal rows carry over from chunk
// to chunk, so a node with thousands of slots (a tenth of a step's slots sit on one node of a power-law graph) costs
// one atomic row update per SPAN chunks.  Measured on MI355X it does not pay: the launch is bound by the chain of
// dependent loads of a wavefront, not by the atomics on the popular rows (SPAN 4 against 1: 57 against 49 us for a
// 4,000-event step, SPAN 2: 19 against 14 us for a 600-event step), so the launcher uses 1.
template <int SPAN>
__global__ __launch_bounds__(256) void seg_reduce_kernel(int R, int S, int dO, const int32_t* __restrict__ sort_total,
                                                         const int32_t* __restrict__ sorted,
                                                         const int32_t* __restrict__ sorted_row,
                                                         SlotGrads sg, int ldkv, float* __restrict__ dP, int ldp,
                                                         QPhi qphi) {
  int block = blockIdx.x;
  if (qphi.part != nullptr) {   // the first blocks are passengers: gradients through the query's Phi(0)
    const int nq = qphi_blocks(qphi);
    if (block < nq) {
      qphi_block(qphi, block);
      return;
    }
    block -= nq;
  }
  const int lane = threadIdx.x & 63;
  const int p0 = (block * 4 + (threadIdx.x >> 6)) * SEG_CHUNK * SPAN;
  // lanes fetch the span's slot ids and rows in parallel, without waiting for the length of the list (entries
  // past it are dropped below); they are broadcast afterwards
  int my_slot = -1, my_row = -1;
  if (lane < SEG_CHUNK * SPAN && p0 + lane < S) {
    my_slot = sorted[p0 + lane];
    my_row = sorted_row[p0 + lane];
  }
  const int total = *sort_total;
  if (p0 >= total) return;
  if (p0 + lane >= total) my_slot = my_row = -1;
  // a neighbour slot's root and position among the root's neighbours: one division per slot, done by the lane that
  // fetched it, not one per element
  int my_r = 0, my_j = 0;
  if (my_slot >= R) {
    const int sl = my_slot - R;
    my_r = sl / sg.k;
    my_j = sl - my_r * sg.k;
  }
  const int HK = sg.H * sg.k;
  for (int cb = 0; cb < dO; cb += 128) {   // 128 columns of each of the two sections per pass, 2 + 2 per lane
    // this lane's columns (the same in the key / query section and in the value / merge section) and their head's
    // offset into a root's score gradients and softmax weights
    int ck[2], hoff[2];
    bool live[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int c = cb + lane + 64 * u;
      live[u] = c < dO;
      ck[u] = live[u] ? c : 0;
      hoff[u] = (ck[u] / sg.dh) * sg.k;
    }
    float aK[2] = {0.f, 0.f}, aV[2] = {0.f, 0.f}, aQ[2] = {0.f, 0.f}, aM[2] = {0.f, 0.f};
    bool any_kv = false, any_qm = false;
    int cur = -1;
    auto flush = [&]() __attribute__((always_inline)) {
      if (cur < 0) return;
      float* row = dP + (size_t)cur * ldp;
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        if (live[u]) {
          if (any_kv) { atomicAdd(row + ck[u], aK[u]); atomicAdd(row + dO + ck[u], aV[u]); }
          if (any_qm) { atomicAdd(row + ldkv + ck[u], aQ[u]); atomicAdd(row + ldkv + dO + ck[u], aM[u]); }
        }
      }
    };
#pragma unroll
    for (int ci = 0; ci < SPAN; ++ci) {
      if (p0 + ci * SEG_CHUNK >= total) break;   // uniform over the wavefront
      __builtin_amdgcn_sched_barrier(0);         // one chunk's loads in flight at a time (registers)
      int slots[SEG_CHUNK], rows[SEG_CHUNK], rr[SEG_CHUNK], jj[SEG_CHUNK];
#pragma unroll
      for (int i = 0; i < SEG_CHUNK; ++i) {
        // (readlane: the values are the same for every lane, so they live in scalar registers)
        slots[i] = __builtin_amdgcn_readlane(my_slot, ci * SEG_CHUNK + i);
        rows[i] = __builtin_amdgcn_readlane(my_row, ci * SEG_CHUNK + i);
        rr[i] = __builtin_amdgcn_readlane(my_r, ci * SEG_CHUNK + i);
        jj[i] = __builtin_amdgcn_readlane(my_j, ci * SEG_CHUNK + i);
      }
      // all row loads of the chunk are issued before any is consumed.  Which arrays a slot reads is uniform over the
      // wavefront (a root slot: its dq and dz rows; a neighbour slot: its root's q and dO rows with the slot's score
      // gradient and softmax weight per head: dK = ds q, dV = p dO)
      float xa[SEG_CHUNK][2], xb[SEG_CHUNK][2], wa[SEG_CHUNK][2], wb[SEG_CHUNK][2];
#pragma unroll
      for (int i = 0; i < SEG_CHUNK; ++i) {
        const bool on = rows[i] >= 0;
        const bool root = slots[i] < R;
        const size_t ro = (size_t)(root ? max(slots[i], 0) : rr[i]);
        const float* pa = (root ? sg.dq : sg.Qroot) + ro * sg.ldh;
        const float* pb = (root ? sg.dz : sg.dOmat) + ro * sg.ldh;
        const float* qa = sg.dscore + ro * HK + jj[i];
        const float* qb = sg.prob + ro * HK + jj[i];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const bool ld = on && live[u];
          xa[i][u] = ld ? pa[ck[u]] : 0.f;
          xb[i][u] = ld ? pb[ck[u]] : 0.f;
          wa[i][u] = (ld && !root) ? qa[hoff[u]] : 1.f;
          wb[i][u] = (ld && !root) ? qb[hoff[u]] : 1.f;
        }
      }
#pragma unroll
      for (int i = 0; i < SEG_CHUNK; ++i) {
        if (rows[i] != cur) {
          flush();
#pragma unroll
          for (int u = 0; u < 2; ++u) aK[u] = aV[u] = aQ[u] = aM[u] = 0.f;
          any_kv = any_qm = false;
          cur = rows[i];
        }
        if (rows[i] >= 0) {
          if (slots[i] < R) {
            any_qm = true;
#pragma unroll
            for (int u = 0; u < 2; ++u) { aQ[u] += xa[i][u]; aM[u] += xb[i][u]; }
          } else {
            any_kv = true;
#pragma unroll
            for (int u = 0; u < 2; ++u) { aK[u] += xa[i][u] * wa[i][u]; aV[u] += xb[i][u] * wb[i][u]; }
          }
        }
      }
    }
    flush();
  }
}

static SlotGrads slot_grads(tgnn_ctx* ctx, int R) {
  const Dims& d = ctx->d;
  Ws& w = ctx->w;
  SlotGrads g;
  g.dscore = w.dscore; g.prob = w.prob; g.Qroot = w.Qroot; g.dOmat = w.dOmat; g.dq = w.dq; g.dz = w.dz;
  g.R = R; g.k = d.k; g.H = d.H; g.dO = d.dO; g.dh = d.dO / d.H; g.ldh = d.ldh;
  return g;
}

void seg_reduce(tgnn_ctx* ctx, int R, int S, const QPhi& qphi, hipStream_t s) {
  const Dims& d = ctx->d;
  Ws& w = ctx->w;
  const int span = 1;   // chunks per wavefront (see the kernel)
  const int waves = (S + SEG_CHUNK * span - 1) / (SEG_CHUNK * span);
  const dim3 grid((waves + 3) / 4 + qphi_blocks(qphi));
#define TGNN_SEG_CASE(SP)                                                                                             \
  hipLaunchKernelGGL(seg_reduce_kernel<SP>, grid, dim3(256), 0, s, R, S, d.dO, w.sort_total, w.sorted, w.sorted_row,  \
                     slot_grads(ctx, R), d.ldkv, w.dP, d.ldp, qphi)
  if (span == 4) TGNN_SEG_CASE(4);
  else if (span == 2) TGNN_SEG_CASE(2);
  else TGNN_SEG_CASE(1);
#undef TGNN_SEG_CASE
}

// slot = row: dP[r] = {0 || dq[r] | dz[r]} for roots, dP[R + j] = {dKV[j] || 0} for neighbour slots
__global__ __launch_bounds__(256) void slots_to_dp_kernel(int R, int RK, int dO, SlotGrads sg, int ldkv,
                                                          float* __restrict__ dP, int ldp, QPhi qphi) {
  int block = blockIdx.x;
  if (qphi.part != nullptr) {   // the first blocks are passengers: gradients through the query's Phi(0)
    const int nq = qphi_blocks(qphi);
    if (block < nq) {
      qphi_block(qphi, block);
      return;
    }
    block -= nq;
  }
  const long long i = block * (long long)blockDim.x + threadIdx.x;
  if (i >= (long long)(R + RK) * ldp) return;
  const int row = (int)(i / ldp), c = (int)(i - (long long)row * ldp);
  float x = 0.f;
  if (row < R) {
    const int cc = c - ldkv;
    if (cc >= 0 && cc < dO) x = sg.dq[(size_t)row * sg.ldh + cc];
    else if (cc >= dO && cc < 2 * dO) x = sg.dz[(size_t)row * sg.ldh + (cc - dO)];
  } else if (c < 2 * dO) {
    x = slot_grad(sg, row - R, c);
  }
  dP[i] = x;
}

void slots_to_dp(tgnn_ctx* ctx, int R, int RK, const QPhi& qphi, hipStream_t s) {
  const Dims& d = ctx->d;
  Ws& w = ctx->w;
  const long long total = (long long)(R + RK) * d.ldp;
  if (total <= 0) return;
  hipLaunchKernelGGL(slots_to_dp_kernel, dim3((int)((total + 255) / 256) + qphi_blocks(qphi)), dim3(256), 0, s, R, RK, d.dO,
                     slot_grads(ctx, R), d.ldkv, w.dP, d.ldp, qphi);
}

// debug: per-slot view of per-row data
__global__ void expand_rows_kernel(int S, int dm, const int32_t* __restrict__ slot_row, const float* __restrict__ src,
                                   int ld, const double* __restrict__ src_d, float* __restrict__ dst,
                                   double* __restrict__ dst_d) {
  const long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x;
  if (dst != nullptr) {
    if (i >= (long long)S * dm) return;
    const int s = (int)(i / dm), c = (int)(i - (long long)s * dm);
    const int row = slot_row[s];
    dst[i] = row >= 0 ? src[(size_t)row * ld + c] : 0.f;
  } else {
    if (i >= S) return;
    const int row = slot_row[i];
    dst_d[i] = row >= 0 ? src_d[row] : 0.0;
  }
}

void expand_rows(tgnn_ctx* ctx, int S, const float* src, int ld, const double* src_d, float* dst, double* dst_d,
                 hipStream_t s) {
  const long long total = dst ? (long long)S * ctx->d.dm : S;
  if (total <= 0) return;
  hipLaunchKernelGGL(expand_rows_kernel, dim3((int)((total + 255) / 256)), dim3(256), 0, s, S, ctx->d.dm,
                     ctx->w.slot_row, src, ld, src_d, dst, dst_d);
}

}  // namespace tgnn
