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
//   neighbour slot s : dP[row, 0 .. 2 d_o)              += dKV[s - R]
//   root slot r      : dP[row, half .. half + 2 d_o)     += {dq[r] | dz[r]}          (half = the pitch of dKV)
// One wavefront owns SEG_CHUNK consecutive entries of the row-sorted slot list; runs of one row are summed
// in registers and leave as one atomic row update per half.
// Per root and head: Zs = sum_j ds[h][j] CE_j and Zp = sum_j p[h][j] CE_j over the root's neighbour slots (see
// AttnSums).  One wavefront per root, 16 bytes of a row per lane; a block is four roots.  HM: heads the
// accumulators are laid out for.
typedef float zsum_f4 __attribute__((ext_vector_type(4)));
template <int HM, int NP>
__device__ __forceinline__ void zsum_root(const AttnSums& a, int r, const float* wv, int lane) {
  const int HK = a.H * a.k, n4 = a.dcp >> 2;
  const int c = a.cnt[r];
  constexpr int NJ = 10;   // rows whose loads are issued together
  // With NP = 2 a lane takes the 16-byte pieces f0 + lane and f0 + 64 + lane of every row: a row of 65 to 128
  // pieces (C1: 68) is then one round trip to memory, not two with the second nearly empty.  (NP = 1: the
  // accumulators for many heads leave no registers for that.)
  for (int f0 = 0; f0 < n4; f0 += 64 * NP) {
    const int fa = f0 + lane, fb = f0 + 64 + lane;
    const bool on_a = fa < n4, on_b = NP > 1 && fb < n4;
    zsum_f4 as[NP][HM], ap[NP][HM];
#pragma unroll
    for (int h = 0; h < HM; ++h)
#pragma unroll
      for (int e = 0; e < NP; ++e) as[e][h] = ap[e][h] = zsum_f4{0.f, 0.f, 0.f, 0.f};
    for (int j0 = 0; j0 < c; j0 += NJ) {
      zsum_f4 ce[NP][NJ];
#pragma unroll
      for (int jj = 0; jj < NJ; ++jj) {
#pragma unroll
        for (int e = 0; e < NP; ++e) ce[e][jj] = zsum_f4{0.f, 0.f, 0.f, 0.f};
        const float* row = a.CE + ((size_t)r * a.k + j0 + jj) * a.ldce;
        if (on_a && j0 + jj < c) ce[0][jj] = *reinterpret_cast<const zsum_f4*>(row + 4 * fa);
        if (NP > 1 && on_b && j0 + jj < c) ce[NP - 1][jj] = *reinterpret_cast<const zsum_f4*>(row + 4 * fb);
      }
#pragma unroll
      for (int jj = 0; jj < NJ; ++jj) {
        if (j0 + jj < c) {
#pragma unroll
          for (int h = 0; h < HM; ++h) {
            if (h < a.H) {
              const float ws = wv[h * a.k + j0 + jj], wp = wv[HK + h * a.k + j0 + jj];
#pragma unroll
              for (int e = 0; e < NP; ++e) {
                as[e][h] += ws * ce[e][jj];
                ap[e][h] += wp * ce[e][jj];
              }
            }
          }
        }
      }
    }
#pragma unroll
    for (int h = 0; h < HM; ++h) {
      if (h < a.H) {
        float* zs = a.Zs + (size_t)r * a.ldz + h * a.dcp;
        float* zp = a.Zp + (size_t)r * a.ldz + h * a.dcp;
        if (on_a) {
          *reinterpret_cast<zsum_f4*>(zs + 4 * fa) = as[0][h];
          *reinterpret_cast<zsum_f4*>(zp + 4 * fa) = ap[0][h];
        }
        if (NP > 1 && on_b) {
          *reinterpret_cast<zsum_f4*>(zs + 4 * fb) = as[NP - 1][h];
          *reinterpret_cast<zsum_f4*>(zp + 4 * fb) = ap[NP - 1][h];
        }
      }
    }
  }
}

__device__ __forceinline__ void zsum_block(const AttnSums& a, int block) {
  __shared__ float w_lds[4][2 * TGNN_MAX_HEADS * TGNN_MAX_K];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int HK = a.H * a.k;
  float* wv = w_lds[wave];
  // ZSUM_PER_WAVE roots per wavefront, one after the other: the launch this rides in holds two blocks per compute
  // unit, and with a block per four roots the last of them waited for a free place for half of the launch
  for (int i = 0; i < ZSUM_PER_WAVE; ++i) {
    const int r = (block * 4 + wave) * ZSUM_PER_WAVE + i;
    if (r >= a.R) return;   // per wavefront; no block barrier below
    for (int p = lane; p < HK; p += 64) {
      wv[p] = a.ds_out[(size_t)r * HK + p];
      wv[HK + p] = a.prob[(size_t)r * HK + p];
    }
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_s_waitcnt(0xc07f);   // the wavefront's LDS writes are visible to all its lanes
    __builtin_amdgcn_wave_barrier();
    if (a.H <= 2) zsum_root<2, 2>(a, r, wv, lane);
    else zsum_root<TGNN_MAX_HEADS, 1>(a, r, wv, lane);
    __builtin_amdgcn_wave_barrier();   // all lanes are done reading wv before the next root overwrites it
  }
}

constexpr int SEG_CHUNK = 16;
__global__ __launch_bounds__(256) void seg_reduce_kernel(int R, int S, int dO, const int32_t* __restrict__ sort_total,
                                                         const int32_t* __restrict__ sorted,
                                                         const int32_t* __restrict__ sorted_row,
                                                         const float* __restrict__ dq, const float* __restrict__ dz,
                                                         int ldh, const float* __restrict__ dKV, int ldkv,
                                                         float* __restrict__ dP, int ldp, QPhi qphi, AttnSums zs) {
  int block = blockIdx.x;
  if (qphi.part != nullptr) {   // the first blocks are passengers: gradients through the query's Phi(0)
    const int nq = qphi_blocks(qphi);
    if (block < nq) {
      qphi_block(qphi, block);
      return;
    }
    block -= nq;
  }
  {   // the last blocks, also passengers: the per-root sums for the weight gradients of the {e | Phi} columns
      // (behind the row sums, which the next launch waits for the longest)
    const int n_seg = ((S + SEG_CHUNK - 1) / SEG_CHUNK + 3) / 4;
    if (block >= n_seg) {
      if (block - n_seg < zsum_blocks(zs)) zsum_block(zs, block - n_seg);
      return;
    }
  }
  const int lane = threadIdx.x & 63;
  const int chunk = block * 4 + (threadIdx.x >> 6);
  const int p0 = chunk * SEG_CHUNK;
  // lanes fetch the chunk's slot ids and rows in parallel, without waiting for the length of the list (entries
  // past it are dropped below); they are broadcast afterwards
  int my_slot = -1, my_row = -1;
  if (lane < SEG_CHUNK && p0 + lane < S) {
    my_slot = sorted[p0 + lane];
    my_row = sorted_row[p0 + lane];
  }
  const int total = *sort_total;
  if (p0 >= total) return;
  if (p0 + lane >= total) my_slot = my_row = -1;
  int slots[SEG_CHUNK], rows[SEG_CHUNK];
#pragma unroll
  for (int i = 0; i < SEG_CHUNK; ++i) {
    slots[i] = __shfl(my_slot, i);
    rows[i] = __shfl(my_row, i);
  }
  for (int cb = 0; cb < 2 * dO; cb += 256) {   // 256 columns per pass, 4 per lane
    // all row loads of the chunk are issued before any is consumed
    float v[SEG_CHUNK][4];
#pragma unroll
    for (int i = 0; i < SEG_CHUNK; ++i) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int c = cb + lane + 64 * q;
        float x = 0.f;
        if (rows[i] >= 0 && c < 2 * dO) {
          const int slot = slots[i];
          if (slot < R) x = c < dO ? dq[(size_t)slot * ldh + c] : dz[(size_t)slot * ldh + (c - dO)];
          else x = dKV[(size_t)(slot - R) * ldkv + c];
        }
        v[i][q] = x;
      }
    }
    float akv[4] = {0.f, 0.f, 0.f, 0.f}, aqm[4] = {0.f, 0.f, 0.f, 0.f};
    bool any_kv = false, any_qm = false;
    int cur = -1;
    auto flush = [&]() __attribute__((always_inline)) {
      if (cur < 0) return;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int c = cb + lane + 64 * q;
        if (c < 2 * dO) {
          if (any_kv) atomicAdd(dP + (size_t)cur * ldp + c, akv[q]);
          if (any_qm) atomicAdd(dP + (size_t)cur * ldp + ldkv + c, aqm[q]);
        }
      }
    };
#pragma unroll
    for (int i = 0; i < SEG_CHUNK; ++i) {
      if (rows[i] != cur) {
        flush();
#pragma unroll
        for (int q = 0; q < 4; ++q) akv[q] = aqm[q] = 0.f;
        any_kv = any_qm = false;
        cur = rows[i];
      }
      if (rows[i] >= 0) {
        if (slots[i] < R) {
          any_qm = true;
#pragma unroll
          for (int q = 0; q < 4; ++q) aqm[q] += v[i][q];
        } else {
          any_kv = true;
#pragma unroll
          for (int q = 0; q < 4; ++q) akv[q] += v[i][q];
        }
      }
    }
    flush();
  }
}

void seg_reduce(tgnn_ctx* ctx, int R, int S, const QPhi& qphi, hipStream_t s, const AttnSums& zs) {
  const Dims& d = ctx->d;
  Ws& w = ctx->w;
  const int chunks = (S + SEG_CHUNK - 1) / SEG_CHUNK;
  hipLaunchKernelGGL(seg_reduce_kernel, dim3((chunks + 3) / 4 + qphi_blocks(qphi) + zsum_blocks(zs)), dim3(256), 0, s, R, S,
                     d.dO, w.sort_total, w.sorted, w.sorted_row, w.dq, w.dz, d.ldh, w.dKV, d.ldkv, w.dP, d.ldp, qphi, zs);
}

// slot = row: dP[r] = {0 || dq[r] | dz[r]} for roots, dP[R + j] = {dKV[j] || 0} for neighbour slots
__global__ __launch_bounds__(256) void slots_to_dp_kernel(int R, int RK, int dO, const float* __restrict__ dq,
                                                          const float* __restrict__ dz, int ldh,
                                                          const float* __restrict__ dKV, int ldkv,
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
    if (cc >= 0 && cc < dO) x = dq[(size_t)row * ldh + cc];
    else if (cc >= dO && cc < 2 * dO) x = dz[(size_t)row * ldh + (cc - dO)];
  } else if (c < 2 * dO) {
    x = dKV[(size_t)(row - R) * ldkv + c];
  }
  dP[i] = x;
}

void slots_to_dp(tgnn_ctx* ctx, int R, int RK, const QPhi& qphi, hipStream_t s) {
  const Dims& d = ctx->d;
  Ws& w = ctx->w;
  const long long total = (long long)(R + RK) * d.ldp;
  if (total <= 0) return;
  hipLaunchKernelGGL(slots_to_dp_kernel, dim3((int)((total + 255) / 256) + qphi_blocks(qphi)), dim3(256), 0, s, R, RK, d.dO,
                     w.dq, w.dz, d.ldh, w.dKV, d.ldkv, w.dP, d.ldp, qphi);
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
