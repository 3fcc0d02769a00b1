// Distinct-node bookkeeping of a step.  UPDT (Eq. 3) depends only on a node's stored state, so every slot
// that refers to the same (replica, node) gets the same s'.  The step therefore evaluates the GRU once per
// distinct node ("row") and lets slots point at rows; this is an exact shortcut of the per-reference
// re-computation of Sec. 3.2.1.  The backward pass needs, per row, the sum of the gradients of its slots:
// slots are counting-sorted by row and reduced in fixed chunks, so a node referenced thousands of times
// (power-law graphs) costs a few dozen atomic row updates instead of thousands.
#include "tgnn_internal.h"

namespace tgnn {

// Adds 1 to counter[key] for every lane with key >= 0 and returns the value before this lane's increment.
// Lanes of a wavefront that share a key are merged into one atomic (power-law graphs put thousands of
// slots on one node, and atomics on one address serialise).  The grouping loop uses only cross-lane ALU
// operations; the atomics of all group leaders are then issued together, so the wave pays one round trip.
__device__ __forceinline__ int wave_counted_add(int32_t* counter, int key, bool want_result) {
  const int lane = threadIdx.x & 63;
  bool pending = key >= 0;
  int leader = lane, count = 0, rank = 0;
  while (true) {
    const unsigned long long todo = __ballot(pending);
    if (todo == 0ull) break;
    const int first = __ffsll((long long)todo) - 1;
    const int k = __shfl(key, first);
    const bool mine = pending && key == k;
    const unsigned long long same = __ballot(mine);
    if (mine) {
      leader = first;
      count = __popcll(same);
      rank = __popcll(same & ((1ull << lane) - 1ull));
      pending = false;
    }
  }
  int base = 0;
  if (key >= 0 && leader == lane) {
    if (want_result) base = atomicAdd(counter + key, count);
    else atomicAdd(counter + key, count);
  }
  if (!want_result) return 0;
  base = __shfl(base, leader);
  return base + rank;
}

// slot -> row, and the number of slots per row
__global__ void uniq_map_kernel(int S, const int32_t* __restrict__ slot_gid, const int32_t* __restrict__ uidx,
                                int32_t* __restrict__ slot_row, int32_t* __restrict__ ucnt) {
  const int s = blockIdx.x * blockDim.x + threadIdx.x;
  int row = -1;
  if (s < S) {
    const int gid = slot_gid[s];
    if (gid >= 0) row = uidx[gid];
    slot_row[s] = row;
  }
  wave_counted_add(ucnt, row, false);
}

// exclusive scan of ucnt[0 .. U) into rowptr[0 .. U] and cursor[0 .. U); one block
__global__ __launch_bounds__(1024) void uniq_scan_kernel(const int32_t* __restrict__ ucount,
                                                         const int32_t* __restrict__ ucnt,
                                                         int32_t* __restrict__ rowptr, int32_t* __restrict__ cursor) {
  __shared__ int part[1024];
  const int U = *ucount;
  const int per = (U + 1023) / 1024;
  const int lo = min(U, (int)threadIdx.x * per), hi = min(U, lo + per);
  int sum = 0;
  for (int i = lo; i < hi; ++i) sum += ucnt[i];
  part[threadIdx.x] = sum;
  __syncthreads();
  for (int off = 1; off < 1024; off <<= 1) {
    int v = threadIdx.x >= off ? part[threadIdx.x - off] : 0;
    __syncthreads();
    part[threadIdx.x] += v;
    __syncthreads();
  }
  int run = part[threadIdx.x] - sum;
  for (int i = lo; i < hi; ++i) {
    rowptr[i] = run;
    cursor[i] = run;
    run += ucnt[i];
  }
  if (threadIdx.x == 1023) rowptr[U] = part[1023];
}

__global__ void uniq_fill_kernel(int S, const int32_t* __restrict__ slot_row, int32_t* __restrict__ cursor,
                                 int32_t* __restrict__ sorted) {
  const int s = blockIdx.x * blockDim.x + threadIdx.x;
  const int row = s < S ? slot_row[s] : -1;
  const int pos = wave_counted_add(cursor, row, true);
  if (row >= 0) sorted[pos] = s;
}

void uniq_map(tgnn_ctx* ctx, int S, hipStream_t s) {
  Ws& w = ctx->w;
  hipLaunchKernelGGL(uniq_map_kernel, dim3((S + 255) / 256), dim3(256), 0, s, S, w.slot_gid, w.uidx, w.slot_row, w.ucnt);
}

void uniq_sort(tgnn_ctx* ctx, int S, hipStream_t s) {
  Ws& w = ctx->w;
  hipLaunchKernelGGL(uniq_scan_kernel, dim3(1), dim3(1024), 0, s, w.ucount, w.ucnt, w.rowptr, w.cursor);
  hipLaunchKernelGGL(uniq_fill_kernel, dim3((S + 255) / 256), dim3(256), 0, s, S, w.slot_row, w.cursor, w.sorted);
}

// ds_row[row, c] += sum over the row's slots of the gradient reaching s' of that slot:
//   root slot r      : dMin[r, dO + c] + dQsub[r, c]     (merge layer + query)
//   neighbour slot   : dCsub[slot - R, c]                (key/value input)
// One wavefront owns SEG_CHUNK consecutive entries of the row-sorted slot list.
constexpr int SEG_CHUNK = 16;
__global__ __launch_bounds__(256) void seg_reduce_kernel(int R, int dm, int dO, const int32_t* __restrict__ ucount,
                                                         const int32_t* __restrict__ rowptr,
                                                         const int32_t* __restrict__ sorted,
                                                         const int32_t* __restrict__ slot_row,
                                                         const int32_t* __restrict__ has,
                                                         const float* __restrict__ dMin, int ldm,
                                                         const float* __restrict__ dQsub,
                                                         const float* __restrict__ dCsub, int ldsub,
                                                         float* __restrict__ ds_row, int ldh) {
  const int lane = threadIdx.x & 63;
  const int chunk = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int total = rowptr[*ucount];
  const int p0 = chunk * SEG_CHUNK;
  if (p0 >= total) return;
  const int n = min(SEG_CHUNK, total - p0);
  // lanes fetch the chunk's slot ids and rows in parallel; they are broadcast below
  int my_slot = -1, my_row = -1;
  if (lane < n) {
    my_slot = sorted[p0 + lane];
    my_row = slot_row[my_slot];
    if (!has[my_row]) my_row = -1;   // no mail consumed: s' is the stored memory, a constant
  }
  // all row loads of the chunk are issued before any is consumed
  float v[SEG_CHUNK][4];
  int rows[SEG_CHUNK];
#pragma unroll
  for (int i = 0; i < SEG_CHUNK; ++i) {
    const int slot = __shfl(my_slot, i);
    rows[i] = __shfl(my_row, i);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int c = lane + 64 * q;
      float x = 0.f;
      if (rows[i] >= 0 && c < dm) {
        if (slot < R) x = dMin[(size_t)slot * ldm + dO + c] + dQsub[(size_t)slot * ldsub + c];
        else x = dCsub[(size_t)(slot - R) * ldsub + c];
      }
      v[i][q] = x;
    }
  }
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  int cur = -1;
#pragma unroll
  for (int i = 0; i < SEG_CHUNK; ++i) {
    if (rows[i] != cur) {
      if (cur >= 0) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int c = lane + 64 * q;
          if (c < dm) atomicAdd(ds_row + (size_t)cur * ldh + c, acc[q]);
        }
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) acc[q] = 0.f;
      cur = rows[i];
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) acc[q] += v[i][q];
  }
  if (cur >= 0) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int c = lane + 64 * q;
      if (c < dm) atomicAdd(ds_row + (size_t)cur * ldh + c, acc[q]);
    }
  }
}

void seg_reduce(tgnn_ctx* ctx, int R, int S, hipStream_t s) {
  const Dims& d = ctx->d;
  Ws& w = ctx->w;
  const int chunks = (S + SEG_CHUNK - 1) / SEG_CHUNK;
  hipLaunchKernelGGL(seg_reduce_kernel, dim3((chunks + 3) / 4), dim3(256), 0, s, R, d.dm, d.dO, w.ucount, w.rowptr,
                     w.sorted, w.slot_row, w.has, w.dMin, d.ldm, w.dQsub, w.dCsub, d.ldsub, w.ds_row, d.ldh);
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
