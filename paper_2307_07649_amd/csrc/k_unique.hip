// Distinct-node bookkeeping of a step.  UPDT (Eq. 3) depends only on a node's stored state, so every slot
// that refers to the same (replica, node) gets the same s'.  The step therefore evaluates the GRU once per
// distinct node ("row") and lets slots point at rows; this is an exact shortcut of the per-reference
// re-computation of Sec. 3.2.1.  The attention projections are linear in their input, so their node part
// is taken per row as well.  The backward pass needs, per row, the sum of the gradients of its slots:
// slots are counting-sorted by row and reduced in fixed chunks, so a node referenced thousands of times
// (power-law graphs) costs a few dozen atomic row updates instead of thousands.
#include "tgnn_internal.h"

namespace tgnn {

// Adds 1 to counter[key] for every lane with key >= 0 and returns the value before this lane's increment.
// Lanes of a wavefront that share a key are merged into one atomic (power-law graphs put thousands of
// slots on one node, and atomics on one address serialise).  Every lane of the wavefront must call it.
// The set of lanes that share lane j's key is the ballot of (key == key of lane j); 64 such ballots, each
// written into lane j's registers, give every lane its set without a data-dependent loop.  The atomics of all
// group leaders are then issued together, so the wave pays one round trip.
__device__ __forceinline__ int wave_counted_add(int32_t* counter, int key, bool want_result) {
  const int lane = threadIdx.x & 63;
  unsigned lo = 0u, hi = 0u;
#pragma unroll
  for (int j = 0; j < 64; ++j) {
    const int kj = __builtin_amdgcn_readlane(key, j);
    const unsigned long long m = __ballot(key == kj);
    lo = lane == j ? (unsigned)m : lo;
    hi = lane == j ? (unsigned)(m >> 32) : hi;
  }
  const int count = __popc(lo) + __popc(hi);
  const int rank = __builtin_amdgcn_mbcnt_hi(hi, __builtin_amdgcn_mbcnt_lo(lo, 0u));   // set members below this lane
  const int leader = lo != 0u ? __ffs((int)lo) - 1 : 32 + __ffs((int)hi) - 1;
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

// exclusive scan of ucnt[0 .. U) into rowptr[0 .. U] and cursor[0 .. U); one block of 16 wavefronts.  Each
// wavefront owns a contiguous range (a multiple of 256 elements) and walks it 256 elements at a time: a lane
// reads four consecutive counts, the wavefront scans the lane sums with shuffles.  The arrays must be
// 16-byte aligned.
__device__ __forceinline__ int4 scan_load4(const int32_t* __restrict__ p, int i, int hi) {
  if (i + 3 < hi) return *reinterpret_cast<const int4*>(p + i);
  int4 v = make_int4(0, 0, 0, 0);
  if (i < hi) v.x = p[i];
  if (i + 1 < hi) v.y = p[i + 1];
  if (i + 2 < hi) v.z = p[i + 2];
  return v;
}
__device__ __forceinline__ void scan_store4(int32_t* __restrict__ p, int i, int hi, const int4& v) {
  if (i + 3 < hi) {
    *reinterpret_cast<int4*>(p + i) = v;
    return;
  }
  if (i < hi) p[i] = v.x;
  if (i + 1 < hi) p[i + 1] = v.y;
  if (i + 2 < hi) p[i + 2] = v.z;
}
__global__ __launch_bounds__(1024) void uniq_scan_kernel(const int32_t* __restrict__ ucount,
                                                         const int32_t* __restrict__ ucnt,
                                                         int32_t* __restrict__ rowptr, int32_t* __restrict__ cursor) {
  __shared__ int wsum[16];
  const int U = *ucount;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int per = ((U + 16 * 256 - 1) / (16 * 256)) * 256;
  const int lo = min(U, wave * per), hi = min(U, lo + per);
  int sum = 0;
  for (int i = lo + lane * 4; i < hi; i += 256) {
    const int4 v = scan_load4(ucnt, i, hi);
    sum += v.x + v.y + v.z + v.w;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
  if (lane == 0) wsum[wave] = sum;
  __syncthreads();
  int run = 0;
  for (int w = 0; w < wave; ++w) run += wsum[w];
  for (int i0 = lo; i0 < hi; i0 += 256) {
    const int i = i0 + lane * 4;
    const int4 v = scan_load4(ucnt, i, hi);
    const int t = v.x + v.y + v.z + v.w;
    int inc = t;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int o = __shfl_up(inc, off);
      if (lane >= off) inc += o;
    }
    const int e = run + inc - t;
    const int4 out = make_int4(e, e + v.x, e + v.x + v.y, e + v.x + v.y + v.z);
    scan_store4(rowptr, i, hi, out);
    scan_store4(cursor, i, hi, out);
    run += __shfl(inc, 63);
  }
  if (threadIdx.x == 1023) rowptr[U] = run;   // the last wavefront ends at U (or owns nothing): run is the total
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

// Per-row sums of the slot gradients that reach the per-node projections P = {K | V || q | merge}:
//   neighbour slot s : dP[row, 0 .. 2 d_o)              += dKV[s - R]
//   root slot r      : dP[row, half .. half + 2 d_o)     += {dq[r] | dz[r]}          (half = the pitch of dKV)
// One wavefront owns SEG_CHUNK consecutive entries of the row-sorted slot list; runs of one row are summed
// in registers and leave as one atomic row update per half.
constexpr int SEG_CHUNK = 16;
__global__ __launch_bounds__(256) void seg_reduce_kernel(int R, int dO, const int32_t* __restrict__ ucount,
                                                         const int32_t* __restrict__ rowptr,
                                                         const int32_t* __restrict__ sorted,
                                                         const int32_t* __restrict__ slot_row,
                                                         const float* __restrict__ dq, const float* __restrict__ dz,
                                                         int ldh, const float* __restrict__ dKV, int ldkv,
                                                         float* __restrict__ dP, int ldp) {
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
  }
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

void seg_reduce(tgnn_ctx* ctx, int R, int S, hipStream_t s) {
  const Dims& d = ctx->d;
  Ws& w = ctx->w;
  const int chunks = (S + SEG_CHUNK - 1) / SEG_CHUNK;
  hipLaunchKernelGGL(seg_reduce_kernel, dim3((chunks + 3) / 4), dim3(256), 0, s, R, d.dO, w.ucount, w.rowptr, w.sorted,
                     w.slot_row, w.dq, w.dz, d.ldh, w.dKV, d.ldkv, w.dP, d.ldp);
}

// slot = row: dP[r] = {0 || dq[r] | dz[r]} for roots, dP[R + j] = {dKV[j] || 0} for neighbour slots
__global__ void slots_to_dp_kernel(int R, int RK, int dO, const float* __restrict__ dq, const float* __restrict__ dz,
                                   int ldh, const float* __restrict__ dKV, int ldkv, float* __restrict__ dP, int ldp) {
  const long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x;
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

void slots_to_dp(tgnn_ctx* ctx, int R, int RK, hipStream_t s) {
  const Dims& d = ctx->d;
  Ws& w = ctx->w;
  const long long total = (long long)(R + RK) * d.ldp;
  if (total <= 0) return;
  hipLaunchKernelGGL(slots_to_dp_kernel, dim3((int)((total + 255) / 256)), dim3(256), 0, s, R, RK, d.dO, w.dq, w.dz, d.ldh,
                     w.dKV, d.ldkv, w.dP, d.ldp);
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
