// Device-side pieces of the counting sort of slots by node row (see k_unique.hip).  The scan and the fill
// are small, so they do not get launches of their own in the training step: the map rides in the state-gather
// launch, the scan (one block) in the GRU-gates launch, the fill in the softmax-attention launch.
#pragma once
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

// exclusive scan of ucnt[0 .. U) into rowptr[0 .. U] and cursor[0 .. U) by one block (any multiple of 64
// threads up to 1024).  Each wavefront owns a contiguous range (a multiple of 256 elements) and walks it 256
// elements at a time: a lane reads four consecutive counts, the wavefront scans the lane sums with shuffles.
// The arrays must be 16-byte aligned.
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
__device__ __forceinline__ void uniq_scan_block(const SortArgs& a) {
  __shared__ int wsum[16];
  const int U = *a.ucount;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, waves = blockDim.x >> 6;
  const int per = ((U + waves * 256 - 1) / (waves * 256)) * 256;
  const int lo = min(U, wave * per), hi = min(U, lo + per);
  int sum = 0;
  for (int i = lo + lane * 4; i < hi; i += 256) {
    const int4 v = scan_load4(a.ucnt, i, hi);
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
    const int4 v = scan_load4(a.ucnt, i, hi);
    const int t = v.x + v.y + v.z + v.w;
    int inc = t;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int o = __shfl_up(inc, off);
      if (lane >= off) inc += o;
    }
    const int e = run + inc - t;
    const int4 out = make_int4(e, e + v.x, e + v.x + v.y, e + v.x + v.y + v.z);
    scan_store4(a.rowptr, i, hi, out);
    scan_store4(a.cursor, i, hi, out);
    run += __shfl(inc, 63);
  }
  // the last wavefront ends at U (or owns nothing): its running sum is the total
  if ((int)threadIdx.x == (int)blockDim.x - 1) {
    a.rowptr[U] = run;
    *a.total = run;
  }
}

// slot -> row, and the number of slots per row; `block` counts the blocks that do this work
__device__ __forceinline__ void uniq_map_block(const SortArgs& a, int block) {
  const int s = block * blockDim.x + threadIdx.x;
  int row = -1;
  if (s < a.S) {
    const int gid = a.slot_gid[s];
    if (gid >= 0) row = a.uidx[gid];
    a.slot_row[s] = row;
  }
  wave_counted_add(a.ucnt, row, false);
}

// slot s goes to the next free position of its row's range; `block` counts the blocks that do this work
__device__ __forceinline__ void uniq_fill_block(const SortArgs& a, int block) {
  const int s = block * blockDim.x + threadIdx.x;
  const int row = s < a.S ? a.slot_row[s] : -1;
  const int pos = wave_counted_add(a.cursor, row, true);
  if (row >= 0) {
    a.sorted[pos] = s;
    a.sorted_row[pos] = row;
  }
}

}  // namespace tgnn
