// Device-side pieces of the counting sort of slots by node row (see k_unique.hip).  The scan and the fill
// are small, so they do not get launches of their own in the training step: the map rides in the state-gather
// launch, the scan (one block) in the GRU-gates launch, the fill in the softmax-attention launch.
#pragma once
#include "tgnn_internal.h"

namespace tgnn {

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

// The map and the fill pass count slots per node row.  On power-law graphs one node holds a tenth of a step's slots,
// and atomics on one address complete one at a time in the L2 (tens of nanoseconds each), so the counts are first
// taken per block in an LDS table (open addressing; LDS atomics on one word cost a few cycles) and only one global
// atomic per block and distinct row follows.  A block of 256 threads takes UNIQ_PER_BLOCK consecutive slots.
constexpr int UNIQ_PER_BLOCK = 1024;
constexpr int UNIQ_TABLE = 2048;   // >= 2 x the distinct rows a block can meet
__host__ __device__ inline int uniq_blocks(int S) { return (S + UNIQ_PER_BLOCK - 1) / UNIQ_PER_BLOCK; }

struct UniqTable {
  int key[UNIQ_TABLE];
  int val[UNIQ_TABLE];
};
__device__ __forceinline__ void uniq_table_clear(UniqTable& t) {
  for (int i = threadIdx.x; i < UNIQ_TABLE; i += blockDim.x) { t.key[i] = -1; t.val[i] = 0; }
}
// the entry of `row` (inserted if absent)
__device__ __forceinline__ int uniq_table_slot(UniqTable& t, int row) {
  int h = (int)(((unsigned)row * 2654435761u) >> 21) & (UNIQ_TABLE - 1);
  for (;;) {
    const int k = atomicCAS(&t.key[h], -1, row);
    if (k == -1 || k == row) return h;
    h = (h + 1) & (UNIQ_TABLE - 1);
  }
}

// slot -> row, and the number of slots per row; `block` counts the blocks that do this work
__device__ __forceinline__ void uniq_map_block(const SortArgs& a, int block) {
  __shared__ UniqTable tab;
  uniq_table_clear(tab);
  __syncthreads();
  for (int s = block * UNIQ_PER_BLOCK + threadIdx.x; s < min(a.S, (block + 1) * UNIQ_PER_BLOCK); s += blockDim.x) {
    const int gid = a.slot_gid[s];
    const int row = gid >= 0 ? a.uidx[gid] : -1;
    a.slot_row[s] = row;
    if (row >= 0) atomicAdd(&tab.val[uniq_table_slot(tab, row)], 1);
  }
  __syncthreads();
  for (int i = threadIdx.x; i < UNIQ_TABLE; i += blockDim.x)
    if (tab.key[i] >= 0) atomicAdd(a.ucnt + tab.key[i], tab.val[i]);
}

// slot s goes to the next free position of its row's range; `block` counts the blocks that do this work
__device__ __forceinline__ void uniq_fill_block(const SortArgs& a, int block) {
  __shared__ UniqTable tab;
  uniq_table_clear(tab);
  __syncthreads();
  const int s_end = min(a.S, (block + 1) * UNIQ_PER_BLOCK);
  // the block's slots per row, then one range per row claimed from the row's cursor, then positions inside it
  int my_slot[UNIQ_PER_BLOCK / 256];
#pragma unroll
  for (int u = 0; u < UNIQ_PER_BLOCK / 256; ++u) {
    const int s = block * UNIQ_PER_BLOCK + u * 256 + (int)threadIdx.x;
    const int row = s < s_end ? a.slot_row[s] : -1;
    my_slot[u] = -1;
    if (row >= 0) {
      my_slot[u] = uniq_table_slot(tab, row);
      atomicAdd(&tab.val[my_slot[u]], 1);
    }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < UNIQ_TABLE; i += blockDim.x)
    if (tab.key[i] >= 0) tab.val[i] = atomicAdd(a.cursor + tab.key[i], tab.val[i]);
  __syncthreads();
#pragma unroll
  for (int u = 0; u < UNIQ_PER_BLOCK / 256; ++u) {
    if (my_slot[u] >= 0) {
      const int s = block * UNIQ_PER_BLOCK + u * 256 + (int)threadIdx.x;
      const int pos = atomicAdd(&tab.val[my_slot[u]], 1);
      a.sorted[pos] = s;
      a.sorted_row[pos] = tab.key[my_slot[u]];
    }
  }
}

}  // namespace tgnn
