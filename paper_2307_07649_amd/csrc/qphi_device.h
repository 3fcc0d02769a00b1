// Gradients through the query's time encoding Phi(0) = cos(time_b) (see QPhi): a block of 256 threads takes
// 256 consecutive (n, c) pairs, numbered n * d_t + c.  Small and off the critical path, so it rides as extra
// blocks of another launch.
#pragma once
#include "tgnn_internal.h"
#include "device_math.h"

namespace tgnn {

__device__ __forceinline__ void qphi_block(const QPhi& q, int block) {
  __shared__ float gb[256];   // per-thread contribution to g_b[c], summed over the block's n per c below
  const int i = block * 256 + threadIdx.x;
  const int n = i / q.dt, c = i - n * q.dt;
  float contrib = 0.f;
  if (n < q.dO) {
    float cs_n = 0.f;
    for (int b = 0; b < QPHI_BLOCKS; ++b) cs_n += q.part[(size_t)b * q.dO + n];
    float sn, cs;
    sincos_reduced((double)q.time_b[c], sn, cs);
    atomicAdd(q.g_wq + (size_t)n * q.dq_w + q.dx + c, cs_n * cs);
    contrib = -sn * cs_n * q.wq[(size_t)n * q.dq_w + q.dx + c];
  }
  gb[threadIdx.x] = contrib;
  __syncthreads();
  // thread t < d_t sums the entries of this block whose c equals (first c of the block + t) mod d_t
  if ((int)threadIdx.x < q.dt) {
    const int c0 = (block * 256 + (int)threadIdx.x) % q.dt;
    float acc = 0.f;
    for (int t = threadIdx.x; t < 256; t += q.dt) acc += gb[t];
    atomicAdd(q.g_b + c0, acc);
  }
}

}  // namespace tgnn
