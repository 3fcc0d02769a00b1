// Device side of the prologue (weight packing, clears, descriptor copies; see PrologueArgs), callable from any
// kernel: the work is laid out on a grid of nbx x (n_pack + zero.cnt + 1) blocks of any size; (bx, y) is the
// calling block's place in it.
#pragma once
#include "tgnn_internal.h"
#include "device_math.h"

namespace tgnn {

__device__ __forceinline__ void prologue_block(const PrologueArgs& a, int bx, int nbx, int y) {
  if (y < a.n_pack) {
    const PackDesc d = a.d[y];
    if (d.mfma_ks > 0) {   // MFMA B-operand order
      const int total = ((d.rows + 15) >> 4) * d.mfma_ks * 256;
      for (int i = bx * blockDim.x + threadIdx.x; i < total; i += nbx * blockDim.x) {
        const int slab = i >> 8, t = i & 255, lane = t >> 2, c = t & 3;
        const int cb = slab / d.mfma_ks, s = slab - cb * d.mfma_ks;
        const int row = cb * 16 + (lane & 15), k = s * 16 + (lane >> 4) * 4 + c;
        d.dst[i] = (row < d.rows && k < d.cols) ? d.src[(size_t)row * d.srs + (size_t)k * d.scs] : 0.f;
      }
      return;
    }
    if (d.nblk > 0) {   // block-diagonal
      const int per = d.rows * d.cols, total = d.nblk * per;
      for (int i = bx * blockDim.x + threadIdx.x; i < total; i += nbx * blockDim.x) {
        const int h = i / per, rc = i - h * per;
        // consecutive threads walk whichever index is contiguous in the source
        int r, c;
        if (d.srs == 1) { c = rc / d.rows; r = rc - c * d.rows; }
        else { r = rc / d.cols; c = rc - r * d.cols; }
        d.dst[(size_t)(h * d.brd + r) * d.ldd + h * d.bcd + c] = d.src[(size_t)h * d.bsrc + (size_t)r * d.srs + (size_t)c * d.scs];
      }
      return;
    }
    const int total = d.rows * d.zero_to;
    const float* __restrict__ src = d.src;
    float* __restrict__ dst = d.dst;
    const int stride = nbx * blockDim.x;
    // four elements per pass, their loads issued together
    for (int i0 = bx * blockDim.x + threadIdx.x; i0 < total; i0 += 4 * stride) {
      float v[4];
      int off[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int i = i0 + j * stride;
        const int r = i / d.zero_to, c = i - r * d.zero_to;
        off[j] = i < total ? r * d.ldd + c : -1;
        v[j] = (i < total && c < d.cols) ? src[(size_t)r * d.srs + (size_t)c * d.scs] : 0.f;
      }
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (off[j] >= 0) dst[off[j]] = v[j];
    }
  } else if (y < a.n_pack + a.zero.cnt) {
    float* p = a.zero.p[y - a.n_pack];
    const int n = a.zero.n[y - a.n_pack];
    for (int i = bx * blockDim.x + threadIdx.x; i < n; i += nbx * blockDim.x) p[i] = 0.f;
  } else if (bx == 0) {
    if (a.bs_dev) {
      const int* src = reinterpret_cast<const int*>(&a.bs);
      int* dst = reinterpret_cast<int*>(a.bs_dev);
      for (int i = threadIdx.x; i < (int)(sizeof(BatchSet) / sizeof(int)); i += blockDim.x) dst[i] = src[i];
    }
    if (a.sgd_dev) {
      const int* src = reinterpret_cast<const int*>(&a.sgd);
      int* dst = reinterpret_cast<int*>(a.sgd_dev);
      for (int i = threadIdx.x; i < (int)(sizeof(SgdSet) / sizeof(int)); i += blockDim.x) dst[i] = src[i];
    }
    for (int i = threadIdx.x; i < a.q_part_n; i += blockDim.x) a.q_part[i] = 0.f;
    if (threadIdx.x == 0) {
      if (a.loss) *a.loss = 0.f;
      if (a.adam_t) *a.adam_t += 1;
      if (a.head_of_step) {
        *a.ucount_next = 0;
      } else {
        *a.epoch += 1ull;
        *a.ucount = 0;
      }
    }
  } else if (a.bq_out != nullptr) {
    // the query's time encoding Phi(0) = cos(time_b) does not depend on the root: fold W_q Phi(0) into the
    // bias.  One wavefront per output row, rows dealt over blocks 1 .. nbx - 1 of this grid row.
    const int lane = threadIdx.x & 63;
    const int wv = (bx - 1) * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const int n_wv = (nbx - 1) * (blockDim.x >> 6);
    for (int n = wv; n < a.dO; n += n_wv) {
      float acc = 0.f;
      for (int c = lane; c < a.dt; c += 64) acc += a.wq[(size_t)n * a.dq + a.dx + c] * time_enc(0.0, 0.f, a.time_b[c]);
      for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
      if (lane == 0) a.bq_out[n] = a.bq[n] + acc;
    }
  }
}

}  // namespace tgnn
