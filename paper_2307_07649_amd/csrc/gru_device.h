// Device side of the GRU gates (Eq. 3; see GruFwdArgs), callable from any kernel with blocks of 256 threads.
#pragma once
#include "tgnn_internal.h"
#include "device_math.h"
#include "unique_device.h"

namespace tgnn {

__device__ __forceinline__ float sigmoidf_(float x) { return 1.0f / (1.0f + expf(-x)); }
__device__ __forceinline__ float tanhf_(float x) {
  // tanh(x) = 1 - 2 / (exp(2x) + 1); exact limits at +-inf, no cancellation problem near 0 at 1e-7 level
  const float e = expf(2.0f * x);
  return 1.0f - 2.0f / (e + 1.0f);
}

// gates layout per row: [r | z | n | W_hn h + b_hn], each block ldh floats wide.  block: 0 .. gru_total_blocks(a) - 1
__device__ __forceinline__ void gru_fwd_block(const GruFwdArgs& a, int block) {
  if (a.scan.ucnt != nullptr) {   // block 0 is a passenger: the scan of the slot sort
    if (block == 0) {
      uniq_scan_block(a.scan);
      return;
    }
    --block;
  }
  const int dm = a.dm, ldh = a.ldh, ld3 = a.ld3;
  const int n = a.n_dev ? min(a.n_max, *a.n_dev) : a.n_max;
  const long long stride = (long long)a.gru_blocks * blockDim.x;
  const long long first = block * (long long)blockDim.x + threadIdx.x;
  for (long long i = first; i < (long long)n * dm; i += stride) {
    const int row = (int)(i / dm), c = (int)(i - (long long)row * dm);
    const float h = a.Hm[(size_t)row * ldh + c];
    float out = h;
    if (a.has[row]) {
      const float* gi = a.gi + (size_t)row * ld3;
      const float* gh = a.gh + (size_t)row * ld3;
      const float r = sigmoidf_(gi[c] + gh[c]);
      const float z = sigmoidf_(gi[dm + c] + gh[dm + c]);
      const float hn = gh[2 * dm + c];
      const float nn = tanhf_(gi[2 * dm + c] + r * hn);
      out = (1.0f - z) * nn + z * h;
      float* g = a.gates + (size_t)row * 4 * ldh;
      g[c] = r;
      g[ldh + c] = z;
      g[2 * ldh + c] = nn;
      g[3 * ldh + c] = hn;
    }
    a.x_out[(size_t)row * a.ld_x + c] = out;
  }
  if (a.stat != nullptr) {   // static node memory (Sec. 3.1) rides along as columns d_m .. d_m + d_s of the node row
    const int ds = a.ds;
    for (long long i = first; i < (long long)n * ds; i += stride) {
      const int row = (int)(i / ds), c = (int)(i - (long long)row * ds);
      a.x_out[(size_t)row * a.ld_x + dm + c] = a.stat[(size_t)(a.gid[row] % a.N) * ds + c];
    }
  }
  if (a.zero_buf != nullptr) {
    for (long long i = first; i < (long long)n * a.zero_w; i += stride) a.zero_buf[i] = 0.f;
  }
}

}  // namespace tgnn
