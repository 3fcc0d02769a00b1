// Element-wise part of UPDT = GRU cell (Eq. 3): gates forward.  The matrix products live in k_gemm.hip; the
// gates' backward pass is an epilogue of the product that yields the gradient reaching s'.
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

// gates layout per row: [r | z | n | W_hn h + b_hn], each block ldh floats wide
__global__ void gru_fwd_kernel(int n_max, const int* __restrict__ n_dev, int dm, int ldh, int ld3,
                               const float* __restrict__ gi, const float* __restrict__ gh,
                               const float* __restrict__ Hm, const int32_t* __restrict__ has,
                               float* __restrict__ gates, float* __restrict__ x_out, int ld_x,
                               const float* __restrict__ stat, int ds, const int32_t* __restrict__ gid, int N,
                               float* __restrict__ zero_buf, int zero_w, int gru_blocks, SortArgs scan) {
  int block = blockIdx.x;
  if (scan.ucnt != nullptr) {   // block 0 is a passenger: the scan of the slot sort
    if (block == 0) {
      uniq_scan_block(scan);
      return;
    }
    --block;
  }
  const int n = n_dev ? min(n_max, *n_dev) : n_max;
  const long long stride = (long long)gru_blocks * blockDim.x;
  const long long first = block * (long long)blockDim.x + threadIdx.x;
  for (long long i = first; i < (long long)n * dm; i += stride) {
    const int row = (int)(i / dm), c = (int)(i - (long long)row * dm);
    const float h = Hm[(size_t)row * ldh + c];
    float out = h;
    if (has[row]) {
      const float* a = gi + (size_t)row * ld3;
      const float* b = gh + (size_t)row * ld3;
      const float r = sigmoidf_(a[c] + b[c]);
      const float z = sigmoidf_(a[dm + c] + b[dm + c]);
      const float hn = b[2 * dm + c];
      const float nn = tanhf_(a[2 * dm + c] + r * hn);
      out = (1.0f - z) * nn + z * h;
      float* g = gates + (size_t)row * 4 * ldh;
      g[c] = r;
      g[ldh + c] = z;
      g[2 * ldh + c] = nn;
      g[3 * ldh + c] = hn;
    }
    x_out[(size_t)row * ld_x + c] = out;
  }
  if (stat != nullptr) {   // static node memory (Sec. 3.1) rides along as columns d_m .. d_m + d_s of the node row
    for (long long i = first; i < (long long)n * ds; i += stride) {
      const int row = (int)(i / ds), c = (int)(i - (long long)row * ds);
      x_out[(size_t)row * ld_x + dm + c] = stat[(size_t)(gid[row] % N) * ds + c];
    }
  }
  if (zero_buf != nullptr) {
    for (long long i = first; i < (long long)n * zero_w; i += stride) zero_buf[i] = 0.f;
  }
}

void gru_gates_fwd(const Dims& d, int n, const int* n_dev, const float* gi, const float* gh, const float* Hm,
                   const int32_t* has, float* gates, float* x_out, int ld_x, const float* stat, const int32_t* gid,
                   float* zero_buf, int zero_w, hipStream_t s, const SortArgs& scan) {
  if (n <= 0) return;
  const long long total = (long long)n * d.dm;
  const int blocks = (int)((total + 255) / 256);
  const int scan_blocks = scan.ucnt != nullptr ? 1 : 0;
  hipLaunchKernelGGL(gru_fwd_kernel, dim3(blocks + scan_blocks), dim3(256), 0, s, n, n_dev, d.dm, d.ldh, d.ld3, gi, gh, Hm,
                     has, gates, x_out, ld_x, stat, d.ds, gid, d.N, zero_buf, zero_w, blocks, scan);
}

}  // namespace tgnn
