// Element-wise parts of UPDT = GRU cell (Eq. 3): gates forward, and the last stage of the gradients of the
// time-encoding parameters.  The matrix products live in k_gemm.hip; the gates' backward pass is an epilogue
// of the product that yields the gradient reaching s'.
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

// The query's time encoding is Phi(0) = cos(time_b): its gradient, and that of the columns of W_q which
// multiply it, need only the column sums of dq over the roots:
//   g_b[c]           += -sin(time_b[c]) * sum_n colsum[n] wq[n, dx + c]
//   g_wq[n, dx + c]  += colsum[n] cos(time_b[c])
// The attention backward kernel adds each root's dq to one of QPHI_BLOCKS partial rows q_part[., d_o] (cleared
// beforehand); time_grad_finish adds the rows up and applies the two formulas (extra grid rows of that kernel).
// Time-encoding gradients, last stage: the NT GEMMs that produce the gradient reaching Phi write, per 64-row
// tile, the column sums of its products with -sin(arg) (and with -sin(arg) delta) instead of the matrix itself;
// this kernel adds the tiles of up to two such launches (keys, mails) to g_w / g_b.
// grid (ceil(2 dt / 32), TGF_SPLIT + q_rows); block = 32 columns x 32 tile groups.  Rows y < TGF_SPLIT add the
// tile sums; rows y >= TGF_SPLIT (present when q.part != NULL) take 1024 consecutive (n, c) pairs of the
// query's Phi(0) gradients each.
constexpr int TGF_SPLIT = 8;
__global__ __launch_bounds__(1024) void time_grad_finish_kernel(TgRegion r0, TgRegion r1, int dt,
                                                                float* __restrict__ g_w, float* __restrict__ g_b,
                                                                QPhi q) {
  __shared__ float red[32][33];
  if (blockIdx.y >= TGF_SPLIT) {
    if (blockIdx.x != 0) return;
    __shared__ float gb[1024];   // per-thread contribution to g_b[c], summed over the block's n per c below
    const int i = (blockIdx.y - TGF_SPLIT) * 1024 + threadIdx.x;
    const int n = i / dt, c = i - n * dt;
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
    // pairs are numbered n * dt + c: thread t < dt sums the entries of this block whose c equals
    // (first c of the block + t) mod dt
    if ((int)threadIdx.x < dt) {
      const int first = (blockIdx.y - TGF_SPLIT) * 1024;
      const int c0 = (first + threadIdx.x) % dt;
      float acc = 0.f;
      for (int t = threadIdx.x; t < 1024; t += dt) acc += gb[t];
      atomicAdd(g_b + c0, acc);
    }
    return;
  }
  const int cx = threadIdx.x & 31, cy = threadIdx.x >> 5;
  const int c = blockIdx.x * 32 + cx;
  float acc = 0.f;
  if (c < 2 * dt) {
#pragma unroll
    for (int reg = 0; reg < 2; ++reg) {
      const TgRegion& r = reg == 0 ? r0 : r1;
      if (r.partial == nullptr) continue;
      const int rows = r.rows_dev != nullptr ? min(r.rows, *r.rows_dev) : r.rows;
      const int tiles = (rows + NT_BM - 1) / NT_BM;
#pragma unroll 4
      for (int b = blockIdx.y * 32 + cy; b < tiles; b += 32 * TGF_SPLIT) acc += r.partial[(size_t)b * 2 * dt + c];
    }
  }
  red[cy][cx] = acc;
  __syncthreads();
  if (cy == 0 && c < 2 * dt) {
    float t = 0.f;
#pragma unroll
    for (int j = 0; j < 32; ++j) t += red[j][cx];
    atomicAdd(c < dt ? g_w + c : g_b + (c - dt), t);
  }
}

void time_grad_finish(const TgRegion& r0, const TgRegion& r1, int dt, float* g_w, float* g_b, const QPhi* q,
                      hipStream_t s) {
  QPhi qq;
  if (q != nullptr) qq = *q;
  const int q_rows = qq.part != nullptr ? (qq.dO * dt + 1023) / 1024 : 0;
  hipLaunchKernelGGL(time_grad_finish_kernel, dim3((2 * dt + 31) / 32, TGF_SPLIT + q_rows), dim3(1024), 0, s, r0, r1, dt,
                     g_w, g_b, qq);
}

}  // namespace tgnn
