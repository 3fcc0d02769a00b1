// Link-prediction decoder and binary cross-entropy (self-supervision by temporal edges with one sampled
// negative destination per event, Sec. 2.1 / 3.2.2).  logit(a, b) = w2 . ReLU(W_s z_a + W_d z_b + b1) + b2.
// Row layout of the 2n pairs of batch b (events before it: off): rows 2*off + i are the true pairs
// (src_i, dst_i), rows 2*off + n + i the pairs (src_i, neg_i).  The hidden layer is an MFMA GEMM.
#include "tgnn_internal.h"
#include "device_math.h"

namespace tgnn {

__device__ __forceinline__ int batch_of_row(const BatchSet& bs, int row, int mult) {
  int b = 0;
  while (b + 1 < bs.nb && row >= mult * bs.b[b + 1].ev_off) ++b;
  return b;
}

template <int VEC>
__global__ __launch_bounds__(256) void dec_assemble_kernel(const BatchSet* __restrict__ bsp, int dO, const float* __restrict__ z, int ldz,
                                                           float* __restrict__ Adec, int lda) {
  const BatchSet& bs = *bsp;
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= 2 * bs.total) return;
  const int b = batch_of_row(bs, row, 2);
  const int off = bs.b[b].ev_off, n = bs.b[b].n;
  const int local = row - 2 * off;
  const bool neg = local >= n;
  const int i = neg ? local - n : local;
  const int ra = 3 * off + i, rb = 3 * off + (neg ? 2 * n : n) + i;
  float* out = Adec + (size_t)row * lda;
  wave_copy<VEC>(out, z + (size_t)ra * ldz, dO, 0, lane);
  wave_copy<VEC>(out + dO, z + (size_t)rb * ldz, dO, lda - 2 * dO, lane);
}

void decoder_assemble(const Dims& d, const BatchSet* bs, int total, const float* z, int ldz, float* Adec, int lda,
                      hipStream_t s) {
  if (total <= 0) return;
  const int blocks = (2 * total + 3) / 4;
  if (d.dO % 4 == 0) hipLaunchKernelGGL(dec_assemble_kernel<4>, dim3(blocks), dim3(256), 0, s, bs, d.dO, z, ldz, Adec, lda);
  else hipLaunchKernelGGL(dec_assemble_kernel<1>, dim3(blocks), dim3(256), 0, s, bs, d.dO, z, ldz, Adec, lda);
}

// Per row: logit, loss term, d(loss)/d(logit), gradient into the hidden layer; per block: partial sums of
// the w2 / b2 gradients.  loss = mean over batches of (1 / 2n_b) sum softplus(-+logit).
constexpr int DL_ROWS = 16;  // rows per block (the block ends with one atomic per column and two on scalars)
__global__ __launch_bounds__(256) void dec_loss_kernel(const BatchSet* __restrict__ bsp, int dO, const float* __restrict__ h1, int ldh,
                                                       const float* __restrict__ w2, const float* __restrict__ b2,
                                                       float* __restrict__ logits, float* __restrict__ out_loss,
                                                       float* __restrict__ dh1, float* __restrict__ g_w2,
                                                       float* __restrict__ g_b2) {
  __shared__ float red[4][260];
  const BatchSet& bs = *bsp;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int rows = 2 * bs.total;
  float gw[4] = {0.f, 0.f, 0.f, 0.f};  // columns lane, lane+64, lane+128, lane+192
  float gb = 0.f, lsum = 0.f;
  for (int u = 0; u < DL_ROWS / 4; ++u) {
    const int row = blockIdx.x * DL_ROWS + u * 4 + wave;
    if (row >= rows) break;
    const int b = batch_of_row(bs, row, 2);
    const int n = bs.b[b].n;
    const bool pos = (row - 2 * bs.b[b].ev_off) < n;
    const float* hr = h1 + (size_t)row * ldh;
    float acc = 0.f;
    for (int c = lane; c < dO; c += 64) acc += hr[c] * w2[c];
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
    const float l = acc + b2[0];
    const float x = pos ? -l : l;                        // loss term softplus(x)
    const float sp = fmaxf(x, 0.f) + log1pf(expf(-fabsf(x)));
    const float sig = 1.0f / (1.0f + expf(-l));
    const float inv = 1.0f / (2.0f * (float)n);
    const float dl = (sig - (pos ? 1.0f : 0.0f)) * inv;  // d(sum_b loss_b) / d logit
    if (lane == 0) {
      logits[row] = l;
      lsum += sp * inv / (float)bs.nb;
      gb += dl;
    }
    int q = 0;
    for (int c = lane; c < dO; c += 64, ++q) {
      const float h = hr[c];
      dh1[(size_t)row * ldh + c] = h > 0.f ? dl * w2[c] : 0.f;
      gw[q] += dl * h;
    }
  }
  int q = 0;
  for (int c = lane; c < dO; c += 64, ++q) red[wave][c] = gw[q];
  if (lane == 0) { red[wave][256] = gb; red[wave][257] = lsum; }
  __syncthreads();
  if (wave == 0) {
    for (int c = lane; c < dO; c += 64) atomicAdd(g_w2 + c, red[0][c] + red[1][c] + red[2][c] + red[3][c]);
    if (lane == 0) {
      atomicAdd(g_b2, red[0][256] + red[1][256] + red[2][256] + red[3][256]);
      atomicAdd(out_loss, red[0][257] + red[1][257] + red[2][257] + red[3][257]);
    }
  }
}

void decoder_loss(const Dims& d, const BatchSet* bs, int total, const float* h1, int ldh, const float* w2, const float* b2,
                  float* logits, float* out_loss, float* dh1, float* g_w2, float* g_b2, hipStream_t s) {
  if (total <= 0) return;
  hipLaunchKernelGGL(dec_loss_kernel, dim3((2 * total + DL_ROWS - 1) / DL_ROWS), dim3(256), 0, s, bs, d.dO, h1, ldh,
                     w2, b2, logits, out_loss, dh1, g_w2, g_b2);
}

// dz (already multiplied by the ReLU mask of the merge layer) per root from the decoder-input gradient.
__global__ void dec_dz_kernel(const BatchSet* __restrict__ bsp, int dO, const float* __restrict__ dA, int lda, const float* __restrict__ z,
                              int ldz, float* __restrict__ dz) {
  const BatchSet& bs = *bsp;
  const long long total = 3LL * bs.total * dO;
  for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < total;
       i += (long long)gridDim.x * blockDim.x) {
    const int root = (int)(i / dO), c = (int)(i - (long long)root * dO);
    const int b = batch_of_row(bs, root, 3);
    const int off = bs.b[b].ev_off, n = bs.b[b].n;
    const int local = root - 3 * off;
    const int role = local / n, ev = local - role * n;
    const size_t prow = (size_t)(2 * off + ev) * lda, nrow = (size_t)(2 * off + n + ev) * lda;
    float g;
    if (role == 0) g = dA[prow + c] + dA[nrow + c];
    else if (role == 1) g = dA[prow + dO + c];
    else g = dA[nrow + dO + c];
    dz[(size_t)root * ldz + c] = z[(size_t)root * ldz + c] > 0.f ? g : 0.f;
  }
}

void decoder_dz(const Dims& d, const BatchSet* bs, int total_ev, const float* dAdec, int lda, const float* z, int ldz,
                float* dz, hipStream_t s) {
  if (total_ev <= 0) return;
  const long long total = 3LL * total_ev * d.dO;
  hipLaunchKernelGGL(dec_dz_kernel, dim3((int)((total + 255) / 256)), dim3(256), 0, s, bs, d.dO, dAdec, lda, z, ldz, dz);
}

__global__ void mask_dz_kernel(int R, int dO, const float* __restrict__ dz_in, int p_in, const float* __restrict__ z,
                               int ldz, float* __restrict__ dz_out) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= R * dO) return;
  const int r = i / dO, c = i - r * dO;
  dz_out[(size_t)r * ldz + c] = z[(size_t)r * ldz + c] > 0.f ? dz_in[(size_t)r * p_in + c] : 0.f;
}

void mask_dz(int R, int dO, const float* dz_in, int p_in, const float* z, int ldz, float* dz_out, hipStream_t s) {
  if (R <= 0) return;
  hipLaunchKernelGGL(mask_dz_kernel, dim3((R * dO + 255) / 256), dim3(256), 0, s, R, dO, dz_in, p_in, z, ldz, dz_out);
}

__global__ void attn_dx_out_kernel(int R, int RK, int dm, const float* __restrict__ ds_row, int ldh,
                                   float* __restrict__ d_x_root, float* __restrict__ d_x_nbr) {
  const long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x;
  if (i >= (long long)(R + RK) * dm) return;
  const int row = (int)(i / dm), c = (int)(i - (long long)row * dm);
  const float x = ds_row[(size_t)row * ldh + c];
  if (row < R) d_x_root[(size_t)row * dm + c] = x;
  else d_x_nbr[(size_t)(row - R) * dm + c] = x;
}

void attn_dx_out(int R, int RK, int dm, const float* ds_row, int ldh, float* d_x_root, float* d_x_nbr, hipStream_t s) {
  const long long total = (long long)(R + RK) * dm;
  if (total <= 0) return;
  hipLaunchKernelGGL(attn_dx_out_kernel, dim3((int)((total + 255) / 256)), dim3(256), 0, s, R, RK, dm, ds_row, ldh,
                     d_x_root, d_x_nbr);
}

__global__ void zero_kernel(float* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0.f;
}
void zero_f32(float* p, int n, hipStream_t s) {
  if (n > 0) hipLaunchKernelGGL(zero_kernel, dim3((n + 255) / 256), dim3(256), 0, s, p, n);
}

}  // namespace tgnn
