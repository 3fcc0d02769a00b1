// Link-prediction decoder and binary cross-entropy (self-supervision by temporal edges with one sampled
// negative destination per event, Sec. 2.1 / 3.2.2).  logit(a, b) = w2 . ReLU(W_s z_a + W_d z_b + b1) + b2.
// The hidden layer is linear in {z_a | z_b} before its ReLU, so the two products are taken once per root
// (one MFMA GEMM, Pdec = z {W_s ; W_d}^T) and a pair only adds two rows: the source's W_s z is shared by its
// true and its negative pair.  Backward, the pair kernel leaves per root the gradient of its row of Pdec; the
// GEMM that maps it back to z applies the ReLU gate of the merge layer in its epilogue.
// Row layout of the (1 + J) n pairs of batch b (events before it: off; J negative sets): rows (1 + J) off + i are the
// true pairs (src_i, dst_i), rows (1 + J) off + (1 + g) n + i the pairs (src_i, neg_{g,i}); roots (2 + J) off +
// {0, n, 2n, ...} + i are src, dst, neg set 0, ...
#include "tgnn_internal.h"
#include "device_math.h"

namespace tgnn {

__device__ __forceinline__ int batch_of_row(const BatchSet& bs, int row, int mult) {
  int b = 0;
  while (b + 1 < bs.nb && row >= mult * bs.b[b + 1].ev_off) ++b;
  return b;
}

// One wavefront per event (both of its pairs), at most DP_BLOCKS blocks of four wavefronts which stride over
// the events (every block ends with one atomic per column of w2: more blocks would queue up there).  Per pair: hidden layer, logit,
// loss term, d(loss)/d(logit); per root: gradient of its Pdec row ({W_s part | W_d part}: a source receives
// the sum of its two pairs in the first half, a destination its pair in the second half, the other halves
// are zero); per block: partial sums of the w2 / b2 gradients and of the loss.
// loss = mean over batches of (1 / 2n_b) sum softplus(-+logit).
constexpr int DP_BLOCKS = 256;
__global__ __launch_bounds__(256) void dec_pair_kernel(const BatchSet* __restrict__ bsp, int dO,
                                                       const float* __restrict__ Pdec, int ldp,
                                                       const float* __restrict__ b1, const float* __restrict__ w2,
                                                       const float* __restrict__ b2, float* __restrict__ logits,
                                                       float* __restrict__ out_loss, float* __restrict__ h1, int ldh,
                                                       float* __restrict__ dPdec, float* __restrict__ g_w2,
                                                       float* __restrict__ g_b2) {
  __shared__ float red[4][260];
  const BatchSet& bs = *bsp;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float gw[4] = {0.f, 0.f, 0.f, 0.f};  // columns lane, lane+64, lane+128, lane+192
  float gb = 0.f, lsum = 0.f;
  float bb[4], ww[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int c = lane + 64 * q;
    bb[q] = c < dO ? b1[c] : 0.f;
    ww[q] = c < dO ? w2[c] : 0.f;
  }
  const float b2v = b2[0];
  const int nneg = bs.nneg;
  for (int ev = blockIdx.x * 4 + wave; ev < bs.total; ev += gridDim.x * 4) {
    const int b = batch_of_row(bs, ev, 1);
    const int off = bs.b[b].ev_off, n = bs.b[b].n;
    const int i = ev - off;
    const size_t ra = (size_t)((2 + nneg) * off + i) * ldp;   // the source's row; the partner of pair g is n (1 + g) rows on
    const float inv = 1.0f / (2.0f * (float)n);
    float ps[4], dsrc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int c = lane + 64 * q;
      ps[q] = c < dO ? Pdec[ra + c] + bb[q] : 0.f;
    }
    float lterm = 0.f;
    // pair 0 is the true pair (src, dst); pair 1 + g pairs the source with the negative destination of set g.  With
    // nneg sets the step stands for nneg trainers that share the positive batch (Sec. 3.2.2): the loss is the mean of
    // their losses, the gradient that of their sum, so the true pair counts nneg times in the gradient.
    for (int pr = 0; pr <= nneg; ++pr) {
      const size_t rb = ra + (size_t)(1 + pr) * n * ldp;
      float h[4], acc = 0.f;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int c = lane + 64 * q;
        h[q] = c < dO ? fmaxf(ps[q] + Pdec[rb + dO + c], 0.f) : 0.f;
        acc += h[q] * ww[q];
      }
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
      const float lg = acc + b2v;
      const float sgm = 1.0f / (1.0f + expf(-lg));
      float dl, sp;
      if (pr == 0) {   // softplus(-logit)
        sp = fmaxf(-lg, 0.f) + log1pf(expf(-fabsf(lg)));
        dl = (sgm - 1.0f) * inv * (float)nneg;
      } else {         // softplus(logit), averaged over the sets in the loss
        sp = (fmaxf(lg, 0.f) + log1pf(expf(-fabsf(lg)))) / (float)nneg;
        dl = sgm * inv;
      }
      const int row = (1 + nneg) * off + pr * n + i;
      if (lane == 0) {
        logits[row] = lg;
        gb += dl;
      }
      lterm += sp;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int c = lane + 64 * q;
        if (c < dO) {
          const float dh = h[q] > 0.f ? dl * ww[q] : 0.f;
          h1[(size_t)row * ldh + c] = h[q];
          dPdec[rb + c] = 0.f;
          dPdec[rb + dO + c] = dh;
          dsrc[q] += dh;
          gw[q] += dl * h[q];
        }
      }
    }
    if (lane == 0) lsum += lterm * inv / (float)bs.nb;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int c = lane + 64 * q;
      if (c < dO) {
        dPdec[ra + c] = dsrc[q];
        dPdec[ra + dO + c] = 0.f;
      }
    }
  }
#pragma unroll
  for (int q = 0; q < 4; ++q) red[wave][lane + 64 * q] = gw[q];
  if (lane == 0) { red[wave][256] = gb; red[wave][257] = lsum; }
  __syncthreads();
  if (wave == 0) {
    if (g_w2 != nullptr)    // (NULL in a forward-only pass)
      for (int c = lane; c < dO; c += 64) atomicAdd(g_w2 + c, red[0][c] + red[1][c] + red[2][c] + red[3][c]);
    if (lane == 0) {
      if (g_b2 != nullptr) atomicAdd(g_b2, red[0][256] + red[1][256] + red[2][256] + red[3][256]);
      if (out_loss != nullptr) atomicAdd(out_loss, red[0][257] + red[1][257] + red[2][257] + red[3][257]);
    }
  }
}

void decoder_pairs(const Dims& d, const BatchSet* bs, int total, const float* Pdec, int ldp, const float* b1,
                   const float* w2, const float* b2, float* logits, float* out_loss, float* h1, float* dPdec,
                   float* g_w2, float* g_b2, hipStream_t s) {
  if (total <= 0) return;
  hipLaunchKernelGGL(dec_pair_kernel, dim3(std::min((total + 3) / 4, DP_BLOCKS)), dim3(256), 0, s, bs, d.dO, Pdec, ldp, b1,
                     w2, b2, logits, out_loss, h1, d.ldh, dPdec, g_w2, g_b2);
}

// Edge-classification head (Sec. 4 "Datasets": C classes, several true per event).  One wavefront per event: hidden
// layer h = ReLU(W_s z_src + W_d z_dst + b1) from the two roots' rows of Pdec, then class by class the logit
// W2[c] . h + b2[c] (a row of W2 per lane round, summed over the wavefront), its cross-entropy term
// softplus(logit) - y logit, d loss / d logit = (sigmoid(logit) - y) / (n C), and the hidden layer's gradient
// sum_c dlogit_c W2[c] gated by the ReLU.  Roots of batch b: [src | dst] from root 2 * ev_off on.  The weight
// gradients of W2 / b2 are left to the weight-gradient GEMM (dlog^T h1).
__global__ __launch_bounds__(256) void dec_class_kernel(const BatchSet* __restrict__ bsp, int dO, int C,
                                                        const float* __restrict__ Pdec, int ldp,
                                                        const float* __restrict__ b1, const float* __restrict__ w2,
                                                        const float* __restrict__ b2, float* __restrict__ logits,
                                                        float* __restrict__ out_loss, float* __restrict__ h1, int ldh,
                                                        float* __restrict__ dPdec, float* __restrict__ dlog, int ldc) {
  __shared__ float red[4];
  const BatchSet& bs = *bsp;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float bb[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) bb[q] = lane + 64 * q < dO ? b1[lane + 64 * q] : 0.f;
  float lsum = 0.f;
  for (int ev = blockIdx.x * 4 + wave; ev < bs.total; ev += gridDim.x * 4) {
    const int b = batch_of_row(bs, ev, 1);
    const int off = bs.b[b].ev_off, n = bs.b[b].n;
    const int i = ev - off;
    const size_t ra = (size_t)(2 * off + i) * ldp, rb = ra + (size_t)n * ldp;   // the source's and the destination's row
    const float* __restrict__ y = bs.b[b].labels + (size_t)i * C;
    const float inv = 1.0f / ((float)n * (float)C);
    float h[4], dh[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int c = lane + 64 * q;
      h[q] = c < dO ? fmaxf(Pdec[ra + c] + bb[q] + Pdec[rb + dO + c], 0.f) : 0.f;
      if (c < dO) h1[(size_t)ev * ldh + c] = h[q];
    }
    float lterm = 0.f;
    for (int cls = 0; cls < C; ++cls) {
      const float* __restrict__ wr = w2 + (size_t)cls * dO;
      float wv[4], acc = 0.f;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int c = lane + 64 * q;
        wv[q] = c < dO ? wr[c] : 0.f;
        acc += h[q] * wv[q];
      }
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
      const float lg = acc + b2[cls], yv = y[cls];
      const float sgm = 1.0f / (1.0f + expf(-lg));
      lterm += fmaxf(lg, 0.f) + log1pf(expf(-fabsf(lg))) - yv * lg;
      const float dl = (sgm - yv) * inv;
      if (lane == 0) {
        logits[(size_t)ev * C + cls] = lg;
        dlog[(size_t)ev * ldc + cls] = dl;
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) dh[q] += dl * wv[q];
    }
    if (lane == 0) lsum += lterm * inv / (float)bs.nb;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int c = lane + 64 * q;
      if (c < dO) {
        const float gq = h[q] > 0.f ? dh[q] : 0.f;
        dPdec[ra + c] = gq; dPdec[ra + dO + c] = 0.f;
        dPdec[rb + c] = 0.f; dPdec[rb + dO + c] = gq;
      }
    }
  }
  if (lane == 0) red[wave] = lsum;
  __syncthreads();
  if (threadIdx.x == 0 && out_loss != nullptr) atomicAdd(out_loss, red[0] + red[1] + red[2] + red[3]);
}

void decoder_classes(const Dims& d, const BatchSet* bs, int total, const float* Pdec, int ldp, const float* b1,
                     const float* w2, const float* b2, float* logits, float* out_loss, float* h1, float* dPdec,
                     float* dlog, hipStream_t s) {
  if (total <= 0) return;
  hipLaunchKernelGGL(dec_class_kernel, dim3(std::min((total + 3) / 4, 4 * DP_BLOCKS)), dim3(256), 0, s, bs, d.dO, d.nC, Pdec,
                     ldp, b1, w2, b2, logits, out_loss, h1, d.ldh, dPdec, dlog, d.ldc);
}

// Rank of every event's true pair among its pairs with the sampled negative destinations (pair layout of the
// epoch-parallel step); one thread per event, the sum of the reciprocal ranks once per block.
__global__ __launch_bounds__(256) void rank_kernel(const BatchSet* __restrict__ bsp, const float* __restrict__ logits,
                                                   float* __restrict__ rank, float* __restrict__ rr_sum) {
  __shared__ float red[4];
  const BatchSet& bs = *bsp;
  const int ev = blockIdx.x * 256 + threadIdx.x;
  float rr = 0.f;
  if (ev < bs.total) {
    const int b = batch_of_row(bs, ev, 1);
    const int off = bs.b[b].ev_off, n = bs.b[b].n, J = bs.nneg;
    const size_t r0 = (size_t)(1 + J) * off + (ev - off);
    const float st = logits[r0];
    int above = 0, same = 0;
    for (int g = 0; g < J; ++g) {
      const float sn = logits[r0 + (size_t)(1 + g) * n];
      above += sn > st ? 1 : 0;
      same += sn == st ? 1 : 0;
    }
    const float r = 1.0f + (float)above + 0.5f * (float)same;
    rank[ev] = r;
    rr = 1.0f / r;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) rr += __shfl_xor(rr, o);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = rr;
  __syncthreads();
  if (threadIdx.x == 0) atomicAdd(rr_sum, red[0] + red[1] + red[2] + red[3]);
}

void reciprocal_ranks(const BatchSet* bs, int total, const float* logits, float* rank, float* rr_sum, hipStream_t s) {
  if (total <= 0) return;
  hipLaunchKernelGGL(rank_kernel, dim3((total + 255) / 256), dim3(256), 0, s, bs, logits, rank, rr_sum);
}

// Predictions of the classification head against the targets: one thread per (event, class), counts summed per
// block before the three device-wide atomics.
__global__ __launch_bounds__(256) void class_count_kernel(const BatchSet* __restrict__ bsp, int C,
                                                          const float* __restrict__ logits, int32_t* __restrict__ counts) {
  __shared__ int red[3];
  const BatchSet& bs = *bsp;
  if (threadIdx.x < 3) red[threadIdx.x] = 0;
  __syncthreads();
  const long long i = blockIdx.x * 256ll + threadIdx.x;
  int tp = 0, fp = 0, fn = 0;
  if (i < (long long)bs.total * C) {
    const int ev = (int)(i / C), cls = (int)(i - (long long)ev * C);
    const int b = batch_of_row(bs, ev, 1);
    const bool y = bs.b[b].labels[(size_t)(ev - bs.b[b].ev_off) * C + cls] > 0.5f;
    const bool pred = logits[i] > 0.f;
    tp = pred && y; fp = pred && !y; fn = !pred && y;
  }
  const int ntp = __popcll(__ballot(tp)), nfp = __popcll(__ballot(fp)), nfn = __popcll(__ballot(fn));
  if ((threadIdx.x & 63) == 0) {
    if (ntp) atomicAdd(&red[0], ntp);
    if (nfp) atomicAdd(&red[1], nfp);
    if (nfn) atomicAdd(&red[2], nfn);
  }
  __syncthreads();
  if (threadIdx.x < 3 && red[threadIdx.x] != 0) atomicAdd(counts + threadIdx.x, red[threadIdx.x]);
}

void class_counts(const BatchSet* bs, int total, int C, const float* logits, int32_t* counts, hipStream_t s) {
  if (total <= 0) return;
  const long long n = (long long)total * C;
  hipLaunchKernelGGL(class_count_kernel, dim3((int)((n + 255) / 256)), dim3(256), 0, s, bs, C, logits, counts);
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
