// Softmax attention over the k sampled neighbours of one root (Eq. 7), forward and backward.
// One wavefront per root: the k key (or value) rows are staged in LDS, the H*k scores are computed by
// H*k lanes, the per-head softmax runs over at most 32 values, and the weighted sums are taken with one
// lane per output element.  The projections themselves (Eq. 4-6) are MFMA GEMMs.
#include "tgnn_internal.h"
#include "unique_device.h"

namespace tgnn {

struct AttnShape {
  int R, k, H, dO, dh, ldq, ldkv, ldo;
};

constexpr int ROWS_IN_FLIGHT = 10;  // neighbour rows whose loads are issued together (k = 10: all of them)
// MAX_E (template parameter of both kernels): columns per lane, lane + 64 u for u < MAX_E; 2 for d_o <= 128, else 4
// (d_o <= 256)

// LDS floats per wave
__host__ __device__ inline int attn_lds_floats(int k, int H, int dO) { return dO + k * (dO + 1) + 2 * H * k; }

// A wavefront has few others on its SIMD to hide behind, so every dependent global load costs a full memory
// latency.  Both kernels therefore issue everything they will need of the first ROWS_IN_FLIGHT neighbours
// (with k = 10 that is everything) as one burst right after the two index loads: the query (or dO) row, the
// key rows and the value rows; rows beyond the first batch are fetched batch by batch where they are used.
template <int MAX_E>
__global__ __launch_bounds__(256) void attn_fwd_kernel(AttnShape sh, const float* __restrict__ q,
                                                       const int32_t* __restrict__ slot_row,
                                                       const float* __restrict__ KV,
                                                       const int32_t* __restrict__ cnt, float* __restrict__ prob,
                                                       float* __restrict__ Omat, SortArgs fill) {
  extern __shared__ float lds[];
  int block = blockIdx.x;
  if (fill.ucnt != nullptr) {   // the first blocks are passengers: the fill pass of the slot sort
    const int fill_blocks = (fill.S + 255) / 256;
    if (block < fill_blocks) {
      uniq_fill_block(fill, block);
      return;
    }
    block -= fill_blocks;
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = block * 4 + wave;
  if (r >= sh.R) return;
  float* sq = lds + (size_t)wave * attn_lds_floats(sh.k, sh.H, sh.dO);
  float* sK = sq + sh.dO;
  float* sa = sK + sh.k * (sh.dO + 1);
  const int c = cnt[r];
  const size_t qrow = slot_row != nullptr ? (size_t)slot_row[r] : (size_t)r;   // q is stored per distinct node
  const int HK = sh.H * sh.k;
  float* pr = prob + (size_t)r * HK;
  float* out = Omat + (size_t)r * sh.ldo;
  if (c == 0) {
    for (int p = lane; p < HK; p += 64) pr[p] = 0.f;
    for (int e = lane; e < sh.dO; e += 64) out[e] = 0.f;
    return;
  }
  const float scale = 1.0f / sqrtf((float)c);
  // the burst: q, and the key and value rows of the first batch
  float qreg[MAX_E], kreg[ROWS_IN_FLIGHT][MAX_E], vreg[ROWS_IN_FLIGHT][MAX_E];
#pragma unroll
  for (int u = 0; u < MAX_E; ++u) {
    const int e = lane + 64 * u;
    qreg[u] = e < sh.dO ? q[qrow * sh.ldq + e] : 0.f;
  }
#pragma unroll
  for (int jj = 0; jj < ROWS_IN_FLIGHT; ++jj) {
    const float* krow = KV + ((size_t)r * sh.k + min(jj, c - 1)) * sh.ldkv;
#pragma unroll
    for (int u = 0; u < MAX_E; ++u) {
      const int e = lane + 64 * u;
      kreg[jj][u] = e < sh.dO ? krow[e] : 0.f;
      vreg[jj][u] = e < sh.dO ? krow[sh.dO + e] : 0.f;
    }
  }
#pragma unroll
  for (int u = 0; u < MAX_E; ++u) {
    const int e = lane + 64 * u;
    if (e < sh.dO) sq[e] = qreg[u];
  }
#pragma unroll
  for (int jj = 0; jj < ROWS_IN_FLIGHT; ++jj) {
    if (jj < c) {
#pragma unroll
      for (int u = 0; u < MAX_E; ++u) {
        const int e = lane + 64 * u;
        if (e < sh.dO) sK[jj * (sh.dO + 1) + e] = kreg[jj][u];
      }
    }
  }
  // key rows beyond the first batch
  for (int j0 = ROWS_IN_FLIGHT; j0 < c; j0 += ROWS_IN_FLIGHT) {
    float k2[ROWS_IN_FLIGHT][MAX_E];
#pragma unroll
    for (int jj = 0; jj < ROWS_IN_FLIGHT; ++jj) {
      const float* krow = KV + ((size_t)r * sh.k + min(j0 + jj, c - 1)) * sh.ldkv;
#pragma unroll
      for (int u = 0; u < MAX_E; ++u) {
        const int e = lane + 64 * u;
        k2[jj][u] = e < sh.dO ? krow[e] : 0.f;
      }
    }
#pragma unroll
    for (int jj = 0; jj < ROWS_IN_FLIGHT; ++jj) {
      if (j0 + jj < c) {
#pragma unroll
        for (int u = 0; u < MAX_E; ++u) {
          const int e = lane + 64 * u;
          if (e < sh.dO) sK[(j0 + jj) * (sh.dO + 1) + e] = k2[jj][u];
        }
      }
    }
  }
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): LDS writes of this wave are visible to all its lanes
  for (int p = lane; p < HK; p += 64) {
    const int h = p / sh.k, j = p - h * sh.k;
    float a = -INFINITY;
    if (j < c) {
      a = 0.f;
      const float* qq = sq + h * sh.dh;
      const float* kk = sK + j * (sh.dO + 1) + h * sh.dh;
      for (int d = 0; d < sh.dh; ++d) a += qq[d] * kk[d];
      a *= scale;
    }
    sa[p] = a;
  }
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_s_waitcnt(0xc07f);
  for (int p = lane; p < HK; p += 64) {
    const int h = p / sh.k, j = p - h * sh.k;
    float v = 0.f;
    if (j < c) {
      float mx = -INFINITY;
      for (int jj = 0; jj < c; ++jj) mx = fmaxf(mx, sa[h * sh.k + jj]);
      float den = 0.f;
      for (int jj = 0; jj < c; ++jj) den += expf(sa[h * sh.k + jj] - mx);
      v = expf(sa[p] - mx) / den;
    }
    sa[HK + p] = v;
    pr[p] = v;
  }
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_s_waitcnt(0xc07f);
  // weighted sums of the value rows: the first batch is in registers
  float o[MAX_E];
#pragma unroll
  for (int u = 0; u < MAX_E; ++u) {
    const int e = lane + 64 * u;
    const int h = min(e, sh.dO - 1) / sh.dh;
    float acc = 0.f;
#pragma unroll
    for (int jj = 0; jj < ROWS_IN_FLIGHT; ++jj)
      if (jj < c) acc += sa[HK + h * sh.k + jj] * vreg[jj][u];
    o[u] = acc;
  }
  for (int j0 = ROWS_IN_FLIGHT; j0 < c; j0 += ROWS_IN_FLIGHT) {
    float v2[ROWS_IN_FLIGHT][MAX_E];
#pragma unroll
    for (int jj = 0; jj < ROWS_IN_FLIGHT; ++jj) {
      const float* vrow = KV + ((size_t)r * sh.k + min(j0 + jj, c - 1)) * sh.ldkv + sh.dO;
#pragma unroll
      for (int u = 0; u < MAX_E; ++u) {
        const int e = lane + 64 * u;
        v2[jj][u] = e < sh.dO ? vrow[e] : 0.f;
      }
    }
#pragma unroll
    for (int u = 0; u < MAX_E; ++u) {
      const int h = min(lane + 64 * u, sh.dO - 1) / sh.dh;
#pragma unroll
      for (int jj = 0; jj < ROWS_IN_FLIGHT; ++jj)
        if (j0 + jj < c) o[u] += sa[HK + h * sh.k + j0 + jj] * v2[jj][u];
    }
  }
#pragma unroll
  for (int u = 0; u < MAX_E; ++u) {
    const int e = lane + 64 * u;
    if (e < sh.dO) out[e] = o[u];
  }
}

template <int MAX_E>
__global__ __launch_bounds__(256) void attn_bwd_kernel(AttnShape sh, const float* __restrict__ q,
                                                       const int32_t* __restrict__ slot_row,
                                                       const float* __restrict__ KV,
                                                       const int32_t* __restrict__ cnt,
                                                       const float* __restrict__ prob,
                                                       const float* __restrict__ dOmat, float* __restrict__ dq,
                                                       float* __restrict__ dKV, float* __restrict__ q_part, AttnSums zs) {
  extern __shared__ float lds[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = blockIdx.x * 4 + wave;
  if (r >= sh.R) return;
  float* sdo = lds + (size_t)wave * attn_lds_floats(sh.k, sh.H, sh.dO);
  float* sV = sdo + sh.dO;
  float* sa = sV + sh.k * (sh.dO + 1);  // [0,HK): prob, [HK,2HK): d(score)
  const int c = cnt[r];
  const size_t qrow = slot_row != nullptr ? (size_t)slot_row[r] : (size_t)r;
  const int HK = sh.H * sh.k;
  // rows of absent neighbours get zero gradients
  for (int j = c; j < sh.k; ++j) {
    float* row = dKV + ((size_t)r * sh.k + j) * sh.ldkv;
    for (int e = lane; e < 2 * sh.dO; e += 64) row[e] = 0.f;
  }
  if (c == 0) {
    for (int e = lane; e < sh.dO; e += 64) dq[(size_t)r * sh.ldo + e] = 0.f;
    if (zs.Zs != nullptr) {
      if (zs.later) {
        for (int p = lane; p < HK; p += 64) zs.ds_out[(size_t)r * HK + p] = 0.f;
      } else {
        for (int i = lane; i < sh.H * zs.dcp; i += 64) zs.Zs[(size_t)r * zs.ldz + i] = zs.Zp[(size_t)r * zs.ldz + i] = 0.f;
      }
      for (int e = lane; e < sh.dO; e += 64) zs.Qroot[(size_t)r * sh.ldo + e] = 0.f;
    }
    return;
  }
  const float scale = 1.0f / sqrtf((float)c);
  // the burst: dO and q rows, the softmax weights, and the key and value rows of the first batch
  float doreg[MAX_E], qreg[MAX_E], kreg[ROWS_IN_FLIGHT][MAX_E], vreg[ROWS_IN_FLIGHT][MAX_E];
#pragma unroll
  for (int u = 0; u < MAX_E; ++u) {
    const int e = lane + 64 * u;
    doreg[u] = e < sh.dO ? dOmat[(size_t)r * sh.ldo + e] : 0.f;
    qreg[u] = e < sh.dO ? q[qrow * sh.ldq + e] : 0.f;
  }
  for (int p = lane; p < HK; p += 64) sa[p] = prob[(size_t)r * HK + p];
#pragma unroll
  for (int jj = 0; jj < ROWS_IN_FLIGHT; ++jj) {
    const float* krow = KV + ((size_t)r * sh.k + min(jj, c - 1)) * sh.ldkv;
#pragma unroll
    for (int u = 0; u < MAX_E; ++u) {
      const int e = lane + 64 * u;
      kreg[jj][u] = e < sh.dO ? krow[e] : 0.f;
      vreg[jj][u] = e < sh.dO ? krow[sh.dO + e] : 0.f;
    }
  }
#pragma unroll
  for (int u = 0; u < MAX_E; ++u) {
    const int e = lane + 64 * u;
    if (e < sh.dO) sdo[e] = doreg[u];
  }
#pragma unroll
  for (int jj = 0; jj < ROWS_IN_FLIGHT; ++jj) {
    if (jj < c) {
#pragma unroll
      for (int u = 0; u < MAX_E; ++u) {
        const int e = lane + 64 * u;
        if (e < sh.dO) sV[jj * (sh.dO + 1) + e] = vreg[jj][u];
      }
    }
  }
  // value rows beyond the first batch
  for (int j0 = ROWS_IN_FLIGHT; j0 < c; j0 += ROWS_IN_FLIGHT) {
    float v2[ROWS_IN_FLIGHT][MAX_E];
#pragma unroll
    for (int jj = 0; jj < ROWS_IN_FLIGHT; ++jj) {
      const float* vrow = KV + ((size_t)r * sh.k + min(j0 + jj, c - 1)) * sh.ldkv + sh.dO;
#pragma unroll
      for (int u = 0; u < MAX_E; ++u) {
        const int e = lane + 64 * u;
        v2[jj][u] = e < sh.dO ? vrow[e] : 0.f;
      }
    }
#pragma unroll
    for (int jj = 0; jj < ROWS_IN_FLIGHT; ++jj) {
      if (j0 + jj < c) {
#pragma unroll
        for (int u = 0; u < MAX_E; ++u) {
          const int e = lane + 64 * u;
          if (e < sh.dO) sV[(j0 + jj) * (sh.dO + 1) + e] = v2[jj][u];
        }
      }
    }
  }
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_s_waitcnt(0xc07f);
  for (int p = lane; p < HK; p += 64) {
    const int h = p / sh.k, j = p - h * sh.k;
    float dp = 0.f;
    if (j < c) {
      const float* dd = sdo + h * sh.dh;
      const float* vv = sV + j * (sh.dO + 1) + h * sh.dh;
      for (int d = 0; d < sh.dh; ++d) dp += dd[d] * vv[d];
    }
    sa[HK + p] = dp;
  }
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_s_waitcnt(0xc07f);
  float da_keep[(TGNN_MAX_HEADS * TGNN_MAX_K + 63) / 64];
  int it = 0;
  for (int p = lane; p < HK; p += 64, ++it) {
    const int h = p / sh.k, j = p - h * sh.k;
    float da = 0.f;
    if (j < c) {
      float sdot = 0.f;
      for (int jj = 0; jj < c; ++jj) sdot += sa[h * sh.k + jj] * sa[HK + h * sh.k + jj];
      da = sa[p] * (sa[HK + p] - sdot) * scale;
    }
    da_keep[it] = da;
  }
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_s_waitcnt(0xc07f);
  it = 0;
  for (int p = lane; p < HK; p += 64, ++it) sa[HK + p] = da_keep[it];
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_s_waitcnt(0xc07f);
  if (zs.Zs != nullptr && zs.later) {
    for (int p = lane; p < HK; p += 64) zs.ds_out[(size_t)r * HK + p] = sa[HK + p];
#pragma unroll
    for (int u = 0; u < MAX_E; ++u) {
      const int e = lane + 64 * u;
      if (e < sh.dO) zs.Qroot[(size_t)r * sh.ldo + e] = qreg[u];
    }
  } else if (zs.Zs != nullptr) {
    // Per head, the sums of the slots' {e | Phi} rows weighted by the score gradients (Zs) and by the softmax
    // weights (Zp): dK_j = ds_j q and dV_j = p_j dO per head, so the weight gradients sum_j dK_j CE_j^T and
    // sum_j dV_j CE_j^T of a root are q Zs^T and dO Zp^T, products over roots instead of over slots.
    for (int c0 = 0; c0 < zs.dcp; c0 += 64) {
      const int cc = c0 + lane;
      float as[TGNN_MAX_HEADS], ap[TGNN_MAX_HEADS];
#pragma unroll
      for (int h = 0; h < TGNN_MAX_HEADS; ++h) as[h] = ap[h] = 0.f;
      for (int j0 = 0; j0 < c; j0 += ROWS_IN_FLIGHT) {
        float ce[ROWS_IN_FLIGHT];
#pragma unroll
        for (int jj = 0; jj < ROWS_IN_FLIGHT; ++jj)
          ce[jj] = (j0 + jj < c && cc < zs.dcols) ? zs.CE[((size_t)r * sh.k + j0 + jj) * zs.ldce + cc] : 0.f;
#pragma unroll
        for (int jj = 0; jj < ROWS_IN_FLIGHT; ++jj) {
          if (j0 + jj < c) {
#pragma unroll
            for (int h = 0; h < TGNN_MAX_HEADS; ++h) {
              if (h < sh.H) {
                as[h] += sa[HK + h * sh.k + j0 + jj] * ce[jj];
                ap[h] += sa[h * sh.k + j0 + jj] * ce[jj];
              }
            }
          }
        }
      }
      if (cc < zs.dcp) {
#pragma unroll
        for (int h = 0; h < TGNN_MAX_HEADS; ++h) {
          if (h < sh.H) {
            zs.Zs[(size_t)r * zs.ldz + h * zs.dcp + cc] = as[h];
            zs.Zp[(size_t)r * zs.ldz + h * zs.dcp + cc] = ap[h];
          }
        }
      }
    }
#pragma unroll
    for (int u = 0; u < MAX_E; ++u) {
      const int e = lane + 64 * u;
      if (e < sh.dO) zs.Qroot[(size_t)r * sh.ldo + e] = qreg[u];
    }
  }
  // dq, and the gradients of the key and value rows: the first batch of key rows is in registers
  float dqe[MAX_E];
#pragma unroll
  for (int u = 0; u < MAX_E; ++u) {
    const int e = lane + 64 * u;
    const int h = min(e, sh.dO - 1) / sh.dh;
    float acc = 0.f;
#pragma unroll
    for (int jj = 0; jj < ROWS_IN_FLIGHT; ++jj) {
      if (jj < c && e < sh.dO) {
        const size_t row = ((size_t)r * sh.k + jj) * sh.ldkv;
        const float da = sa[HK + h * sh.k + jj];
        acc += da * kreg[jj][u];
        dKV[row + e] = da * qreg[u];
        dKV[row + sh.dO + e] = sa[h * sh.k + jj] * doreg[u];
      }
    }
    dqe[u] = acc;
  }
  for (int j0 = ROWS_IN_FLIGHT; j0 < c; j0 += ROWS_IN_FLIGHT) {
    float k2[ROWS_IN_FLIGHT][MAX_E];
#pragma unroll
    for (int jj = 0; jj < ROWS_IN_FLIGHT; ++jj) {
      const float* krow = KV + ((size_t)r * sh.k + min(j0 + jj, c - 1)) * sh.ldkv;
#pragma unroll
      for (int u = 0; u < MAX_E; ++u) {
        const int e = lane + 64 * u;
        k2[jj][u] = e < sh.dO ? krow[e] : 0.f;
      }
    }
#pragma unroll
    for (int u = 0; u < MAX_E; ++u) {
      const int e = lane + 64 * u;
      const int h = min(e, sh.dO - 1) / sh.dh;
#pragma unroll
      for (int jj = 0; jj < ROWS_IN_FLIGHT; ++jj) {
        const int j = j0 + jj;
        if (j < c && e < sh.dO) {
          const size_t row = ((size_t)r * sh.k + j) * sh.ldkv;
          const float da = sa[HK + h * sh.k + j];
          dqe[u] += da * k2[jj][u];
          dKV[row + e] = da * qreg[u];
          dKV[row + sh.dO + e] = sa[h * sh.k + j] * doreg[u];
        }
      }
    }
  }
#pragma unroll
  for (int u = 0; u < MAX_E; ++u) {
    const int e = lane + 64 * u;
    if (e < sh.dO) {
      dq[(size_t)r * sh.ldo + e] = dqe[u];
      // column sums of dq over the roots, spread over QPHI_BLOCKS partial rows to keep the atomics apart
      if (q_part != nullptr) atomicAdd(q_part + (size_t)(blockIdx.x & (QPHI_BLOCKS - 1)) * sh.dO + e, dqe[u]);
    }
  }
}

static AttnShape shape_of(const Dims& d, int R, int ldq, int ldkv, int ldo) {
  return AttnShape{R, d.k, d.H, d.dO, d.dO / d.H, ldq, ldkv, ldo};
}

void attn_core_fwd(const Dims& d, int R, const float* q, int ldq, const int32_t* slot_row, const float* KV, int ldkv,
                   const int32_t* cnt, float* prob, float* Omat, int ldo, hipStream_t s,
                   const SortArgs& fill) {
  if (R <= 0) return;
  const size_t lds = 4 * sizeof(float) * attn_lds_floats(d.k, d.H, d.dO);
  const int fill_blocks = fill.ucnt != nullptr ? (fill.S + 255) / 256 : 0;
  if (d.dO <= 128)
    hipLaunchKernelGGL(attn_fwd_kernel<2>, dim3((R + 3) / 4 + fill_blocks), dim3(256), lds, s, shape_of(d, R, ldq, ldkv, ldo),
                       q, slot_row, KV, cnt, prob, Omat, fill);
  else
    hipLaunchKernelGGL(attn_fwd_kernel<4>, dim3((R + 3) / 4 + fill_blocks), dim3(256), lds, s, shape_of(d, R, ldq, ldkv, ldo),
                       q, slot_row, KV, cnt, prob, Omat, fill);
}

// dq and dOmat share the pitch ldo
void attn_core_bwd(const Dims& d, int R, const float* q, int ldq, const int32_t* slot_row, const float* KV, int ldkv,
                   const int32_t* cnt, const float* prob, const float* dOmat, int ldo, float* dq, float* dKV,
                   float* q_part, hipStream_t s, const AttnSums& zs) {
  if (R <= 0) return;
  const size_t lds = 4 * sizeof(float) * attn_lds_floats(d.k, d.H, d.dO);
  if (d.dO <= 128)
    hipLaunchKernelGGL(attn_bwd_kernel<2>, dim3((R + 3) / 4), dim3(256), lds, s, shape_of(d, R, ldq, ldkv, ldo), q, slot_row,
                       KV, cnt, prob, dOmat, dq, dKV, q_part, zs);
  else
    hipLaunchKernelGGL(attn_bwd_kernel<4>, dim3((R + 3) / 4), dim3(256), lds, s, shape_of(d, R, ldq, ldkv, ldo), q, slot_row,
                       KV, cnt, prob, dOmat, dq, dKV, q_part, zs);
}

}  // namespace tgnn
