// Temporal attention over the k sampled neighbours of one root (Eq. 4-7), forward and backward, without ever
// forming a key or value row.
//
// A neighbour slot's key is K_j = Pk[w_j] + W_k^c c_j with c_j = {e_vw | Phi(dt_j)} the slot's own input and
// Pk[w_j] the projection of the neighbour node's row {s' | static} (taken once per distinct node by an MFMA
// GEMM).  A head's score is therefore
//     q_h . K_jh = q_h . Pk_h[w_j] + u_h . c_j            with u_h = (W_k^c)_h^T q_h   (per node row: U, one GEMM)
// and its output
//     sum_j p_jh V_jh = sum_j p_jh Pv_h[w_j] + (W_v^c)_h zp_h     with zp_h = sum_j p_jh c_j   (Zp; one GEMM over roots)
// so the per-slot work is two short dot products and two weighted sums of c_j, done here on the vector ALUs, one
// wavefront per root, with c_j put together in registers: the edge-feature row is gathered straight from the
// table and the time encoding is evaluated in place.  Nothing of size (slots x width) goes to memory.
// The backward pass has the same shape: with g_h = (W_v^c)_h^T dO_h (G, one GEMM over roots)
//     dp_jh = dO_h . Pv_h[w_j] + g_h . c_j,   ds_jh = p_jh (dp_jh - sum_j p_jh dp_jh) / sqrt(|N_v|)
//     dq_h = sum_j ds_jh Pk_h[w_j] + (W_k^c)_h zs_h            with zs_h = sum_j ds_jh c_j   (Zs; one GEMM over roots)
// the weight gradients of W_k^c, W_v^c are products over roots of q, dO with Zs, Zp, the gradient reaching the key's
// time encoding is d Phi_j = sum_h ds_jh u_h + p_jh g_h (time columns), reduced per root against -sin(.) here (Y)
// and over the roots by the weight-gradient launch, and the gradients of the neighbour rows' projections are
// dK_j = ds_j q, dV_j = p_j dO, formed where they are summed per node row.
#include "tgnn_internal.h"
#include "device_math.h"
#include "unique_device.h"

namespace tgnn {

// LDS floats per wavefront: softmax weights and score gradients
__host__ __device__ inline int fattn_lds_floats(int k, int H) { return 2 * H * k; }

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
  return x;
}

__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0): this wavefront's LDS writes are visible to all its lanes
  __builtin_amdgcn_wave_barrier();
}

// slot (r, j): edge-feature row index, node row, time difference of Eq. 5-6
__device__ __forceinline__ void slot_ids(const FusedAttn& a, int r, int j, int c, int& e, int& row, double& dt,
                                         bool forward) {
  e = -1; row = 0; dt = 0.0;
  const int s = r * a.k + j;
  if (j < c) {
    e = a.neid != nullptr ? a.neid[s] : s;
    row = a.slot_row != nullptr ? a.slot_row[a.R + s] : a.R + s;
    if (!forward) dt = a.dtk[s];
    else if (a.dt_in != nullptr) dt = a.dt_in[s];
    else if (a.dt_source != 0) dt = a.root_t[r] - a.nts[s];
    else dt = a.root_t[r] - a.tau[row];
  }
}

// ---------------------------------------------------------------------------------------------------------
// Fast path: k <= KR neighbours, d_e <= 64 NE and d_t <= 64 NT columns, d_o <= 128, at most two heads.  A lane
// owns edge-feature columns lane + 64 m and time columns lane + 64 m of every slot; everything a root needs is
// asked for in one burst after the index loads (a wavefront has few others on its SIMD to hide behind).
// ---------------------------------------------------------------------------------------------------------
constexpr int FA_KR = 10, FA_NE = 3, FA_NT = 2, FA_HM = 2, FA_E = 2;

struct SlotRegs {
  float ce[FA_KR][FA_NE];   // edge-feature columns
  float ct[FA_KR][FA_NT];   // time-encoding columns (cos)
  float pk[FA_KR][FA_E];    // node part of the key
  float pv[FA_KR][FA_E];    // node part of the value
};

// the loads of every slot's edge-feature columns and node rows
__device__ __forceinline__ void fast_issue_slots(const FusedAttn& a, int lane, int c, const int (&e_j)[FA_KR],
                                                 const int (&row_j)[FA_KR], SlotRegs& s) {
  // Column offsets are clamped into the row instead of guarded (no per-lane branch around a load).  What a lane
  // beyond the row's width reads that way (a copy of the row's last column) is NOT replaced by zero: everything a
  // slot column is multiplied with (the per-head rows from load_head_row, the head-masked query and output-gradient
  // rows) is zero on those lanes, and every sum that keeps slot columns is stored under a width guard.  Absent slots
  // (j >= c, uniform over the wavefront) are skipped and stay zero.
  int ecol[FA_NE], pcol[FA_E];
#pragma unroll
  for (int m = 0; m < FA_NE; ++m) ecol[m] = min(lane + 64 * m, max(a.de - 1, 0));
#pragma unroll
  for (int u = 0; u < FA_E; ++u) pcol[u] = min(lane + 64 * u, a.dO - 1);
#pragma unroll
  for (int j = 0; j < FA_KR; ++j) {
#pragma unroll
    for (int m = 0; m < FA_NE; ++m) s.ce[j][m] = 0.f;
#pragma unroll
    for (int u = 0; u < FA_E; ++u) s.pk[j][u] = s.pv[j][u] = 0.f;
    if (j < c) {
      if (a.de > 0) {
        const float* erow = a.efeat + (size_t)e_j[j] * a.de;
#pragma unroll
        for (int m = 0; m < FA_NE; ++m) s.ce[j][m] = erow[ecol[m]];
      }
      const float* prow = a.P + (size_t)row_j[j] * a.ldp;
#pragma unroll
      for (int u = 0; u < FA_E; ++u) {
        s.pk[j][u] = prow[pcol[u]];
        s.pv[j][u] = prow[a.dO + pcol[u]];
      }
    }
  }
}

// which head a lane's output columns lane + 64 u belong to: 1.0 where it is head hh, else 0 (0 beyond d_o)
__device__ __forceinline__ void head_masks(const FusedAttn& a, int lane, float (&mh)[FA_HM][FA_E]) {
#pragma unroll
  for (int u = 0; u < FA_E; ++u) {
    const int e = lane + 64 * u;
    const int h = e / a.dh;   // (two divisions per wavefront, not one per slot and head)
#pragma unroll
    for (int hh = 0; hh < FA_HM; ++hh) mh[hh][u] = (e < a.dO && h == hh) ? 1.f : 0.f;
  }
}

// time encoding of every slot, evaluated in place (Eq. 5-6); the backward pass also needs the sine
template <bool BWD>
__device__ __forceinline__ void fast_time_cols(const FusedAttn& a, int lane, int c, const double (&dt_j)[FA_KR],
                                               SlotRegs& s, float (&st)[FA_KR][FA_NT]) {
#pragma unroll
  for (int m = 0; m < FA_NT; ++m) {
    const int tc = lane + 64 * m;
    const bool live = tc < a.dt;
    const double w = live ? (double)a.time_w[tc] : 0.0, b = live ? (double)a.time_b[tc] : 0.0;
#pragma unroll
    for (int j = 0; j < FA_KR; ++j) {
      float sn = 0.f, cs = 0.f;
      if (j < c)     // (uniform over the wavefront; lanes beyond d_t compute on w = b = 0, see fast_issue_slots)
        sincos_reduced(fma(w, dt_j[j], b), sn, cs);
      s.ct[j][m] = cs;
      if (BWD) st[j][m] = sn;
    }
  }
}

template <bool BWD>
__device__ __forceinline__ void fast_load_slots(const FusedAttn& a, int lane, int c, const int (&e_j)[FA_KR],
                                                const int (&row_j)[FA_KR], const double (&dt_j)[FA_KR], SlotRegs& s,
                                                float (&st)[FA_KR][FA_NT]) {
  fast_issue_slots(a, lane, c, e_j, row_j, s);
  fast_time_cols<BWD>(a, lane, c, dt_j, s, st);
}

// the per-head rows u_h (or g_h): edge-feature and time columns of head h's block of a row of pitch ldz
struct HeadRow {
  float e[FA_HM][FA_NE], t[FA_HM][FA_NT];
};
__device__ __forceinline__ void load_head_row(const FusedAttn& a, const float* row, int lane, HeadRow& h) {
  // (clamped column offsets instead of per-lane guards around the loads; a head beyond H is uniform)
#pragma unroll
  for (int hh = 0; hh < FA_HM; ++hh) {
    const float* blk = row + hh * a.dcp;
#pragma unroll
    for (int m = 0; m < FA_NE; ++m) {
      const int col = lane + 64 * m;
      float v = 0.f;
      if (hh < a.H && a.de > 0) v = blk[min(col, a.de - 1)];
      h.e[hh][m] = col < a.de ? v : 0.f;
    }
#pragma unroll
    for (int m = 0; m < FA_NT; ++m) {
      const int tc = lane + 64 * m;
      float v = 0.f;
      if (hh < a.H) v = blk[a.de + min(tc, a.dt - 1)];
      h.t[hh][m] = tc < a.dt ? v : 0.f;
    }
  }
}

// store a root's per-head sums (Zp or Zs): head h's block holds d_e + d_t values, padded with zeros to dcp
__device__ __forceinline__ void store_head_row(const FusedAttn& a, float* row, int lane, const HeadRow& h) {
  const int pad = a.dcp - a.de - a.dt;
#pragma unroll
  for (int hh = 0; hh < FA_HM; ++hh) {
    if (hh >= a.H) break;
    float* blk = row + hh * a.dcp;
#pragma unroll
    for (int m = 0; m < FA_NE; ++m) {
      const int col = lane + 64 * m;
      if (col < a.de) blk[col] = h.e[hh][m];
    }
#pragma unroll
    for (int m = 0; m < FA_NT; ++m) {
      const int tc = lane + 64 * m;
      if (tc < a.dt + pad) blk[a.de + tc] = tc < a.dt ? h.t[hh][m] : 0.f;
    }
  }
}

__device__ __forceinline__ void zero_head_rows(const FusedAttn& a, float* row, int lane) {
  for (int i = lane; i < a.H * a.dcp; i += 64) row[i] = 0.f;
}

// per-head softmax over the c valid scores in sa[0 .. HK): weights to sa[HK ..) and to prob
__device__ __forceinline__ void softmax_heads(float* sa, int HK, int k, int c, int lane, float* pr) {
  for (int p = lane; p < HK; p += 64) {
    const int h = p / k, j = p - h * k;
    float v = 0.f;
    if (j < c) {
      float mx = -INFINITY;
      for (int jj = 0; jj < c; ++jj) mx = fmaxf(mx, sa[h * k + jj]);
      float den = 0.f;
      for (int jj = 0; jj < c; ++jj) den += expf(sa[h * k + jj] - mx);
      v = expf(sa[p] - mx) / den;
    }
    sa[HK + p] = v;
    pr[p] = v;
  }
}

// Wavefronts per SIMD the forward kernel is compiled for.  It needs 124 registers once the wave index and the
// neighbour count are kept scalar, so four fit without a spill (with the count in a vector register it spilled nine
// registers at four and measured 4 to 19 % slower than at three; at four without the spill it is another 6 % faster
// on 12,000 roots).
#ifndef TGNN_FATTN_FWD_WAVES
#define TGNN_FATTN_FWD_WAVES 4
#endif
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(TGNN_FATTN_FWD_WAVES, TGNN_FATTN_FWD_WAVES))) void fattn_fwd_fast_kernel(FusedAttn a) {
  extern __shared__ float lds[];
  int block = blockIdx.x;
  if (a.fill.ucnt != nullptr) {   // the first blocks are passengers: the fill pass of the slot sort
    const int fill_blocks = uniq_blocks(a.fill.S);
    if (block < fill_blocks) {
      uniq_fill_block(a.fill, block);
      return;
    }
    block -= fill_blocks;
  }
  // (wave index and neighbour count are the same for all lanes: saying so keeps them, and every test on them, scalar)
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int r = block * 4 + wave;
  if (r >= a.R) return;
  const int HK = a.H * a.k;
  float* sa = lds + (size_t)wave * fattn_lds_floats(a.k, a.H);   // [0, HK): scores, [HK, 2 HK): softmax weights
  const int c = __builtin_amdgcn_readfirstlane(a.cnt[r]);
  float* pr = a.prob + (size_t)r * HK;
  float* out = a.Onode + (size_t)r * a.ldh;
  // Round trip 1 (issued together with the count above, none depends on another): this lane's slot ids, the root's
  // node row and query time.  Padding slots carry -1 in both index arrays.
  const int sl = r * a.k + min(lane, a.k - 1);
  int my_e = a.neid != nullptr ? a.neid[sl] : sl;
  int my_row = a.slot_row != nullptr ? a.slot_row[a.R + sl] : a.R + sl;
  const int my_qrow = a.slot_row != nullptr ? a.slot_row[r] : r;
  double my_dt = 0.0;
  const bool from_tau = a.dt_in == nullptr && a.dt_source == 0;
  if (a.dt_in != nullptr) my_dt = a.dt_in[sl];
  else if (a.dt_source != 0) my_dt = a.root_t[r] - a.nts[sl];
  else my_dt = a.root_t[r];
  const bool own = lane < a.k && lane < c;
  if (!own) { my_e = -1; my_row = 0; }
  if (c == 0) {
    if (lane < a.k) a.dtk[(size_t)r * a.k + lane] = 0.0;
    for (int p = lane; p < HK; p += 64) pr[p] = 0.f;
    for (int e = lane; e < a.dO; e += 64) out[e] = 0.f;
    zero_head_rows(a, a.Zp + (size_t)r * a.ldz, lane);
    return;
  }
  // Round trip 2: the update time of the neighbour's memory (Eq. 5-6: the time difference is taken against it),
  // asked for first, and behind it the burst of everything else the root needs
  double my_tau = 0.0;
  if (from_tau && own) my_tau = a.tau[my_row];
  const size_t qrow = (size_t)my_qrow;
  const float scale = 1.0f / sqrtf((float)c);
  int e_j[FA_KR], row_j[FA_KR];
#pragma unroll
  for (int j = 0; j < FA_KR; ++j) {
    // (readlane: one value for the whole wavefront, kept in scalar registers)
    e_j[j] = __builtin_amdgcn_readlane(my_e, j);
    row_j[j] = __builtin_amdgcn_readlane(my_row, j);
  }
  // the burst: the root's query and u rows, then every slot's columns
  float qreg[FA_E];
#pragma unroll
  for (int u = 0; u < FA_E; ++u) {
    const int e = lane + 64 * u;
    qreg[u] = e < a.dO ? a.P[qrow * a.ldp + a.off_q + e] : 0.f;
  }
  HeadRow ur;
  load_head_row(a, a.U + qrow * a.ldz, lane, ur);
  SlotRegs s;
  fast_issue_slots(a, lane, c, e_j, row_j, s);
  // the time differences, once the update times are in
  if (from_tau) my_dt -= my_tau;
  if (!own) my_dt = 0.0;
  if (lane < a.k) a.dtk[(size_t)r * a.k + lane] = my_dt;
  double dt_j[FA_KR];
#pragma unroll
  for (int j = 0; j < FA_KR; ++j)
    dt_j[j] = __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(my_dt), j),
                               __builtin_amdgcn_readlane(__double2loint(my_dt), j));
  float unused[FA_KR][FA_NT];
  fast_time_cols<false>(a, lane, c, dt_j, s, unused);
  // scores (Eq. 7): per slot and head, this lane's share of q . Pk + u . c, summed over the wavefront
  float mh[FA_HM][FA_E], qh[FA_HM][FA_E];
  head_masks(a, lane, mh);
#pragma unroll
  for (int hh = 0; hh < FA_HM; ++hh)
#pragma unroll
    for (int u = 0; u < FA_E; ++u) qh[hh][u] = mh[hh][u] * qreg[u];
  float part[FA_KR][FA_HM];
#pragma unroll
  for (int j = 0; j < FA_KR; ++j) {
#pragma unroll
    for (int hh = 0; hh < FA_HM; ++hh) {
      float acc = 0.f;
#pragma unroll
      for (int m = 0; m < FA_NE; ++m) acc += ur.e[hh][m] * s.ce[j][m];
#pragma unroll
      for (int m = 0; m < FA_NT; ++m) acc += ur.t[hh][m] * s.ct[j][m];
#pragma unroll
      for (int u = 0; u < FA_E; ++u) acc += qh[hh][u] * s.pk[j][u];
      part[j][hh] = acc;
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1)
#pragma unroll
    for (int j = 0; j < FA_KR; ++j)
#pragma unroll
      for (int hh = 0; hh < FA_HM; ++hh) part[j][hh] += __shfl_xor(part[j][hh], o);
  float mine = -INFINITY;
#pragma unroll
  for (int j = 0; j < FA_KR; ++j)
#pragma unroll
    for (int hh = 0; hh < FA_HM; ++hh)
      if (lane == hh * a.k + j && j < c && hh < a.H) mine = part[j][hh] * scale;
  if (lane < HK) sa[lane] = mine;
  wave_lds_sync();
  softmax_heads(sa, HK, a.k, c, lane, pr);
  wave_lds_sync();
  // weighted sums: node part of the output, and the per-head sums of the slots' own inputs
  float o[FA_E] = {0.f, 0.f};
  HeadRow zp;
#pragma unroll
  for (int hh = 0; hh < FA_HM; ++hh) {
#pragma unroll
    for (int m = 0; m < FA_NE; ++m) zp.e[hh][m] = 0.f;
#pragma unroll
    for (int m = 0; m < FA_NT; ++m) zp.t[hh][m] = 0.f;
  }
#pragma unroll
  for (int j = 0; j < FA_KR; ++j) {   // (slots j >= c hold zeros and zero weights: no branch, the loop stays unrolled)
    float pj[FA_HM];
#pragma unroll
    for (int hh = 0; hh < FA_HM; ++hh) pj[hh] = (hh < a.H && j < a.k) ? sa[HK + hh * a.k + j] : 0.f;
#pragma unroll
    for (int u = 0; u < FA_E; ++u) o[u] += (mh[0][u] * pj[0] + mh[FA_HM - 1][u] * pj[FA_HM - 1]) * s.pv[j][u];
#pragma unroll
    for (int hh = 0; hh < FA_HM; ++hh) {
#pragma unroll
      for (int m = 0; m < FA_NE; ++m) zp.e[hh][m] += pj[hh] * s.ce[j][m];
#pragma unroll
      for (int m = 0; m < FA_NT; ++m) zp.t[hh][m] += pj[hh] * s.ct[j][m];
    }
  }
#pragma unroll
  for (int u = 0; u < FA_E; ++u) {
    const int e = lane + 64 * u;
    if (e < a.dO) out[e] = o[u];
  }
  store_head_row(a, a.Zp + (size_t)r * a.ldz, lane, zp);
}

#ifdef TGNN_FATTN_BWD_WAVES
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(TGNN_FATTN_BWD_WAVES, TGNN_FATTN_BWD_WAVES))) void fattn_bwd_fast_kernel(FusedAttn a) {
#else
__global__ __launch_bounds__(256) void fattn_bwd_fast_kernel(FusedAttn a) {
#endif
  extern __shared__ float lds[];
  // (wave index and neighbour count are the same for all lanes: saying so keeps them, and every test on them, scalar)
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int r = blockIdx.x * 4 + wave;
  if (r >= a.R) return;
  const int HK = a.H * a.k;
  float* sa = lds + (size_t)wave * fattn_lds_floats(a.k, a.H);   // [0, HK): softmax weights, [HK, 2 HK): dp, then ds
  const int c = __builtin_amdgcn_readfirstlane(a.cnt[r]);
  float* yrow = a.Y + (size_t)r * a.ldy;
  if (c == 0) {
    for (int p = lane; p < HK; p += 64) a.dscore[(size_t)r * HK + p] = 0.f;
    for (int e = lane; e < a.dO; e += 64) a.dqn[(size_t)r * a.ldh + e] = a.Qroot[(size_t)r * a.ldh + e] = 0.f;
    zero_head_rows(a, a.Zs + (size_t)r * a.ldz, lane);
    for (int i = lane; i < 2 * a.dt; i += 64) yrow[i] = 0.f;
    return;
  }
  int my_e, my_row;
  double my_dt;
  slot_ids(a, r, min(lane, a.k - 1), lane < a.k ? c : 0, my_e, my_row, my_dt, false);
  const size_t qrow = a.slot_row != nullptr ? (size_t)a.slot_row[r] : (size_t)r;
  const float scale = 1.0f / sqrtf((float)c);
  int e_j[FA_KR], row_j[FA_KR];
  double dt_j[FA_KR];
#pragma unroll
  for (int j = 0; j < FA_KR; ++j) {
    // (readlane: one value for the whole wavefront, kept in scalar registers)
    e_j[j] = __builtin_amdgcn_readlane(my_e, j);
    row_j[j] = __builtin_amdgcn_readlane(my_row, j);
    dt_j[j] = __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(my_dt), j),
                               __builtin_amdgcn_readlane(__double2loint(my_dt), j));
  }
  float qreg[FA_E], doreg[FA_E];
#pragma unroll
  for (int u = 0; u < FA_E; ++u) {
    const int e = lane + 64 * u;
    qreg[u] = e < a.dO ? a.P[qrow * a.ldp + a.off_q + e] : 0.f;
    doreg[u] = e < a.dO ? a.dOmat[(size_t)r * a.ldh + e] : 0.f;
  }
  if (lane < HK) sa[lane] = a.prob[(size_t)r * HK + lane];
  HeadRow ur, gr;
  load_head_row(a, a.U + qrow * a.ldz, lane, ur);
  load_head_row(a, a.G + (size_t)r * a.ldz, lane, gr);
  SlotRegs s;
  float st[FA_KR][FA_NT];
  fast_load_slots<true>(a, lane, c, e_j, row_j, dt_j, s, st);
  // dp_jh = dO_h . V_jh = dO_h . Pv_h[w_j] + g_h . c_j
  float mh[FA_HM][FA_E], doh[FA_HM][FA_E];
  head_masks(a, lane, mh);
#pragma unroll
  for (int hh = 0; hh < FA_HM; ++hh)
#pragma unroll
    for (int u = 0; u < FA_E; ++u) doh[hh][u] = mh[hh][u] * doreg[u];
  float part[FA_KR][FA_HM];
#pragma unroll
  for (int j = 0; j < FA_KR; ++j) {
#pragma unroll
    for (int hh = 0; hh < FA_HM; ++hh) {
      float acc = 0.f;
#pragma unroll
      for (int m = 0; m < FA_NE; ++m) acc += gr.e[hh][m] * s.ce[j][m];
#pragma unroll
      for (int m = 0; m < FA_NT; ++m) acc += gr.t[hh][m] * s.ct[j][m];
#pragma unroll
      for (int u = 0; u < FA_E; ++u) acc += doh[hh][u] * s.pv[j][u];
      part[j][hh] = acc;
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1)
#pragma unroll
    for (int j = 0; j < FA_KR; ++j)
#pragma unroll
      for (int hh = 0; hh < FA_HM; ++hh) part[j][hh] += __shfl_xor(part[j][hh], o);
  float dp = 0.f;
#pragma unroll
  for (int j = 0; j < FA_KR; ++j)
#pragma unroll
    for (int hh = 0; hh < FA_HM; ++hh)
      if (lane == hh * a.k + j && j < c && hh < a.H) dp = part[j][hh];
  if (lane < HK) sa[HK + lane] = dp;
  wave_lds_sync();
  float da = 0.f;
  if (lane < HK) {   // softmax backward, scaled by 1 / sqrt(|N_v|)
    const int h = lane / a.k, j = lane - h * a.k;
    if (j < c) {
      float sdot = 0.f;
      for (int jj = 0; jj < c; ++jj) sdot += sa[h * a.k + jj] * sa[HK + h * a.k + jj];
      da = sa[lane] * (sa[HK + lane] - sdot) * scale;
    }
  }
  wave_lds_sync();
  if (lane < HK) {
    sa[HK + lane] = da;
    a.dscore[(size_t)r * HK + lane] = da;
  }
  wave_lds_sync();
  // per-root sums: dq (node part), Zs, and the time-encoding gradient against -sin(.)
  float dq[FA_E] = {0.f, 0.f};
  HeadRow zs;
  float yw[FA_NT], yb[FA_NT];
#pragma unroll
  for (int hh = 0; hh < FA_HM; ++hh) {
#pragma unroll
    for (int m = 0; m < FA_NE; ++m) zs.e[hh][m] = 0.f;
#pragma unroll
    for (int m = 0; m < FA_NT; ++m) zs.t[hh][m] = 0.f;
  }
#pragma unroll
  for (int m = 0; m < FA_NT; ++m) yw[m] = yb[m] = 0.f;
#pragma unroll
  for (int j = 0; j < FA_KR; ++j) {   // (slots j >= c hold zeros and zero weights: no branch, the loop stays unrolled)
    float dsj[FA_HM], pj[FA_HM];
#pragma unroll
    for (int hh = 0; hh < FA_HM; ++hh) {
      dsj[hh] = (hh < a.H && j < a.k) ? sa[HK + hh * a.k + j] : 0.f;
      pj[hh] = (hh < a.H && j < a.k) ? sa[hh * a.k + j] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < FA_E; ++u) dq[u] += (mh[0][u] * dsj[0] + mh[FA_HM - 1][u] * dsj[FA_HM - 1]) * s.pk[j][u];
    const float dtf = (float)dt_j[j];
#pragma unroll
    for (int hh = 0; hh < FA_HM; ++hh) {
#pragma unroll
      for (int m = 0; m < FA_NE; ++m) zs.e[hh][m] += dsj[hh] * s.ce[j][m];
#pragma unroll
      for (int m = 0; m < FA_NT; ++m) zs.t[hh][m] += dsj[hh] * s.ct[j][m];
    }
#pragma unroll
    for (int m = 0; m < FA_NT; ++m) {
      float dphi = 0.f;
#pragma unroll
      for (int hh = 0; hh < FA_HM; ++hh) dphi += dsj[hh] * ur.t[hh][m] + pj[hh] * gr.t[hh][m];
      const float t = -dphi * st[j][m];
      yb[m] += t;
      yw[m] += t * dtf;
    }
  }
#pragma unroll
  for (int u = 0; u < FA_E; ++u) {
    const int e = lane + 64 * u;
    if (e < a.dO) {
      a.dqn[(size_t)r * a.ldh + e] = dq[u];
      a.Qroot[(size_t)r * a.ldh + e] = qreg[u];
    }
  }
  store_head_row(a, a.Zs + (size_t)r * a.ldz, lane, zs);
#pragma unroll
  for (int m = 0; m < FA_NT; ++m) {
    const int tc = lane + 64 * m;
    if (tc < a.dt) {
      yrow[tc] = yw[m];
      yrow[a.dt + tc] = yb[m];
    }
  }
}

// ---------------------------------------------------------------------------------------------------------
// Generic path: any k <= TGNN_MAX_K, any widths, any number of heads.  Same arithmetic with plain loops: a
// slot's columns are recomputed wherever they are needed instead of being kept in registers.
// ---------------------------------------------------------------------------------------------------------
// column `col` < d_e + d_t of slot input c_j; sn receives the sine of a time column (0 for an edge-feature column)
__device__ __forceinline__ float slot_col(const FusedAttn& a, int e, double dt, int col, float& sn) {
  sn = 0.f;
  if (col < a.de) return a.efeat[(size_t)e * a.de + col];
  float cs;
  const int tc = col - a.de;
  sincos_reduced(fma((double)a.time_w[tc], dt, (double)a.time_b[tc]), sn, cs);
  return cs;
}

// per-wavefront LDS of the generic kernels: [0, HK) and [HK, 2 HK) as in the fast ones, then k slot ids, node rows
// and time differences
__host__ __device__ inline int gattn_lds_bytes(int k, int H) { return 2 * H * k * 4 + k * (4 + 4 + 8) + 8; }

struct GenLds {
  float* sa;
  int *e, *row;
  double* dt;
};
__device__ __forceinline__ GenLds gen_lds(char* base, int wave, int k, int H) {
  char* p = base + (size_t)wave * gattn_lds_bytes(k, H);
  GenLds g;
  g.dt = reinterpret_cast<double*>(p);              // 8-byte aligned: the per-wave size is a multiple of 8
  g.sa = reinterpret_cast<float*>(p + 8 * k);
  g.e = reinterpret_cast<int*>(p + 8 * k + 8 * H * k);
  g.row = g.e + k;
  return g;
}

__global__ __launch_bounds__(256) void fattn_fwd_gen_kernel(FusedAttn a) {
  extern __shared__ __attribute__((aligned(16))) char lds_raw[];
  int block = blockIdx.x;
  if (a.fill.ucnt != nullptr) {
    const int fill_blocks = uniq_blocks(a.fill.S);
    if (block < fill_blocks) {
      uniq_fill_block(a.fill, block);
      return;
    }
    block -= fill_blocks;
  }
  // (wave index and neighbour count are the same for all lanes: saying so keeps them, and every test on them, scalar)
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int r = block * 4 + wave;
  if (r >= a.R) return;
  const int HK = a.H * a.k, dc = a.de + a.dt;
  GenLds L = gen_lds(lds_raw, wave, a.k, a.H);
  const int c = __builtin_amdgcn_readfirstlane(a.cnt[r]);
  float* pr = a.prob + (size_t)r * HK;
  float* out = a.Onode + (size_t)r * a.ldh;
  for (int j = lane; j < a.k; j += 64) {
    int e, row;
    double dt;
    slot_ids(a, r, j, c, e, row, dt, true);
    L.e[j] = e; L.row[j] = row; L.dt[j] = dt;
    a.dtk[(size_t)r * a.k + j] = dt;
  }
  if (c == 0) {
    for (int p = lane; p < HK; p += 64) pr[p] = 0.f;
    for (int e = lane; e < a.dO; e += 64) out[e] = 0.f;
    zero_head_rows(a, a.Zp + (size_t)r * a.ldz, lane);
    return;
  }
  wave_lds_sync();
  const size_t qrow = a.slot_row != nullptr ? (size_t)a.slot_row[r] : (size_t)r;
  const float* qv = a.P + qrow * a.ldp + a.off_q;
  const float* urow = a.U + qrow * a.ldz;
  const float scale = 1.0f / sqrtf((float)c);
  for (int j = 0; j < c; ++j) {
    const float* prow = a.P + (size_t)L.row[j] * a.ldp;
    for (int h = 0; h < a.H; ++h) {
      float acc = 0.f;
      for (int col = lane; col < dc; col += 64) {
        float sn;
        acc += urow[h * a.dcp + col] * slot_col(a, L.e[j], L.dt[j], col, sn);
      }
      for (int e = h * a.dh + lane; e < (h + 1) * a.dh; e += 64) acc += qv[e] * prow[e];
      acc = wave_sum(acc);
      if (lane == 0) L.sa[h * a.k + j] = acc * scale;
    }
  }
  wave_lds_sync();
  softmax_heads(L.sa, HK, a.k, c, lane, pr);
  wave_lds_sync();
  for (int e = lane; e < a.dO; e += 64) {
    const int h = e / a.dh;
    float acc = 0.f;
    for (int j = 0; j < c; ++j) acc += L.sa[HK + h * a.k + j] * a.P[(size_t)L.row[j] * a.ldp + a.dO + e];
    out[e] = acc;
  }
  float* zrow = a.Zp + (size_t)r * a.ldz;
  for (int col = lane; col < a.dcp; col += 64) {
    float acc[TGNN_MAX_HEADS];
#pragma unroll
    for (int h = 0; h < TGNN_MAX_HEADS; ++h) acc[h] = 0.f;
    if (col < dc) {
      for (int j = 0; j < c; ++j) {
        float sn;
        const float cv = slot_col(a, L.e[j], L.dt[j], col, sn);
#pragma unroll
        for (int h = 0; h < TGNN_MAX_HEADS; ++h)
          if (h < a.H) acc[h] += L.sa[HK + h * a.k + j] * cv;
      }
    }
#pragma unroll
    for (int h = 0; h < TGNN_MAX_HEADS; ++h)
      if (h < a.H) zrow[h * a.dcp + col] = acc[h];
  }
}

__global__ __launch_bounds__(256) void fattn_bwd_gen_kernel(FusedAttn a) {
  extern __shared__ __attribute__((aligned(16))) char lds_raw[];
  // (wave index and neighbour count are the same for all lanes: saying so keeps them, and every test on them, scalar)
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int r = blockIdx.x * 4 + wave;
  if (r >= a.R) return;
  const int HK = a.H * a.k, dc = a.de + a.dt;
  GenLds L = gen_lds(lds_raw, wave, a.k, a.H);
  const int c = __builtin_amdgcn_readfirstlane(a.cnt[r]);
  float* yrow = a.Y + (size_t)r * a.ldy;
  if (c == 0) {
    for (int p = lane; p < HK; p += 64) a.dscore[(size_t)r * HK + p] = 0.f;
    for (int e = lane; e < a.dO; e += 64) a.dqn[(size_t)r * a.ldh + e] = a.Qroot[(size_t)r * a.ldh + e] = 0.f;
    zero_head_rows(a, a.Zs + (size_t)r * a.ldz, lane);
    for (int i = lane; i < 2 * a.dt; i += 64) yrow[i] = 0.f;
    return;
  }
  for (int j = lane; j < a.k; j += 64) {
    int e, row;
    double dt;
    slot_ids(a, r, j, c, e, row, dt, false);
    L.e[j] = e; L.row[j] = row; L.dt[j] = dt;
  }
  for (int p = lane; p < HK; p += 64) L.sa[p] = a.prob[(size_t)r * HK + p];
  wave_lds_sync();
  const size_t qrow = a.slot_row != nullptr ? (size_t)a.slot_row[r] : (size_t)r;
  const float* qv = a.P + qrow * a.ldp + a.off_q;
  const float* urow = a.U + qrow * a.ldz;
  const float* grow = a.G + (size_t)r * a.ldz;
  const float* dov = a.dOmat + (size_t)r * a.ldh;
  const float scale = 1.0f / sqrtf((float)c);
  for (int j = 0; j < c; ++j) {
    const float* prow = a.P + (size_t)L.row[j] * a.ldp + a.dO;
    for (int h = 0; h < a.H; ++h) {
      float acc = 0.f;
      for (int col = lane; col < dc; col += 64) {
        float sn;
        acc += grow[h * a.dcp + col] * slot_col(a, L.e[j], L.dt[j], col, sn);
      }
      for (int e = h * a.dh + lane; e < (h + 1) * a.dh; e += 64) acc += dov[e] * prow[e];
      acc = wave_sum(acc);
      if (lane == 0) L.sa[HK + h * a.k + j] = acc;
    }
  }
  wave_lds_sync();
  float da_keep[(TGNN_MAX_HEADS * TGNN_MAX_K + 63) / 64];
  int it = 0;
  for (int p = lane; p < HK; p += 64, ++it) {
    const int h = p / a.k, j = p - h * a.k;
    float da = 0.f;
    if (j < c) {
      float sdot = 0.f;
      for (int jj = 0; jj < c; ++jj) sdot += L.sa[h * a.k + jj] * L.sa[HK + h * a.k + jj];
      da = L.sa[p] * (L.sa[HK + p] - sdot) * scale;
    }
    da_keep[it] = da;
  }
  wave_lds_sync();
  it = 0;
  for (int p = lane; p < HK; p += 64, ++it) {
    L.sa[HK + p] = da_keep[it];
    a.dscore[(size_t)r * HK + p] = da_keep[it];
  }
  wave_lds_sync();
  for (int e = lane; e < a.dO; e += 64) {
    const int h = e / a.dh;
    float acc = 0.f;
    for (int j = 0; j < c; ++j) acc += L.sa[HK + h * a.k + j] * a.P[(size_t)L.row[j] * a.ldp + e];
    a.dqn[(size_t)r * a.ldh + e] = acc;
    a.Qroot[(size_t)r * a.ldh + e] = qv[e];
  }
  float* zrow = a.Zs + (size_t)r * a.ldz;
  for (int col = lane; col < a.dcp; col += 64) {
    float acc[TGNN_MAX_HEADS];
#pragma unroll
    for (int h = 0; h < TGNN_MAX_HEADS; ++h) acc[h] = 0.f;
    float yw = 0.f, yb = 0.f;
    if (col < dc) {
      for (int j = 0; j < c; ++j) {
        float sn;
        const float cv = slot_col(a, L.e[j], L.dt[j], col, sn);
        float dphi = 0.f;
#pragma unroll
        for (int h = 0; h < TGNN_MAX_HEADS; ++h) {
          if (h < a.H) {
            const float ds = L.sa[HK + h * a.k + j];
            acc[h] += ds * cv;
            dphi += ds * urow[h * a.dcp + col] + L.sa[h * a.k + j] * grow[h * a.dcp + col];
          }
        }
        const float t = -dphi * sn;
        yb += t;
        yw += t * (float)L.dt[j];
      }
    }
#pragma unroll
    for (int h = 0; h < TGNN_MAX_HEADS; ++h)
      if (h < a.H) zrow[h * a.dcp + col] = acc[h];
    if (col >= a.de && col < dc) {
      yrow[col - a.de] = yw;
      yrow[a.dt + col - a.de] = yb;
    }
  }
}

static bool fast_path(const FusedAttn& a) {
  return !a.force_generic && a.k <= FA_KR && a.de <= 64 * FA_NE && a.dt <= 64 * FA_NT && a.dO <= 64 * FA_E &&
         a.H <= FA_HM && a.H * a.k <= 64;
}

void fattn_fwd(const FusedAttn& a, hipStream_t s) {
  if (a.R <= 0) return;
  const int fill_blocks = a.fill.ucnt != nullptr ? uniq_blocks(a.fill.S) : 0;
  const dim3 grid((a.R + 3) / 4 + fill_blocks);
  if (fast_path(a))
    hipLaunchKernelGGL(fattn_fwd_fast_kernel, grid, dim3(256), 4 * sizeof(float) * fattn_lds_floats(a.k, a.H), s, a);
  else
    hipLaunchKernelGGL(fattn_fwd_gen_kernel, grid, dim3(256), 4 * gattn_lds_bytes(a.k, a.H), s, a);
}

void fattn_bwd(const FusedAttn& a, hipStream_t s) {
  if (a.R <= 0) return;
  const dim3 grid((a.R + 3) / 4);
  if (fast_path(a))
    hipLaunchKernelGGL(fattn_bwd_fast_kernel, grid, dim3(256), 4 * sizeof(float) * fattn_lds_floats(a.k, a.H), s, a);
  else
    hipLaunchKernelGGL(fattn_bwd_gen_kernel, grid, dim3(256), 4 * gattn_lds_bytes(a.k, a.H), s, a);
}

}  // namespace tgnn
