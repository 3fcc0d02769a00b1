// The root-level chain of a training step in one launch: merge layer z = ReLU(W_o {h_v | x_v} + b_o) (Eq. 7's
// output layer), link-prediction decoder with its BCE loss (Sec. 2.1 / 3.2.2, one negative destination per event),
// and the way back down to the gradient of the attention output.  Everything between the attention output of a
// root and its gradient is local to an event's three roots (source, true destination, negative destination), so a
// workgroup takes 16 events = three 16-row MFMA blocks (one per role, each contiguous in the root order
// [src | dst | neg] of a batch) through four small products whose operands stay in LDS:
//   z      = ReLU(h W_oh^T + P_o[row(root)])                      (P_o: node part of the merge layer, bias included)
//   Pdec   = z W_s^T for sources, z W_d^T for destinations         (only the half a root needs)
//   pairs  : hidden = ReLU(Pdec_src + Pdec_dst + b1), logit, loss, d/d(logit), d/d(hidden) -> dPdec per root
//   dz     = gate_z(dPdec W_s) for sources, gate_z(dPdec W_d) for destinations
//   dOmat  = dz W_oh
// The weights are read from global memory (L2) as MFMA B operands, a lane's run of a weight row per 16-wide k slab.
// z, h1, dPdec ({W_s part | W_d part}, the unused half zero), dz and dOmat go to memory for the weight-gradient
// products and the attention backward pass.
#include "tgnn_internal.h"
#include "device_math.h"

namespace tgnn {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int RC_E = 16;                 // events per workgroup
constexpr int RC_WAVES = 8;
constexpr int RC_UNITS = 3;              // a wavefront's units: the three role blocks of its column block
constexpr int RC_MAXD = 128;             // widest d_o (8 column blocks of 16, one per wavefront)
constexpr int RC_PL = RC_MAXD + 4;       // LDS row pitch: 33 float4 chunks, so 16 rows x one chunk cover all banks

// The B operands of a wavefront for one product: a lane's run [16 s + 4 lg, +4) of its weight row for every k
// slab s; set 0 serves the sources, set 1 the destinations (products whose weights do not depend on the role
// use set 0 for all three role blocks).  Two such sets alternate: the loads of the next product's weights
// (they depend on nothing computed here) are issued among the current product's MFMAs.
template <int KS> struct RcSet {
  floatx4 w[2][KS];
};

struct RcWho {   // a wavefront's units: role block j, column block cb (the same for all three)
  int rb[RC_UNITS], cb[RC_UNITS];
  bool has[RC_UNITS];
};

// W: weight block with one row per output column; the destinations' block starts dst_off floats later
// (SPLIT = false: one block for all roles).
template <int KS, bool SPLIT>
__device__ __forceinline__ void rc_load(RcSet<KS>& set, const RcWho& who, const float* __restrict__ W, size_t dst_off,
                                        int ldw, int N, int li, int lg) {
  const float* p = W + (size_t)min(who.cb[0] * 16 + li, N - 1) * ldw + lg * 4;
#pragma unroll
  for (int s = 0; s < KS; ++s) set.w[0][s] = *reinterpret_cast<const floatx4*>(p + s * 16);
  if (SPLIT) {
#pragma unroll
    for (int s = 0; s < KS; ++s) set.w[1][s] = *reinterpret_cast<const floatx4*>(p + dst_off + s * 16);
  }
}

// acc[j][v] = sum_k T[16 j + li][k] W_j[col][k]  -> element (16 j + 4 lg + v, 16 cb + li).  The three
// accumulation chains are independent and interleaved, so an MFMA never waits for the one before it.
// PF != 0: the next product's weights (PF == 2: with a separate block for the destinations) are fetched into
// `next` on the way, one k slab per k slab: the weight rows are 64-byte pieces of scattered lines, which the
// vector memory path takes about as long to bring in as the MFMAs of a product take.
// The MFMAs are unconditional (a wavefront without a column block skips the whole call): a wave-uniform `if`
// around single MFMAs made the compiler branch around each of them and pad with s_nop, at twice the time.
template <int KS, bool SPLIT, int PF>
__device__ __forceinline__ void rc_mma(const RcSet<KS>& set, const RcWho& who, const float* T, int li, int lg,
                                       floatx4 (&acc)[RC_UNITS], RcSet<KS>& next, const float* __restrict__ Wn,
                                       size_t dst_off_n, int ldw_n, int N) {
  const float* pa[RC_UNITS];
#pragma unroll
  for (int j = 0; j < RC_UNITS; ++j) {
    acc[j] = floatx4{0.f, 0.f, 0.f, 0.f};
    pa[j] = T + (who.rb[j] * 16 + li) * RC_PL + lg * 4;
  }
  const float* pn = PF ? Wn + (size_t)min(who.cb[0] * 16 + li, N - 1) * ldw_n + lg * 4 : nullptr;
#pragma unroll
  for (int s = 0; s < KS; ++s) {
    if (PF >= 1) next.w[0][s] = *reinterpret_cast<const floatx4*>(pn + s * 16);
    if (PF == 2) next.w[1][s] = *reinterpret_cast<const floatx4*>(pn + dst_off_n + s * 16);
    floatx4 a4[RC_UNITS];
#pragma unroll
    for (int j = 0; j < RC_UNITS; ++j) a4[j] = *reinterpret_cast<const floatx4*>(pa[j] + s * 16);
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
      for (int j = 0; j < RC_UNITS; ++j)
        acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a4[j][c], set.w[(SPLIT && j > 0) ? 1 : 0][s][c], acc[j], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);   // nothing moves across k slabs
  }
}

template <int KS>
__global__ __launch_bounds__(64 * RC_WAVES) void root_chain_kernel(ChainArgs a) {
  __shared__ __attribute__((aligned(16))) float T0[3 * RC_E * RC_PL];   // h -> Pdec -> dPdec
  __shared__ __attribute__((aligned(16))) float T1[3 * RC_E * RC_PL];   // z -> dz
  __shared__ float red[RC_E][2 * 64 + 2];

  // which 16 events: tiles are dealt batch by batch (sizes from the argument block: no memory round trip)
  int b = 0, tile = blockIdx.x, off = 0;
  while (b + 1 < a.nb && tile >= (a.n[b] + RC_E - 1) / RC_E) {
    tile -= (a.n[b] + RC_E - 1) / RC_E;
    off += a.n[b];
    ++b;
  }
  const int n = a.n[b], nb = a.nb;
  const int i0 = tile * RC_E;
  if (i0 >= n) return;   // uniform
  const int n_here = min(RC_E, n - i0);

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int li = lane & 15, lg = lane >> 4;
  const int dO = a.dO, ldh = a.ldh, ldkv = a.ldkv;
  constexpr int n_cb = KS;
  // local row role * 16 + e  <->  root row 3 off + role n + i0 + e (e clamped to the tile's last event for loads)
  const int root0 = 3 * off + i0;

  RcWho who;
#pragma unroll
  for (int j = 0; j < RC_UNITS; ++j) {   // (a wavefront beyond the last column block repeats it, without storing)
    who.has[j] = wave < n_cb;
    who.rb[j] = j;
    who.cb[j] = min(wave, n_cb - 1);
  }
  RcSet<KS> wa, wb;
  // Order of the first loads (they return in order): the attention output, which the first product waits
  // for; its weights; the node rows of the roots this lane finishes.  Once those rows are known, the node part
  // of the merge layer, needed only after the first product's MFMAs.
  // (all of a thread's pieces of the attention output are loaded before the first goes to LDS: a load -> store loop
  // would pay one memory latency per pass)
  constexpr int OM_CHUNKS = 3 * RC_E * (RC_PL / 4), OM_PER = (OM_CHUNKS + 64 * RC_WAVES - 1) / (64 * RC_WAVES);
  floatx4 om[OM_PER];
#pragma unroll
  for (int u = 0; u < OM_PER; ++u) {
    const int idx = min(tid + u * 64 * RC_WAVES, OM_CHUNKS - 1);
    const int lr = idx / (RC_PL / 4), c = (idx - lr * (RC_PL / 4)) * 4;
    const int role = lr >> 4, e = min(lr & 15, n_here - 1);
    om[u] = floatx4{0.f, 0.f, 0.f, 0.f};
    if (c < dO) om[u] = *reinterpret_cast<const floatx4*>(a.Omat + (size_t)(root0 + role * n + e) * ldh + c);
  }
  __builtin_amdgcn_sched_barrier(0);   // keep this issue order
  rc_load<KS, false>(wa, who, a.Wo_o, 0, ldh, dO, li, lg);
  int prow[RC_UNITS][4];
#pragma unroll
  for (int j = 0; j < RC_UNITS; ++j)
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int r = root0 + who.rb[j] * n + min(lg * 4 + v, n_here - 1);
      prow[j][v] = a.slot_row != nullptr ? a.slot_row[r] : r;
    }
  const float b2v = a.b2[0];
  const int l32 = lane & 31;
  float bb[4], ww[4];   // decoder bias and output weights, columns l32 + 32 q
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int c = l32 + 32 * q;
    bb[q] = c < dO ? a.b1[c] : 0.f;
    ww[q] = c < dO ? a.w2[c] : 0.f;
  }
  __builtin_amdgcn_sched_barrier(0);
  // attention output rows -> T0 (columns >= d_o zero)
#pragma unroll
  for (int u = 0; u < OM_PER; ++u) {
    const int idx = tid + u * 64 * RC_WAVES;
    if (idx < OM_CHUNKS) {
      const int lr = idx / (RC_PL / 4), c = (idx - lr * (RC_PL / 4)) * 4;
      *reinterpret_cast<floatx4*>(&T0[lr * RC_PL + c]) = om[u];
    }
  }
  __builtin_amdgcn_sched_barrier(0);
  float addv[RC_UNITS][4];
#pragma unroll
  for (int j = 0; j < RC_UNITS; ++j) {
    const int col = min(who.cb[j] * 16 + li, dO - 1);
#pragma unroll
    for (int v = 0; v < 4; ++v) addv[j][v] = a.P_o[(size_t)prow[j][v] * a.ldp + col];
  }
  __syncthreads();

  // ---- z = ReLU(h W_oh^T + P_o[row]) ----
  // next: Pdec, sources through W_s (rows 0 .. d_o-1 of the packed block), destinations through W_d
  floatx4 acc[RC_UNITS];
  if (who.has[0]) rc_mma<KS, false, 2>(wa, who, T0, li, lg, acc, wb, a.Wdec_p, (size_t)dO * ldh, ldh, dO);
#pragma unroll
  for (int j = 0; j < RC_UNITS; ++j) {
    if (who.has[j]) {
      const int col = who.cb[j] * 16 + li;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int e = lg * 4 + v;
        const float x = col < dO ? fmaxf(acc[j][v] + addv[j][v], 0.f) : 0.f;
        T1[(who.rb[j] * 16 + e) * RC_PL + col] = x;
        if (col < dO && e < n_here) a.z[(size_t)(root0 + who.rb[j] * n + e) * ldh + col] = x;
      }
    }
  }
  __syncthreads();

  // ---- Pdec ----
  // next: dz; row c of the transposed block is {W_s[:, c] | W_d[:, c]}
  if (who.has[0]) rc_mma<KS, true, 2>(wb, who, T1, li, lg, acc, wa, a.WdecT, (size_t)dO, ldkv, dO);
#pragma unroll
  for (int j = 0; j < RC_UNITS; ++j) {
    if (who.has[j]) {
      const int col = who.cb[j] * 16 + li;
#pragma unroll
      for (int v = 0; v < 4; ++v) T0[(who.rb[j] * 16 + lg * 4 + v) * RC_PL + col] = col < dO ? acc[j][v] : 0.f;
    }
  }
  __syncthreads();

  // ---- pairs: a half wavefront per event (16 events, 8 wavefronts); a lane takes columns l + 32 q ----
  {
    const float inv = 1.0f / (2.0f * (float)n);
    const int e = wave * 2 + (lane >> 5);
    const bool valid = e < n_here;
    float gb = 0.f, lsum = 0.f;
    float hp[4], hn[4];
    float ap = 0.f, an = 0.f;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int c = l32 + 32 * q;
      hp[q] = hn[q] = 0.f;
      if (c < dO) {
        const float ps = T0[e * RC_PL + c] + bb[q];
        hp[q] = fmaxf(ps + T0[(16 + e) * RC_PL + c], 0.f);
        hn[q] = fmaxf(ps + T0[(32 + e) * RC_PL + c], 0.f);
      }
      ap += hp[q] * ww[q];
      an += hn[q] * ww[q];
    }
#pragma unroll
    for (int o = 16; o > 0; o >>= 1) {
      ap += __shfl_xor(ap, o);
      an += __shfl_xor(an, o);
    }
    const float lp = ap + b2v, ln = an + b2v;
    const float spp = fmaxf(-lp, 0.f) + log1pf(expf(-fabsf(lp)));
    const float spn = fmaxf(ln, 0.f) + log1pf(expf(-fabsf(ln)));
    const float dlp = valid ? (1.0f / (1.0f + expf(-lp)) - 1.0f) * inv : 0.f;   // d(sum_b loss_b) / d logit
    const float dln = valid ? (1.0f / (1.0f + expf(-ln))) * inv : 0.f;
    const int row_p = 2 * off + i0 + e, row_n = row_p + n;
    if (valid && l32 == 0) {
      a.logits[row_p] = lp;
      a.logits[row_n] = ln;
      lsum = (spp + spn) * inv / (float)nb;
      gb = dlp + dln;
    }
    const size_t ra = (size_t)(root0 + e) * ldkv, rbb = ra + (size_t)n * ldkv, rc = rbb + (size_t)n * ldkv;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int c = l32 + 32 * q;
      float gw = 0.f;
      if (c < dO) {
        const float dhp = hp[q] > 0.f ? dlp * ww[q] : 0.f;
        const float dhn = hn[q] > 0.f ? dln * ww[q] : 0.f;
        T0[e * RC_PL + c] = dhp + dhn;
        T0[(16 + e) * RC_PL + c] = dhp;
        T0[(32 + e) * RC_PL + c] = dhn;
        if (valid) {
          a.h1[(size_t)row_p * ldh + c] = hp[q];
          a.h1[(size_t)row_n * ldh + c] = hn[q];
          a.dPdec[ra + c] = dhp + dhn;
          a.dPdec[ra + dO + c] = 0.f;
          a.dPdec[rbb + c] = 0.f;
          a.dPdec[rbb + dO + c] = dhp;
          a.dPdec[rc + c] = 0.f;
          a.dPdec[rc + dO + c] = dhn;
          gw = dlp * hp[q] + dln * hn[q];
        }
      }
      red[e][c] = gw;
    }
    if (l32 == 0) { red[e][128] = gb; red[e][129] = lsum; }
  }
  __syncthreads();
  if (wave == RC_WAVES - 1) {   // per-workgroup sums of the w2, b2 gradients and of the loss
    for (int c = lane; c < 130; c += 64) {
      float sum = 0.f;
#pragma unroll
      for (int e = 0; e < RC_E; ++e) sum += red[e][c];
      if (c < dO) atomicAdd(a.g_w2 + c, sum);
      else if (c == 128) atomicAdd(a.g_b2, sum);
      else if (c == 129) atomicAdd(a.loss, sum);
    }
  }

  // ---- dz = gate_z(dPdec {W_s | W_d}) ----
  if (who.has[0]) rc_mma<KS, true, 1>(wa, who, T0, li, lg, acc, wb, a.WoT_o, 0, ldh, dO);
#pragma unroll
  for (int j = 0; j < RC_UNITS; ++j) {
    if (who.has[j]) {
      const int col = who.cb[j] * 16 + li;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int e = lg * 4 + v;
        float* t = &T1[(who.rb[j] * 16 + e) * RC_PL + col];
        const float x = (col < dO && *t > 0.f) ? acc[j][v] : 0.f;
        *t = x;
        if (col < dO && e < n_here) a.dz[(size_t)(root0 + who.rb[j] * n + e) * ldh + col] = x;
      }
    }
  }
  __syncthreads();

  // ---- dOmat = dz W_oh ----
  if (who.has[0]) rc_mma<KS, false, 0>(wb, who, T1, li, lg, acc, wa, nullptr, 0, 0, dO);
#pragma unroll
  for (int j = 0; j < RC_UNITS; ++j) {
    if (who.has[j]) {
      const int col = who.cb[j] * 16 + li;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int e = lg * 4 + v;
        if (col < dO && e < n_here) a.dOmat[(size_t)(root0 + who.rb[j] * n + e) * ldh + col] = acc[j][v];
      }
    }
  }
}

bool root_chain_fits(const Dims& d) {
  // float4 runs of the weight rows (also at the W_d offset d_o), and the k slabs of the W_d half stay inside a row
  return d.dO % 4 == 0 && d.dO <= RC_MAXD && d.ldh >= ((d.dO + 15) / 16) * 16 &&
         d.ldkv >= d.dO + ((d.dO + 15) / 16) * 16;
}

void root_chain(ChainArgs a, const BatchSet& bs_host, hipStream_t s) {
  int tiles = 0;
  a.nb = bs_host.nb;
  for (int b = 0; b < bs_host.nb; ++b) {
    a.n[b] = bs_host.b[b].n;
    tiles += (bs_host.b[b].n + RC_E - 1) / RC_E;
  }
  if (tiles <= 0) return;
#define TGNN_RC_CASE(KSV) \
  case KSV: hipLaunchKernelGGL((root_chain_kernel<KSV>), dim3(tiles), dim3(64 * RC_WAVES), 0, s, a); break;
  switch ((a.dO + 15) / 16) {
    TGNN_RC_CASE(1) TGNN_RC_CASE(2) TGNN_RC_CASE(3) TGNN_RC_CASE(4)
    TGNN_RC_CASE(5) TGNN_RC_CASE(6) TGNN_RC_CASE(7) TGNN_RC_CASE(8)
    default: break;   // root_chain_fits() rules these out
  }
#undef TGNN_RC_CASE
}

}  // namespace tgnn
