// The root-level chain of a training step in one launch: merge layer z = ReLU(W_o {h_v | x_v} + b_o) (Eq. 7's
// output layer), link-prediction decoder with its BCE loss (Sec. 2.1 / 3.2.2, one negative destination per event),
// and the way back down to the gradient of the attention output.  Everything between the attention output of a
// root and its gradient is local to an event's three roots (source, true destination, negative destination), so a
// workgroup takes E events through four small products whose operands stay in LDS: E = 16, three 16-row MFMA
// blocks, one per role (each contiguous in the root order [src | dst | neg] of a batch), when a step has many
// events; E = 5, one 16-row block {5 src | 5 dst | 5 neg | pad}, when it has few and more workgroups (compute
// units) are worth more than full blocks:
//   z      = ReLU(h W_oh^T + P_o[row(root)])                      (P_o: node part of the merge layer, bias included)
//   Pdec   = z W_s^T for sources, z W_d^T for destinations         (only the half a root needs)
//   pairs  : hidden = ReLU(Pdec_src + Pdec_dst + b1), logit, loss, d/d(logit), d/d(hidden) -> dPdec per root
//   dz     = gate_z(dPdec W_s) for sources, gate_z(dPdec W_d) for destinations
//   dOmat  = dz W_oh
// The weights are read from global memory (L2) as MFMA B operands, from copies laid out in operand order (the
// prologue writes them): 1 KB of contiguous memory per wavefront, column block and 16-wide k slab.
// z, h1, dPdec ({W_s part | W_d part}, the unused half zero), dz and dOmat go to memory for the weight-gradient
// products and the attention backward pass.
#include "tgnn_internal.h"
#include "device_math.h"

namespace tgnn {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int RC_WAVES = 8;
constexpr int RC_MAXD = 128;             // widest d_o (8 column blocks of 16, one per wavefront)
constexpr int RC_PL = RC_MAXD + 4;       // LDS row pitch: 33 float4 chunks, so 16 rows x one chunk cover all banks

// Geometry of a tile of E events.  Local rows: E = 16: role * 16 + e; E = 5: role * 5 + e, row 15 is padding.
// A product whose weights depend on the role ("split": W_s for sources, W_d for both kinds of destinations) is a
// list of units (row block, weight set); with E = 5 the one row block meets both weight sets and each unit keeps
// the rows of its roles.
template <int E> struct RcGeom {
  static_assert(E == 16 || E == 5, "tile shapes: three full row blocks, or one block of 5 + 5 + 5 rows");
  static constexpr int NB = E == 16 ? 3 : 1;           // 16-row blocks
  static constexpr int ROWS = 16 * NB;
  static constexpr int NU_SHARED = NB;                 // units of a product with one weight block
  static constexpr int NU_SPLIT = E == 16 ? 3 : 2;     // units of a split product
  __device__ static __forceinline__ int role(int lr) { return E == 16 ? lr >> 4 : min(lr / E, 2); }
  __device__ static __forceinline__ int ev(int lr) { return E == 16 ? lr & 15 : lr - role(lr) * E; }   // >= E: padding
  __device__ static __forceinline__ int row(int role, int e) { return E == 16 ? role * 16 + e : role * E + e; }
  template <bool SPLIT> __device__ static __forceinline__ constexpr int unit_rb(int j) { return E == 16 ? j : 0; }
  template <bool SPLIT> __device__ static __forceinline__ constexpr int unit_ws(int j) {
    return SPLIT ? (E == 16 ? (j > 0 ? 1 : 0) : j) : 0;
  }
  // does split unit j keep local row lr of its block?
  __device__ static __forceinline__ bool keeps(int j, int lr) { return E == 16 ? true : (j == 0 ? lr < E : lr >= E); }
};

// The B operands of a wavefront for one product: a lane's run [16 s + 4 lg, +4) of its weight row for every k
// slab s; set 0 serves the sources, set 1 the destinations (products whose weights do not depend on the role
// use set 0 only).  Two such sets alternate: the loads of the next product's weights (they depend on nothing
// computed here) are issued among the current product's MFMAs.
template <int KS> struct RcSet {
  floatx4 w[2][KS];
};

// W0 (and W1 for the destinations when SPLIT): weight blocks in MFMA B-operand order: the lanes' float4 pieces of
// column block cb and k slab s are the 1 KB at (cb KS + s) * 256 floats.
template <int KS, bool SPLIT>
__device__ __forceinline__ void rc_load(RcSet<KS>& set, int cb, const float* __restrict__ W0, const float* __restrict__ W1,
                                        int lane) {
  const float* p0 = W0 + ((size_t)cb * KS * 64 + lane) * 4;
#pragma unroll
  for (int s = 0; s < KS; ++s) set.w[0][s] = *reinterpret_cast<const floatx4*>(p0 + s * 256);
  if (SPLIT) {
    const float* p1 = W1 + ((size_t)cb * KS * 64 + lane) * 4;
#pragma unroll
    for (int s = 0; s < KS; ++s) set.w[1][s] = *reinterpret_cast<const floatx4*>(p1 + s * 256);
  }
}

// acc[j][v] = sum_k T[16 rb_j + li][k] W_j[col][k]  -> element (16 rb_j + 4 lg + v, 16 cb + li) of unit j.  The
// units' accumulation chains are independent and interleaved, so an MFMA never waits for the one before it.
// PF != 0: the next product's weights (PF == 2: with a separate block for the destinations) are fetched into
// `next` on the way, one k slab per k slab.
// The MFMAs are unconditional (a wavefront without a column block skips the whole call): a wave-uniform `if`
// around single MFMAs made the compiler branch around each of them and pad with s_nop, at twice the time.
template <int KS, int E, bool SPLIT, int PF>
__device__ __forceinline__ void rc_mma(const RcSet<KS>& set, int cb, const float* T, int li, int lg, floatx4 (&acc)[3],
                                       RcSet<KS>& next, const float* __restrict__ Wn0, const float* __restrict__ Wn1) {
  typedef RcGeom<E> G;
  constexpr int NU = SPLIT ? G::NU_SPLIT : G::NU_SHARED;
  const float* pa[NU];
#pragma unroll
  for (int j = 0; j < NU; ++j) {
    acc[j] = floatx4{0.f, 0.f, 0.f, 0.f};
    pa[j] = T + (G::template unit_rb<SPLIT>(j) * 16 + li) * RC_PL + lg * 4;
  }
  const int lane64 = lg * 16 + li;
  const float* pn0 = PF ? Wn0 + ((size_t)cb * KS * 64 + lane64) * 4 : nullptr;
  const float* pn1 = PF == 2 ? Wn1 + ((size_t)cb * KS * 64 + lane64) * 4 : nullptr;
#pragma unroll
  for (int s = 0; s < KS; ++s) {
    if (PF >= 1) next.w[0][s] = *reinterpret_cast<const floatx4*>(pn0 + s * 256);
    if (PF == 2) next.w[1][s] = *reinterpret_cast<const floatx4*>(pn1 + s * 256);
    floatx4 a4[NU];
#pragma unroll
    for (int j = 0; j < NU; ++j)
      a4[j] = (E != 16 && j > 0) ? a4[0] : *reinterpret_cast<const floatx4*>(pa[j] + s * 16);   // one row block: one read
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
      for (int j = 0; j < NU; ++j)
        acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a4[j][c], set.w[G::template unit_ws<SPLIT>(j)][s][c], acc[j], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);   // nothing moves across k slabs
  }
}

template <int KS, int E>
__global__ __launch_bounds__(64 * RC_WAVES) void root_chain_kernel(ChainArgs a) {
  typedef RcGeom<E> G;
  __shared__ __attribute__((aligned(16))) float T0[G::ROWS * RC_PL];   // h -> Pdec -> dPdec
  __shared__ __attribute__((aligned(16))) float T1[G::ROWS * RC_PL];   // z -> dz
  __shared__ float red[E][2 * 64 + 2];

  // which E events: tiles are dealt batch by batch (sizes from the argument block: no memory round trip)
  int b = 0, tile = blockIdx.x, off = 0;
  while (b + 1 < a.nb && tile >= (a.n[b] + E - 1) / E) {
    tile -= (a.n[b] + E - 1) / E;
    off += a.n[b];
    ++b;
  }
  const int n = a.n[b], nb = a.nb;
  const int i0 = tile * E;
  if (i0 >= n) return;   // uniform
  const int n_here = min(E, n - i0);

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int li = lane & 15, lg = lane >> 4;
  const int dO = a.dO, ldh = a.ldh, ldkv = a.ldkv;
  const bool has_cb = wave < KS;            // a wavefront beyond the last column block takes no part in the products
  const int cb = min(wave, KS - 1);
  // local row <-> root row 3 off + role n + i0 + e (e clamped to the tile's last event for loads)
  const int root0 = 3 * off + i0;
  auto groot = [&](int lr) { return root0 + G::role(lr) * n + min(G::ev(lr), n_here - 1); };
  auto live = [&](int lr) { return G::ev(lr) < n_here; };   // not padding, not past a ragged batch end

  RcSet<KS> wa, wb;
  // Order of the first loads (they return in order): the attention output, which the first product waits
  // for; its weights; the node rows of the roots this lane finishes.  Once those rows are known, the node part
  // of the merge layer, needed only after the first product's MFMAs.
  // (all of a thread's pieces of the attention output are loaded before the first goes to LDS: a load -> store loop
  // would pay one memory latency per pass)
  constexpr int OM_CHUNKS = G::ROWS * (RC_PL / 4), OM_PER = (OM_CHUNKS + 64 * RC_WAVES - 1) / (64 * RC_WAVES);
  floatx4 om[OM_PER];
#pragma unroll
  for (int u = 0; u < OM_PER; ++u) {
    const int idx = min(tid + u * 64 * RC_WAVES, OM_CHUNKS - 1);
    const int lr = idx / (RC_PL / 4), c = (idx - lr * (RC_PL / 4)) * 4;
    om[u] = floatx4{0.f, 0.f, 0.f, 0.f};
    if (c < dO) om[u] = *reinterpret_cast<const floatx4*>(a.Omat + (size_t)groot(lr) * ldh + c);
  }
  __builtin_amdgcn_sched_barrier(0);   // keep this issue order
  rc_load<KS, false>(wa, cb, a.Wo_pk, nullptr, lane);
  int prow[G::NB][4];
#pragma unroll
  for (int j = 0; j < G::NB; ++j)
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int r = groot(j * 16 + lg * 4 + v);
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
  float addv[G::NB][4];
#pragma unroll
  for (int j = 0; j < G::NB; ++j) {
    const int col = min(cb * 16 + li, dO - 1);
#pragma unroll
    for (int v = 0; v < 4; ++v) addv[j][v] = a.P_o[(size_t)prow[j][v] * a.ldp + col];
  }
  __syncthreads();

  const int col = cb * 16 + li;   // this lane's column in every product
  floatx4 acc[3];

  // ---- z = ReLU(h W_oh^T + P_o[row]) ----
  // next: Pdec, sources through W_s, destinations through W_d
  if (has_cb) {
    rc_mma<KS, E, false, 2>(wa, cb, T0, li, lg, acc, wb, a.Ws_pk, a.Wd_pk);
#pragma unroll
    for (int j = 0; j < G::NU_SHARED; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int lr = j * 16 + lg * 4 + v;
        const float x = col < dO ? fmaxf(acc[j][v] + addv[j][v], 0.f) : 0.f;
        T1[lr * RC_PL + col] = x;
        if (col < dO && live(lr)) a.z[(size_t)groot(lr) * ldh + col] = x;
      }
  }
  __syncthreads();

  // ---- Pdec ----
  // next: dz, through the transposed blocks
  if (has_cb) {
    rc_mma<KS, E, true, 2>(wb, cb, T1, li, lg, acc, wa, a.WsT_pk, a.WdT_pk);
#pragma unroll
    for (int j = 0; j < G::NU_SPLIT; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int lb = lg * 4 + v, lr = G::template unit_rb<true>(j) * 16 + lb;
        if (G::keeps(j, lb)) T0[lr * RC_PL + col] = col < dO ? acc[j][v] : 0.f;
      }
  }
  __syncthreads();

  // ---- pairs: a half wavefront per event; a lane takes columns l + 32 q ----
  {
    const float inv = 1.0f / (2.0f * (float)n);
    const int e_raw = wave * 2 + (lane >> 5);
    // (E = 5: the last half wavefronts have no event; they go through the arithmetic on the last event's rows,
    // which its owner may be rewriting meanwhile, and drop the result)
    const bool mine = e_raw < E;
    const int e = min(e_raw, E - 1);
    const bool valid = mine && e < n_here;
    const int r_src = G::row(0, e), r_dst = G::row(1, e), r_neg = G::row(2, e);
    float gb = 0.f, lsum = 0.f;
    float hp[4], hn[4];
    float ap = 0.f, an = 0.f;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int c = l32 + 32 * q;
      hp[q] = hn[q] = 0.f;
      if (c < dO) {
        const float ps = T0[r_src * RC_PL + c] + bb[q];
        hp[q] = fmaxf(ps + T0[r_dst * RC_PL + c], 0.f);
        hn[q] = fmaxf(ps + T0[r_neg * RC_PL + c], 0.f);
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
    if (mine) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int c = l32 + 32 * q;
        float gw = 0.f;
        if (c < dO) {
          const float dhp = hp[q] > 0.f ? dlp * ww[q] : 0.f;
          const float dhn = hn[q] > 0.f ? dln * ww[q] : 0.f;
          T0[r_src * RC_PL + c] = dhp + dhn;
          T0[r_dst * RC_PL + c] = dhp;
          T0[r_neg * RC_PL + c] = dhn;
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
  }
  __syncthreads();
  if (wave == RC_WAVES - 1) {   // per-workgroup sums of the w2, b2 gradients and of the loss
    for (int c = lane; c < 130; c += 64) {
      float sum = 0.f;
#pragma unroll
      for (int e = 0; e < E; ++e) sum += red[e][c];
      if (c < dO) atomicAdd(a.g_w2 + c, sum);
      else if (c == 128) atomicAdd(a.g_b2, sum);
      else if (c == 129) atomicAdd(a.loss, sum);
    }
  }

  // ---- dz = gate_z(dPdec {W_s | W_d}) ----
  if (has_cb) {
    rc_mma<KS, E, true, 1>(wa, cb, T0, li, lg, acc, wb, a.WoT_pk, nullptr);
#pragma unroll
    for (int j = 0; j < G::NU_SPLIT; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int lb = lg * 4 + v, lr = G::template unit_rb<true>(j) * 16 + lb;
        if (G::keeps(j, lb)) {
          float* t = &T1[lr * RC_PL + col];
          const float x = (col < dO && *t > 0.f) ? acc[j][v] : 0.f;
          *t = x;
          if (col < dO && live(lr)) a.dz[(size_t)groot(lr) * ldh + col] = x;
        }
      }
  }
  __syncthreads();

  // ---- dOmat = dz W_oh ----
  if (has_cb) {
    rc_mma<KS, E, false, 0>(wb, cb, T1, li, lg, acc, wa, nullptr, nullptr);
#pragma unroll
    for (int j = 0; j < G::NU_SHARED; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int lr = j * 16 + lg * 4 + v;
        if (col < dO && live(lr)) a.dOmat[(size_t)groot(lr) * ldh + col] = acc[j][v];
      }
  }
}

bool root_chain_fits(const Dims& d) {
  // float4 runs of the weight rows (also at the W_d offset d_o), and the k slabs of the W_d half stay inside a row
  return d.dO % 4 == 0 && d.dO <= RC_MAXD && d.ldh >= ((d.dO + 15) / 16) * 16 &&
         d.ldkv >= d.dO + ((d.dO + 15) / 16) * 16;
}

// Few events (wide == false is then chosen): 5 per workgroup, so that a 600-event step occupies 120 compute units
// instead of 38; many: 16 per workgroup, full MFMA row blocks.
constexpr int RC_FEW_EVENTS = 1280;

void root_chain(ChainArgs a, const BatchSet& bs_host, bool force_wide, hipStream_t s) {
  int total = 0;
  a.nb = bs_host.nb;
  for (int b = 0; b < bs_host.nb; ++b) {
    a.n[b] = bs_host.b[b].n;
    total += bs_host.b[b].n;
  }
  if (total <= 0) return;
  const bool wide = force_wide || total > RC_FEW_EVENTS;
  const int E = wide ? 16 : 5;
  int tiles = 0;
  for (int b = 0; b < bs_host.nb; ++b) tiles += (bs_host.b[b].n + E - 1) / E;
#define TGNN_RC_CASE(KSV)                                                                                        \
  case KSV:                                                                                                      \
    if (wide) hipLaunchKernelGGL((root_chain_kernel<KSV, 16>), dim3(tiles), dim3(64 * RC_WAVES), 0, s, a);       \
    else hipLaunchKernelGGL((root_chain_kernel<KSV, 5>), dim3(tiles), dim3(64 * RC_WAVES), 0, s, a);             \
    break;
  switch ((a.dO + 15) / 16) {
    TGNN_RC_CASE(1) TGNN_RC_CASE(2) TGNN_RC_CASE(3) TGNN_RC_CASE(4)
    TGNN_RC_CASE(5) TGNN_RC_CASE(6) TGNN_RC_CASE(7) TGNN_RC_CASE(8)
    default: break;   // root_chain_fits() rules these out
  }
#undef TGNN_RC_CASE
}

}  // namespace tgnn
