// fp32 MFMA GEMMs for the dense contractions of the step: the GRU and attention projections
// (Eq. 3-6), the merge layer, the decoder, and their data / weight gradients.
//
// v_mfma_f32_16x16x4_f32: lane l supplies A[i = l%16][kk = l/16] and B[kk = l/16][j = l%16]; its four
// accumulators hold D[i = 4*(l/16) + v][j = l%16].  The sum over kk is order independent, so a lane may
// feed any four k indices per instruction as long as both operands use the same ones: lane group g reads
// one float4 (k = 4g .. 4g+3 of a 16-wide slab) and issues four MFMAs from it.
//
// Both kernels keep two register tile sets in flight (global loads issued two stages ahead) and two LDS
// buffers, so a workgroup waits for memory only when the chip has nothing else resident to run.
#include <stdlib.h>

#include <algorithm>
#include <cstring>

#include "tgnn_internal.h"
#include "device_math.h"
#include "writeback_device.h"

namespace tgnn {

typedef float floatx4 __attribute__((ext_vector_type(4)));

// A row count that an earlier kernel left in memory, read through the scalar cache (a third of the latency of a
// vector load; nothing in these kernels writes it).
__device__ __forceinline__ int load_count(const int* p) {
  return *reinterpret_cast<const int __attribute__((address_space(4)))*>(reinterpret_cast<size_t>(p));
}

// ------------------------------------------------------------------------------------------------
// NT: C = A * B^T.  One workgroup = 4 waves stacked along M (16 rows each); every wave spans the
// whole 16*TN-wide column tile.  A stage is 32 k-columns.
// ------------------------------------------------------------------------------------------------
constexpr int NT_BK = 32;
constexpr int NT_P = 32;
// LDS rows are 32 floats = 8 chunks of 16 bytes, unpadded; chunk c of row r is stored at chunk position
// c ^ ((r >> 1) & 7).  Sixteen lanes that access the same logical chunk of sixteen consecutive rows (MFMA
// operand reads), or the eight chunks of two consecutive rows (stage stores), then cover all 64 banks once.
__device__ __forceinline__ int nt_swz(int row, int chunk) { return row * NT_P + ((chunk ^ ((row >> 1) & 7)) << 2); }

template <int TN>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, (TN <= 5 ? 4 : 2)))) void gemm_nt_kernel(NtGroup grp) {
  constexpr int BM = NT_BM, BN = 16 * TN;
  if ((int)blockIdx.x >= grp.gemm_wgs) {   // passengers after the products' workgroups: write-back scatter + SGD
    wb_sgd_block(grp.tail, blockIdx.x - grp.gemm_wgs);
    return;
  }
  // Up to two independent problems share a launch; the second one's workgroups follow the first one's.
  // The argument block is read through the kernel-argument segment (scalar loads at a computed offset).
  typedef const NtGroup __attribute__((address_space(4))) * GroupPtr;
  const GroupPtr gp = (GroupPtr)__builtin_amdgcn_kernarg_segment_ptr();
  const int pi = (gp->n > 1 && (int)blockIdx.x >= gp->p[1].wg_begin) ? 1 : 0;
  const auto& q = gp->p[pi];
  const float* __restrict__ A = q.A;
  const float* __restrict__ B = q.B;
  const float* __restrict__ bias = q.bias;
  float* __restrict__ C = q.C;
  const int lda = q.lda, ldb = q.ldb, ldc = q.ldc, N = q.N, Kp = q.Kp, n_store = q.n_store, relu = q.relu;
  const int col_tiles = q.col_tiles;
  int M = q.M;
  const int* m_dev = q.m_dev;
  RowAdd add;
  add.src = q.add.src; add.index = q.add.index; add.ld = q.add.ld; add.row0 = q.add.row0;
  add.gate = q.add.gate; add.ld_gate = q.add.ld_gate;
  TimeGradOut tg;
  tg.delta = q.tg.delta; tg.w = q.tg.w; tg.b = q.tg.b; tg.g_w = q.tg.g_w; tg.g_b = q.tg.g_b;
  GruBwdOut gb;
  gb.gates = q.gb.gates; gb.Hm = q.gb.Hm; gb.has = q.gb.has; gb.dgi = q.gb.dgi; gb.dgh = q.gb.dgh;
  gb.dm = q.gb.dm; gb.ldh = q.gb.ldh; gb.ld3 = q.gb.ld3;
  // Workgroups are dealt round-robin to the 8 XCDs, each with its own L2.  The column tiles of one row tile
  // read the same rows of A, so they are given consecutive slots of one XCD.
  const int block = (int)blockIdx.x - q.wg_begin;   // wg_begin is a multiple of 8
  const int xcd = block & 7, slot = block >> 3;
  const int row_tile = (slot / col_tiles) * 8 + xcd, col_tile = slot % col_tiles;
  if (m_dev != nullptr) M = min(M, load_count(m_dev));
  if (row_tile * BM >= M) return;   // uniform for the workgroup, before any barrier
  constexpr int A_PER = BM * 8 / 256, B_F4 = BN * 8;  // float4 loads per stage and thread
  constexpr int B_PER = (B_F4 + 255) / 256;
  // two stage buffers of A and of B; the finished tile is staged in the same memory for its row-wise stores
  __shared__ __attribute__((aligned(16))) float smem[2 * (BM + BN) * NT_P];
  float (*As)[BM * NT_P] = reinterpret_cast<float (*)[BM * NT_P]>(smem);
  float (*Bs)[BN * NT_P] = reinterpret_cast<float (*)[BN * NT_P]>(smem + 2 * BM * NT_P);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane & 15, lg = lane >> 4;
  const int m0 = row_tile * BM, n0 = col_tile * BN;

  floatx4 acc[TN];
#pragma unroll
  for (int b = 0; b < TN; ++b) acc[b] = floatx4{0.f, 0.f, 0.f, 0.f};

  // Row indices are clamped instead of guarded, so the hot loop has no branches: rows >= M and weight
  // rows >= N read valid memory whose products are dropped in the epilogue.
  // the k range of this column tile: all of it, or with a block-diagonal B the stages its blocks reach into
  int k_lo = 0, k_hi = Kp, k_end = q.k_live > 0 ? q.k_live : Kp;
  if (q.bd_n > 0) {
    const int h_lo = min(n0, N - 1) / q.bd_n, h_hi = (min(n0 + BN, N) - 1) / q.bd_n;
    k_lo = (h_lo * q.bd_k) & ~(NT_BK - 1);
    k_end = min(k_end, (h_hi + 1) * q.bd_k);
    k_hi = min(Kp, (k_end + NT_BK - 1) & ~(NT_BK - 1));
    if (k_hi <= k_lo) k_lo = max(k_hi - NT_BK, 0);   // (live columns end before the tile's blocks begin: one stage of zeros)
  }
  const float* pa[A_PER];
  const float* pb[B_PER];
#pragma unroll
  for (int u = 0; u < A_PER; ++u) {
    const int f = tid + u * 256;
    pa[u] = A + (size_t)min(m0 + (f >> 3), M - 1) * lda + (f & 7) * 4 + k_lo;
  }
#pragma unroll
  for (int u = 0; u < B_PER; ++u) {
    const int f = min(tid + u * 256, B_F4 - 1);
    pb[u] = B + (size_t)min(n0 + (f >> 3), N - 1) * ldb + (f & 7) * 4 + k_lo;
  }
  struct Regs {
    floatx4 a[A_PER], b[B_PER];
  };
  Regs r0, r1;  // the two register tile sets
  auto gload = [&](Regs& r, int k0) __attribute__((always_inline)) {
#pragma unroll
    for (int u = 0; u < A_PER; ++u) r.a[u] = *reinterpret_cast<const floatx4*>(pa[u] + k0);
#pragma unroll
    for (int u = 0; u < B_PER; ++u) r.b[u] = *reinterpret_cast<const floatx4*>(pb[u] + k0);
  };
  auto sstore = [&](const Regs& r, int buf) __attribute__((always_inline)) {
#pragma unroll
    for (int u = 0; u < A_PER; ++u) {
      const int f = tid + u * 256;
      *reinterpret_cast<floatx4*>(&As[buf][nt_swz(f >> 3, f & 7)]) = r.a[u];
    }
#pragma unroll
    for (int u = 0; u < B_PER; ++u) {
      const int f = tid + u * 256;
      if (B_F4 % 256 == 0 || f < B_F4) *reinterpret_cast<floatx4*>(&Bs[buf][nt_swz(f >> 3, f & 7)]) = r.b[u];
    }
  };
  // the last stage stops after its first slab when the live columns end there
  const int k_tail = (q.k_live > 0 || q.bd_n > 0) ? k_end - (k_hi - NT_BK) : NT_BK;
  const bool short_tail = k_tail > 0 && k_tail <= 16;
  auto compute = [&](int buf, bool last = false) __attribute__((always_inline)) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {  // two 16-wide k slabs per stage
      if (h == 1 && last && short_tail) break;
      const floatx4 a4 = *reinterpret_cast<const floatx4*>(&As[buf][nt_swz(wave * 16 + li, h * 4 + lg)]);
      floatx4 b4[TN];
#pragma unroll
      for (int b = 0; b < TN; ++b)
        b4[b] = *reinterpret_cast<const floatx4*>(&Bs[buf][nt_swz(b * 16 + li, h * 4 + lg)]);
#pragma unroll
      for (int b = 0; b < TN; ++b) acc[b] = __builtin_amdgcn_mfma_f32_16x16x4f32(a4.x, b4[b].x, acc[b], 0, 0, 0);
#pragma unroll
      for (int b = 0; b < TN; ++b) acc[b] = __builtin_amdgcn_mfma_f32_16x16x4f32(a4.y, b4[b].y, acc[b], 0, 0, 0);
#pragma unroll
      for (int b = 0; b < TN; ++b) acc[b] = __builtin_amdgcn_mfma_f32_16x16x4f32(a4.z, b4[b].z, acc[b], 0, 0, 0);
#pragma unroll
      for (int b = 0; b < TN; ++b) acc[b] = __builtin_amdgcn_mfma_f32_16x16x4f32(a4.w, b4[b].w, acc[b], 0, 0, 0);
    }
  };

  // Kp is a multiple of the stage depth.  Stage s lives in register set s & 1 until it is stored to LDS
  // buffer s & 1; loads run two stages ahead of the MFMAs.
  const int nk = (k_hi - k_lo) / NT_BK;
  // rows this lane writes: m0 + wave * 16 + lg * 4 + v.  Their gather-add source rows (or -1), and then the
  // values to add, are fetched now: two dependent loads that would otherwise sit between the last MFMA and
  // the stores.
  // The first two stages are asked for first; the index loads are four independent ones (clamped rows, no
  // branch between them: one wait, not four).
  gload(r0, 0);
  gload(r1, nk > 1 ? NT_BK : 0);
  int arow[4] = {-1, -1, -1, -1};
  if (add.src != nullptr) {
    const int row0 = m0 + wave * 16 + lg * 4;
    if (add.index != nullptr) {
      int idx[4];
#pragma unroll
      for (int v = 0; v < 4; ++v) idx[v] = add.index[min(row0 + v, M - 1)];
#pragma unroll
      for (int v = 0; v < 4; ++v) arow[v] = row0 + v < M ? idx[v] : -1;
    } else {
#pragma unroll
      for (int v = 0; v < 4; ++v) arow[v] = row0 + v < M ? row0 + v + add.row0 : -1;
    }
  }
  sstore(r0, 0);
  float addv[TN][4], bv[TN];
#pragma unroll
  for (int b = 0; b < TN; ++b) {
    const int col = n0 + b * 16 + li;
    bv[b] = (bias != nullptr && col < N) ? bias[col] : 0.f;
#pragma unroll
    for (int v = 0; v < 4; ++v)
      addv[b][v] = (add.src != nullptr && arow[v] >= 0 && col < N) ? add.src[(size_t)arow[v] * add.ld + col] : 0.f;
  }
  __syncthreads();
  int kt = 0;
  for (; kt + 3 < nk; kt += 2) {
    gload(r0, (kt + 2) * NT_BK);
    compute(0);
    sstore(r1, 1);
    __syncthreads();
    gload(r1, (kt + 3) * NT_BK);
    compute(1);
    sstore(r0, 0);
    __syncthreads();
  }
  // 1, 2 or 3 stages remain: kt (in LDS 0), kt+1 (in set 1), kt+2 (not loaded yet)
  const int rem = nk - kt;
  if (rem == 3) gload(r0, (kt + 2) * NT_BK);
  compute(0, rem == 1);
  if (rem >= 2) {
    sstore(r1, 1);
    __syncthreads();
    compute(1, rem == 2);
    if (rem == 3) {
      sstore(r0, 0);
      __syncthreads();
      compute(0, true);
    }
  }

  if (tg.g_w != nullptr) {
    // Time-encoding gradient epilogue: the tile is not stored.  Each lane multiplies its 4 rows x TN columns
    // by -sin(w_col delta_row + b_col) (the argument formed exactly as in the forward kernels), sums over its
    // rows, then over the four lane groups (shuffles) and the four waves (LDS).
    __syncthreads();   // all waves are done reading the last stage: the stage buffer becomes scratch
    float* red = &As[0][0];   // [2][4 waves][BN]
    double dl[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int row = m0 + wave * 16 + lg * 4 + v;
      dl[v] = row < M ? tg.delta[row] : 0.0;
    }
#pragma unroll
    for (int b = 0; b < TN; ++b) {
      const int col = n0 + b * 16 + li;
      float sw = 0.f, sb = 0.f;
      if (col < N) {
        const double wv = (double)tg.w[col], bv = (double)tg.b[col];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          if (m0 + wave * 16 + lg * 4 + v < M) {
            float sn, cs;
            sincos_reduced(fma(wv, dl[v], bv), sn, cs);
            const float t = -acc[b][v] * sn;
            sb += t;
            sw += t * (float)dl[v];
          }
        }
      }
      sw += __shfl_xor(sw, 16); sw += __shfl_xor(sw, 32);
      sb += __shfl_xor(sb, 16); sb += __shfl_xor(sb, 32);
      if (lg == 0) {
        red[wave * BN + b * 16 + li] = sw;
        red[(4 + wave) * BN + b * 16 + li] = sb;
      }
    }
    __syncthreads();
    for (int c = tid; c < BN; c += 256) {
      const int col = n0 + c;
      if (col < N) {
        atomicAdd(tg.g_w + col, red[c] + red[BN + c] + red[2 * BN + c] + red[3 * BN + c]);
        atomicAdd(tg.g_b + col, red[4 * BN + c] + red[5 * BN + c] + red[6 * BN + c] + red[7 * BN + c]);
      }
    }
    return;
  }
  if (gb.dgi != nullptr) {
    // GRU gates backward epilogue: acc is the gradient reaching s' = (1 - z) n + z h.  All loads first, then
    // arithmetic and stores: a load between two stores would wait for the earlier store to complete.
    bool hs[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int row = m0 + wave * 16 + lg * 4 + v;
      hs[v] = row < M && gb.has[row] != 0;
    }
    constexpr int GB = TN < 2 ? TN : 2;   // column blocks per group (bounds the registers of wide tiles)
#pragma unroll
    for (int b0 = 0; b0 < TN; b0 += GB) {
      float gr[GB][4], gz[GB][4], gn[GB][4], ghn[GB][4], gh[GB][4];
#pragma unroll
      for (int bb = 0; bb < GB; ++bb) {
        const int col = n0 + (b0 + bb) * 16 + li;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int row = m0 + wave * 16 + lg * 4 + v;
          gr[bb][v] = gz[bb][v] = gn[bb][v] = ghn[bb][v] = gh[bb][v] = 0.f;
          if (b0 + bb < TN && col < N && hs[v]) {
            const float* g = gb.gates + (size_t)row * 4 * gb.ldh;
            gr[bb][v] = g[col]; gz[bb][v] = g[gb.ldh + col]; gn[bb][v] = g[2 * gb.ldh + col];
            ghn[bb][v] = g[3 * gb.ldh + col];
            gh[bb][v] = gb.Hm[(size_t)row * gb.ldh + col];
          }
        }
      }
#pragma unroll
      for (int bb = 0; bb < GB; ++bb) {
        const int b = b0 + bb;
        const int col = n0 + b * 16 + li;
        if (b >= TN || col >= N) continue;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int row = m0 + wave * 16 + lg * 4 + v;
          if (row >= M) continue;
          float drp = 0.f, dzp = 0.f, dnp = 0.f, dnr = 0.f;
          if (hs[v]) {
            const float ds = acc[b < TN ? b : 0][v];
            const float r = gr[bb][v], z = gz[bb][v], nn = gn[bb][v], hn = ghn[bb][v], h = gh[bb][v];
            const float dn = ds * (1.0f - z);
            const float dz = ds * (h - nn);
            dnp = dn * (1.0f - nn * nn);
            const float dr = dnp * hn;
            dzp = dz * z * (1.0f - z);
            drp = dr * r * (1.0f - r);
            dnr = dnp * r;
          }
          float* a = gb.dgi + (size_t)row * gb.ld3;
          float* h_ = gb.dgh + (size_t)row * gb.ld3;
          a[col] = drp; a[gb.dm + col] = dzp; a[2 * gb.dm + col] = dnp;
          h_[col] = drp; h_[gb.dm + col] = dzp; h_[2 * gb.dm + col] = dnr;
        }
      }
    }
    return;
  }
  // A lane holds 4 rows x 16-column-strided pieces of the tile: stored from here, every instruction would write
  // 64-byte pieces of four rows.  The tile goes through LDS instead and leaves as whole rows, 16 bytes per lane.
  const bool rowwise = (n_store & 3) == 0 && (ldc & 3) == 0 && (reinterpret_cast<size_t>(C) & 15) == 0;
  constexpr int CP = BN + 4;   // pitch = 4 mod 16 floats: the 4 x 16 lanes of a store hit 64 different banks
  unsigned closed = 0u;   // bit 4 b + v: the gate of that element is closed (result 0)
  if (add.gate != nullptr) {   // all gate values first: no load, and no wait for one, between the stores below
#pragma unroll
    for (int b = 0; b < TN; ++b) {
      const int col = n0 + b * 16 + li;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int row = m0 + wave * 16 + lg * 4 + v;
        if (col < N && row < M && !(add.gate[(size_t)row * add.ld_gate + col] > 0.f)) closed |= 1u << (4 * b + v);
      }
    }
  }
#pragma unroll
  for (int b = 0; b < TN; ++b) {
    const int col = n0 + b * 16 + li;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int row = m0 + wave * 16 + lg * 4 + v;
      const bool live = col < N && row < M && ((closed >> (4 * b + v)) & 1u) == 0u;
      const float x = acc[b][v] + bv[b] + addv[b][v];
      acc[b][v] = live ? (relu ? fmaxf(x, 0.f) : x) : 0.f;
    }
  }
  if (q.colsum != nullptr) {   // column sums of the tile: a lane's four rows, then the four lane groups; one atomic per wave
    float* cs = q.colsum + (size_t)((row_tile * 4 + wave) & (q.colsum_rows - 1)) * N;
#pragma unroll
    for (int b = 0; b < TN; ++b) {
      float t = acc[b][0] + acc[b][1] + acc[b][2] + acc[b][3];
      t += __shfl_xor(t, 16);
      t += __shfl_xor(t, 32);
      const int col = n0 + b * 16 + li;
      if (lg == 0 && col < N) atomicAdd(cs + col, t);
    }
  }
  if (!rowwise) {
#pragma unroll
    for (int b = 0; b < TN; ++b) {
      const int col = n0 + b * 16 + li;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int row = m0 + wave * 16 + lg * 4 + v;
        if (col < n_store && row < M) C[(size_t)row * ldc + col] = acc[b][v];
      }
    }
    return;
  }
  __syncthreads();   // all waves are done reading the last stage
#pragma unroll
  for (int b = 0; b < TN; ++b)
#pragma unroll
    for (int v = 0; v < 4; ++v) smem[(wave * 16 + lg * 4 + v) * CP + b * 16 + li] = acc[b][v];
  __syncthreads();
  constexpr int F4_ROW = BN / 4, F4_ALL = BM * F4_ROW;
#pragma unroll
  for (int u = 0; u < (F4_ALL + 255) / 256; ++u) {
    const int f = tid + u * 256;
    const int r = f / F4_ROW, c = (f - r * F4_ROW) * 4;
    if ((F4_ALL % 256 == 0 || f < F4_ALL) && m0 + r < M && n0 + c < n_store)
      *reinterpret_cast<floatx4*>(C + (size_t)(m0 + r) * ldc + n0 + c) = *reinterpret_cast<const floatx4*>(&smem[r * CP + c]);
  }
}

// Column-tile width in 16-wide MFMA blocks, from sweeps on MI355X: problems of a few thousand rows want the
// narrowest tiles (many short workgroups, all resident at once), tens of thousands of rows want 2 blocks,
// and only beyond that do wider tiles (less re-reading of A) pay off.
static int nt_tile_blocks(int M, int n_store) {
  const int nb = (n_store + 15) / 16;
  int best = 1;
  if (M > 4096 && M <= 65536) {
#ifndef TGNN_NT_MID_TILE
#define TGNN_NT_MID_TILE 2
#endif
    best = TGNN_NT_MID_TILE;
  } else if (M > 65536) {
    float best_cost = 1e30f;
    static const int cand[] = {5, 4, 7, 2};
    for (int c : cand) {
      const float cost = (float)(((nb + c - 1) / c) * c) / nb;   // padded / useful columns
      if (cost < best_cost - 1e-6f) { best_cost = cost; best = c; }
    }
  }
  return best;
}

void gemm_nt_group(const NtProblem* probs, int n, hipStream_t s, const WbArgs* tail) {
  NtGroup g;
  memset(&g, 0, sizeof(g));
  int tail_blocks = 0;
  if (tail != nullptr) {
    g.tail = *tail;
    tail_blocks = wb_total_blocks(*tail);
  }
  int tn = 0, total = 0;
  for (int i = 0; i < n && g.n < 2; ++i) {
    NtProblem p = probs[i];
    if (p.M <= 0 || p.N <= 0) continue;
    if (p.n_store < p.N) p.n_store = p.N;
    if (tn == 0) tn = nt_tile_blocks(p.M, p.n_store);   // the first problem decides the tile width
    p.col_tiles = (p.n_store + 16 * tn - 1) / (16 * tn);
    p.wg_begin = total;
    total += p.col_tiles * (((p.M + NT_BM - 1) / NT_BM + 7) & ~7);
    g.p[g.n++] = p;
  }
  if (g.n == 0 && tail_blocks == 0) return;
  if (tn == 0) tn = 1;
  g.gemm_wgs = total;
  total += tail_blocks;
#define TGNN_NT_CASE(TNV) \
  case TNV: hipLaunchKernelGGL((gemm_nt_kernel<TNV>), dim3(total), dim3(256), 0, s, g); break;
  switch (tn) {
    TGNN_NT_CASE(7)
    TGNN_NT_CASE(5)
    TGNN_NT_CASE(4)
    TGNN_NT_CASE(2)
    default:
    TGNN_NT_CASE(1)
  }
#undef TGNN_NT_CASE
}

void gemm_nt(const float* A, int lda, const float* B, int ldb, const float* bias, float* C, int ldc, int M, int N,
             int Kp, int n_store, bool relu, hipStream_t s, const int* m_dev, const RowAdd& add, const TimeGradOut& tg,
             const GruBwdOut& gb) {
  const NtProblem p = nt_problem(A, lda, B, ldb, bias, C, ldc, M, N, Kp, n_store, relu, m_dev, add, tg, gb);
  gemm_nt_group(&p, 1, s);
}

// ------------------------------------------------------------------------------------------------
// TN with accumulation: G[n, k] += sum_m D[m, n] * A[m, k], bias[n] += sum_m D[m, n].
// Both operands are m-major.  The MFMA sums over four m values per instruction (one per lane group), and
// which n (k) a lane feeds is free as long as the result is read back the same way: lane (li, lg) takes TD
// consecutive floats D[m][n0 + TD*li ..] and TA consecutive floats A[m][k0 + TA*li ..] of row m = 4 step + lg
// and issues TD*TA MFMAs from them, instruction (t, u) covering the strided columns n = n0 + TD*i + t,
// k = k0 + TA*j + u.  Those two runs are one vector load each straight from global memory (a lane group reads
// one contiguous piece of a row), and no element is used by more than one wavefront, so nothing is staged in
// LDS and the main loop has no barrier: every wavefront streams its own rows, several steps of loads ahead.
// A workgroup of TN_W wavefronts owns a (16 TD) x (16 TA) tile of G (64 x 64 in the bulk, narrower pieces
// at the right and bottom edges so that little of the tile is padding) over a chunk of the rows; its
// wavefronts take the 4-row steps of the chunk in turn, and their partial tiles are added in LDS before one
// float atomic per element goes to memory.  The reduction over m is split over workgroups.
// The bias gradient rides along as column K of A, which the loader replaces by ones.
// ------------------------------------------------------------------------------------------------
constexpr int TT = 64;        // bulk tile edge
#ifndef TGNN_TN_WAVES
#define TGNN_TN_WAVES 8
#endif
constexpr int TN_W = TGNN_TN_WAVES;   // wavefronts per workgroup
constexpr int TN_AHEAD = 4;   // 4-row steps whose loads a wavefront keeps in flight
constexpr int TN_ROWS = 32;   // row chunks are multiples of this

// A length is cut into 64-wide pieces plus one narrower one (16, 32 or again 64 wide) for the remainder.  (With
// TGNN_TN_SPLIT48 a remainder of 33 .. 48 becomes a 32- and a 16-wide piece instead of a padded 64-wide one: fewer
// MFMAs, one more tile; measured on MI355X the extra tile costs slightly more than the padding.)
#ifndef TGNN_TN_SPLIT48
#define TGNN_TN_SPLIT48 0
#endif
__host__ __device__ inline int tn_pieces(int len) {
  const int r = len % TT;
  return len / TT + (r == 0 ? 0 : (TGNN_TN_SPLIT48 && r > 32 && r <= 48) ? 2 : 1);
}
__device__ __forceinline__ void tn_piece(int len, int idx, int& off, int& width) {
  const int full = len / TT;
  if (idx < full) { off = idx * TT; width = TT; return; }
  const int r = len - full * TT;
  off = full * TT;
  if (r <= 16) width = 16;
  else if (r <= 32) width = 32;
  else if (TGNN_TN_SPLIT48 && r <= 48) { if (idx == full) width = 32; else { off += 32; width = 16; } }
  else width = TT;
}
// Column window of D that one head of head_n columns is tiled over (its start is rounded down to 16 bytes).
__host__ __device__ inline int tn_head_width(int head_n) { return head_n + 3; }

template <int TD> struct FragT;
template <> struct FragT<1> { typedef float type; };
template <> struct FragT<2> { typedef float type __attribute__((ext_vector_type(2))); };
template <> struct FragT<4> { typedef float type __attribute__((ext_vector_type(4))); };
template <int T> __device__ __forceinline__ float frag_get(const typename FragT<T>::type& f, int i) { return f[i]; }
template <> __device__ __forceinline__ float frag_get<1>(const float& f, int) { return f; }
template <int T> __device__ __forceinline__ void frag_set(typename FragT<T>::type& f, int i, float x) { f[i] = x; }
template <> __device__ __forceinline__ void frag_set<1>(float& f, int, float x) { f = x; }
template <int T> __device__ __forceinline__ typename FragT<T>::type frag_zero() {
  typename FragT<T>::type f;
#pragma unroll
  for (int i = 0; i < T; ++i) frag_set<T>(f, i, 0.f);
  return f;
}

// One global load of T floats per lane, issued without a wait; tn_wait_loads<N> then waits until at most N of
// the loads issued so far are pending and ties the registers to that wait, so that no use can move above it.
template <int T> __device__ __forceinline__ void tn_issue_load(typename FragT<T>::type& r, const float* p);
template <> __device__ __forceinline__ void tn_issue_load<4>(FragT<4>::type& r, const float* p) {
  asm volatile("global_load_dwordx4 %0, %1, off" : "=&v"(r) : "v"(p) : "memory");
}
template <> __device__ __forceinline__ void tn_issue_load<2>(FragT<2>::type& r, const float* p) {
  asm volatile("global_load_dwordx2 %0, %1, off" : "=&v"(r) : "v"(p) : "memory");
}
template <> __device__ __forceinline__ void tn_issue_load<1>(float& r, const float* p) {
  asm volatile("global_load_dword %0, %1, off" : "=&v"(r) : "v"(p) : "memory");
}
template <int N, class FD, class FA> __device__ __forceinline__ void tn_wait_loads(FD& d, FA& a) {
  asm volatile("s_waitcnt vmcnt(%2)" : "+v"(d), "+v"(a) : "n"(N));
}

// Where partial-tile element (t, u, v) of lane (li, lg) lives in a reduction buffer: element-major, lane-minor
// (stores of one instruction touch 64 consecutive words), with the lane rotated by 16 u so that the final
// pass, which walks a row of the tile (li and u vary, lg fixed), also touches 64 different words.
template <int TA>
__device__ __forceinline__ int tn_slot(int t, int u, int v, int li, int lg) {
  return ((t * TA + u) * 4 + v) * 64 + ((lg * 16 + li + 16 * u) & 63);
}

template <int TD, int TA>
__device__ __forceinline__ void tn_tile(const float* __restrict__ D, const float* __restrict__ A, int ldd, int lda, int dw,
                                        int aw, int n_lo, int N, int K, float* p00, float* p01, float* p10, float* p11,
                                        int ld00, int ld01, int ld10, int ld11, int n_split, int k_split, float* bias0,
                                        float* bias1, int M, int m_lo, int m_hi, int n0, int k0, float* lds) {
  typedef typename FragT<TD>::type FD;
  typedef typename FragT<TA>::type FA;
  const bool with_bias = bias0 != nullptr || bias1 != nullptr;   // column K of A reads as ones
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: loop bounds stay scalar
  const int li = lane & 15, lg = lane >> 4;

  floatx4 acc[TD][TA];
#pragma unroll
  for (int t = 0; t < TD; ++t)
#pragma unroll
    for (int u = 0; u < TA; ++u) acc[t][u] = floatx4{0.f, 0.f, 0.f, 0.f};

  // Column offsets are clamped into the row (results of columns >= N or > K are dropped at the end); rows
  // >= m_hi are clamped and D is zeroed there by a select when the step is used.
  const int c_nom = k0 + TA * li;
  const float* pd = D + min(n0 + TD * li, dw - TD);   // dw, aw: columns that may be read from D, A (<= the pitch)
  const float* pa = A + min(c_nom, aw - TA);
  const int one_comp = (with_bias && K >= c_nom && K < c_nom + TA) ? K - c_nom : -1;
  const int n_steps = (m_hi - m_lo + 3) >> 2;

  // The loads are issued as inline assembly and waited for by count: left to itself the compiler sinks them
  // next to their uses and the wavefront then waits out the full memory latency at every step.  Loads return in
  // order, so when slot p is needed only the loads of the other TN_AHEAD - 1 slots (two each) may be pending.
  // 4-row steps whose loads a wavefront keeps in flight: a step of a narrow tile has few MFMAs to hide the
  // memory latency behind, so more of them are kept in flight.
  constexpr int AH = TD * TA >= 16 ? TN_AHEAD : TD * TA >= 8 ? TN_AHEAD + 2 : 2 * TN_AHEAD;
  FD fd[AH];
  FA fa[AH];
  auto issue = [&](int step, FD& d, FA& a) __attribute__((always_inline)) {
    const size_t m = (size_t)min(m_lo + 4 * step + lg, M - 1);
    tn_issue_load<TD>(d, pd + m * ldd);
    tn_issue_load<TA>(a, pa + m * lda);
  };
  auto use = [&](int step, FD d, FA a) __attribute__((always_inline)) {
    if (m_lo + 4 * step + lg >= m_hi) d = frag_zero<TD>();   // rows out of range: zeros times whatever A holds
    if (one_comp >= 0) {
#pragma unroll
      for (int u = 0; u < TA; ++u)
        if (one_comp == u) frag_set<TA>(a, u, 1.f);
    }
#pragma unroll
    for (int t = 0; t < TD; ++t)
#pragma unroll
      for (int u = 0; u < TA; ++u)
        acc[t][u] = __builtin_amdgcn_mfma_f32_16x16x4f32(frag_get<TD>(d, t), frag_get<TA>(a, u), acc[t][u], 0, 0, 0);
  };

  // Steps are not dealt out in advance beyond the first TN_AHEAD per wavefront: a wavefront that is done with a
  // step claims the next free one from a counter in LDS.  The wavefronts of a workgroup share their SIMDs
  // unevenly (the oldest wins the MFMA pipe), and with a fixed split the youngest would still be at work, alone
  // and unable to hide its load latency, long after the others had reached the barrier below.
  int* next_step = reinterpret_cast<int*>(lds + (TN_W / 2) * TT * TT);
  auto claim = [&]() __attribute__((always_inline)) {
    int v = 0;
    if (lane == 0) v = atomicAdd(next_step, 1);
    return __builtin_amdgcn_readfirstlane(v);
  };
  int sidx[AH];   // the step each slot holds; claims only grow, so a slot past the end means all later are
#pragma unroll
  for (int p = 0; p < AH; ++p) {
    sidx[p] = wave + p * TN_W;
    issue(sidx[p], fd[p], fa[p]);   // past the end: clamped rows, unused
  }
  if (tid == 0) *next_step = TN_W * AH;   // (after the first loads are on their way)
  __syncthreads();
  int nxt = claim();
  // slot 0 holds the oldest claim: once that is past the end, so are the others
  while (sidx[0] < n_steps) {
#pragma unroll
    for (int p = 0; p < AH; ++p) {   // (unrolled: the slots are registers)
      tn_wait_loads<2 * (AH - 1)>(fd[p], fa[p]);
      if (sidx[p] < n_steps) use(sidx[p], fd[p], fa[p]);
      sidx[p] = nxt;
      issue(nxt, fd[p], fa[p]);
      nxt = claim();
    }
  }
  // every issued load has to land before its registers are given to anything else
#pragma unroll
  for (int p = 0; p < AH; ++p) tn_wait_loads<0>(fd[p], fa[p]);

  // Add the wavefronts' partial tiles in LDS: the lower half of the wavefronts store theirs into a buffer
  // each, the upper half add theirs on top, then every thread sums the buffers for its elements and issues
  // one atomic per element.  acc[t][u][v] of lane (li, lg) is n = TD (4 lg + v) + t, k = TA li + u of the tile.
  constexpr int TW = 16 * TA, TILE = 16 * TD * TW, NB = TN_W / 2;
  float* red = lds + (wave % NB) * TILE;
  if (wave < NB) {
#pragma unroll
    for (int t = 0; t < TD; ++t)
#pragma unroll
      for (int u = 0; u < TA; ++u)
#pragma unroll
        for (int v = 0; v < 4; ++v) red[tn_slot<TA>(t, u, v, li, lg)] = acc[t][u][v];
  }
  __syncthreads();
  if (wave >= NB) {
#pragma unroll
    for (int t = 0; t < TD; ++t)
#pragma unroll
      for (int u = 0; u < TA; ++u)
#pragma unroll
        for (int v = 0; v < 4; ++v) red[tn_slot<TA>(t, u, v, li, lg)] += acc[t][u][v];
  }
  __syncthreads();
  constexpr int NT = 64 * TN_W;
#pragma unroll
  for (int i = 0; i < (TILE + NT - 1) / NT; ++i) {
    const int e = tid + i * NT;
    if (TILE % NT != 0 && e >= TILE) break;
    const int tn = e / TW, tk = e % TW;           // position in the tile
    const int n = n0 + tn, k = k0 + tk;
    if (n < n_lo || n >= N || k > K) continue;
    const int slot = tn_slot<TA>(tn % TD, tk % TA, (tn / TD) & 3, tk / TA, tn / (4 * TD));
    float x = 0.f;
#pragma unroll
    for (int b = 0; b < NB; ++b) x += lds[b * TILE + slot];
    // (selects instead of indexing: a dynamically indexed local array would live in scratch memory)
    const bool ns = n >= n_split;
    const int nn = n - (ns ? n_split : 0);
    if (k == K) {
      float* const bias = ns ? bias1 : bias0;
      if (bias != nullptr) atomicAdd(bias + nn, x);
    } else {
      const bool ks = k >= k_split;
      float* base = ns ? (ks ? p11 : p10) : (ks ? p01 : p00);
      const int ld = ns ? (ks ? ld11 : ld10) : (ks ? ld01 : ld00);
      atomicAdd(base + (size_t)nn * ld + (k - (ks ? k_split : 0)), x);
    }
  }
}

static_assert(sizeof(TnGroup) <= 4096, "the group travels as a kernel argument");
__global__ __launch_bounds__(64 * TN_W) void gemm_tn_kernel(TnGroup grp) {
  // Several independent problems share one launch (all weight gradients of a step): find this workgroup's.
  // The argument block is indexed through the kernel-argument segment itself (scalar loads at a computed
  // offset); indexing the by-value parameter would make the compiler spill the whole block to scratch.
  typedef const TnGroup __attribute__((address_space(4))) * GroupPtr;
  const GroupPtr gp = (GroupPtr)__builtin_amdgcn_kernarg_segment_ptr();
  const int xcd = blockIdx.x & 7, pos = blockIdx.x >> 3;
  // (a loop over the problems with its scalar loads one after the other took 5 us before the first row was asked for)
  typedef int int16v __attribute__((ext_vector_type(16)));
  typedef unsigned uint4v __attribute__((ext_vector_type(4)));
  const int16v qb = *reinterpret_cast<const int16v __attribute__((address_space(4)))*>(&gp->qbegin[xcd][0]);
  const uint4v qp = *reinterpret_cast<const uint4v __attribute__((address_space(4)))*>(&gp->qprob[0]);
  int slot = -1, begin = 0, end = 0;
#pragma unroll
  for (int t = 0; t < TN_MAX_GROUP; ++t)
    if (pos >= qb[t]) { slot = t; begin = qb[t]; end = qb[t + 1]; }
  if (slot < 0 || slot >= gp->n || pos >= end) return;   // this XCD's queue is shorter than the longest one
  unsigned word = qp[0];
#pragma unroll
  for (int t = 1; t < 4; ++t)
    if ((slot >> 2) == t) word = qp[t];
  const int pi = (word >> (8 * (slot & 3))) & 255u;
  const int local = pos - begin;
  const auto& q = gp->p[pi];
  const int v = (xcd + q.rot) & 7;
  const int tiles = q.tiles, chunks = q.chunks, N = q.N, K = q.K;
  int M = q.M, m_chunk = q.m_chunk;
  const int* m_dev = q.m_dev;
  float* const bias0 = q.out.bias[0];
  const bool with_bias = bias0 != nullptr || q.out.bias[1] != nullptr;
  const int chunk = (local / tiles) * 8 + v;
  int tile = local % tiles;
  if (m_dev != nullptr) {  // row count known only on the device: split it evenly over the launched chunks
    M = min(M, load_count(m_dev));
    m_chunk = ((M + chunks - 1) / chunks + TN_ROWS - 1) / TN_ROWS * TN_ROWS;
  }
  if (chunk * m_chunk >= M) return;   // uniform for the workgroup, before any barrier
  __shared__ __attribute__((aligned(16))) float lds[(TN_W / 2) * TT * TT + 4];   // reduction buffers + step counter
  int m_lo = chunk * m_chunk;
  int m_hi = min(M, m_lo + m_chunk);
  // A problem with per-head blocks is H problems of the same shape side by side: head h multiplies columns
  // [h head_n, (h + 1) head_n) of D with columns [h head_k, h head_k + head_cols) of A.  Its column window of D
  // starts at the 16-byte boundary below the head's first column; the columns in front are not written.
  const float* Dp = q.D;
  const float* Ap = q.A;
  float* p00 = q.out.p[0][0];
  int dw = q.ldd, aw = q.lda, n_lo = 0, n_hi = N, n_tiling = N, Kt = K;
  if (q.out.head_k > 0) {
    const int per_head = tiles / q.heads, h = tile / per_head;
    tile -= h * per_head;
    const int first = h * q.out.head_n, a0 = first & ~3;
    Dp += a0; dw -= a0;
    Ap += h * q.out.head_k; aw -= h * q.out.head_k;
    p00 += (size_t)a0 * q.out.ld[0][0];
    n_lo = first - a0; n_hi = n_lo + q.out.head_n;
    n_tiling = tn_head_width(q.out.head_n);
    Kt = q.out.head_cols;
  }
  const int Kb = Kt + (with_bias ? 1 : 0);
  const int k_tiles = tn_pieces(Kb);
  const int np = tile / k_tiles, kp = tile - np * k_tiles;
  int n0, wn, k0, wk;
  tn_piece(n_tiling, np, n0, wn);
  tn_piece(Kb, kp, k0, wk);
#define TGNN_TN_CASE(WN, WK)                                                                                          \
  if (wn == WN && wk == WK) {                                                                                         \
    tn_tile<WN / 16, WK / 16>(Dp, Ap, q.ldd, q.lda, dw, aw, n_lo, n_hi, Kt, p00, q.out.p[0][1], q.out.p[1][0],          \
                              q.out.p[1][1], q.out.ld[0][0], q.out.ld[0][1], q.out.ld[1][0], q.out.ld[1][1],            \
                              q.out.n_split, q.out.k_split, bias0, q.out.bias[1], M, m_lo, m_hi, n0, k0, lds);      \
    return;                                                                                                           \
  }
  TGNN_TN_CASE(64, 64) TGNN_TN_CASE(64, 32) TGNN_TN_CASE(64, 16)
  TGNN_TN_CASE(32, 64) TGNN_TN_CASE(32, 32) TGNN_TN_CASE(32, 16)
  TGNN_TN_CASE(16, 64) TGNN_TN_CASE(16, 32) TGNN_TN_CASE(16, 16)
#undef TGNN_TN_CASE
}

void TnBatch::add(const float* D, int ldd, const float* A, int lda, int M, int N, int K, const OutMap& out,
                  const int* m_dev) {
  // the loader clamps column offsets to ld - 4 and reads whole float4s: pitches below 4 (or below the logical
  // width) would send it out of bounds
  // (K == 0 with a bias output: column sums of D only; A is then any readable matrix of M rows)
  const bool with_bias = out.bias[0] != nullptr || out.bias[1] != nullptr;
  if (M <= 0 || N <= 0 || K < 0 || (K == 0 && !with_bias) || g.n >= TN_MAX_GROUP || ldd < 4 || lda < 4 || (ldd & 3) ||
      (lda & 3) || N > ldd || K > lda)
    return;
  TnProblem& p = g.p[g.n];
  p.D = D; p.ldd = ldd; p.A = A; p.lda = lda; p.M = M; p.N = N; p.K = K;
  if (out.head_k > 0) {   // H problems of head_n x head_cols side by side
    p.heads = N / out.head_n;
    p.tiles = p.heads * tn_pieces(tn_head_width(out.head_n)) * tn_pieces(out.head_cols);
  } else {
    p.heads = 1;
    p.tiles = tn_pieces(N) * tn_pieces(K + (out.bias[0] != nullptr || out.bias[1] != nullptr ? 1 : 0));
  }
  p.m_dev = m_dev; p.out = out;
  g.n++;
}

// Chunking and placement.  A workgroup's life is a first wait for data, its share of the rows at the pace of
// the MFMA pipes it shares, and a reduction with one float atomic per tile element; a launch takes as long
// as the number of rounds the chip needs to hold all workgroups times the life of one.  So a small launch
// (all weight gradients of a step on a few thousand rows) gets the largest number of row chunks with which
// no XCD queue exceeds TN_WGS_PER_XCD workgroups, and a large one gets chunks of TN_MAX_ROWS rows and runs
// in rounds.  An XCD holds 64 workgroups at once (two per compute unit); workgroups with narrow edge tiles
// finish early, and queues of 72 to 88 measured best on MI355X for the weight gradients of a 600-event step
// (64 and 96: a fifth slower).  All problems of a launch use the same chunk length.
// What in-kernel timestamps say about such a launch: a workgroup sees its first rows 3 to 5 us after it starts
// (argument block, device-side row count, then the rows: three dependent round trips), a wavefront then takes
// 0.5 to 0.8 us per 4-row step whatever the tile width, because the loads of narrow tiles are 64- to 256-byte
// pieces of four rows and the texture addresser, not the MFMA pipe, is what the 16 wavefronts of a compute unit
// queue for; the reduction and the atomics take 2 to 3 us.
#ifndef TGNN_TN_MAX_ROWS
#define TGNN_TN_MAX_ROWS 1024
#endif
#ifndef TGNN_TN_WGS_PER_XCD
#define TGNN_TN_WGS_PER_XCD 80
#endif
constexpr int TN_MAX_ROWS = TGNN_TN_MAX_ROWS;
constexpr int TN_WGS_PER_XCD = TGNN_TN_WGS_PER_XCD;

// Chunks of `rows_per_chunk` rows for every problem, then the placement on the eight XCDs: problems in order
// of decreasing size, each rotated so that the XCDs which receive one chunk more than the others are the least
// loaded ones so far.  Returns the length of the longest XCD queue.
static int tn_place(TnGroup& g, const int* rows, int rows_per_chunk) {
  for (int i = 0; i < g.n; ++i) {
    TnProblem& p = g.p[i];
    int chunks = (rows[i] + rows_per_chunk - 1) / rows_per_chunk;
    p.m_chunk = ((p.M + chunks - 1) / chunks + TN_ROWS - 1) / TN_ROWS * TN_ROWS;
    if (p.m_dev == nullptr) chunks = (p.M + p.m_chunk - 1) / p.m_chunk;
    p.chunks = chunks;
  }
  int order[TN_MAX_GROUP], load[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int i = 0; i < g.n; ++i) order[i] = i;
  std::sort(order, order + g.n, [&](int a, int b) { return g.p[a].tiles * g.p[a].chunks > g.p[b].tiles * g.p[b].chunks; });
  for (int oi = 0; oi < g.n; ++oi) {
    TnProblem& p = g.p[order[oi]];
    int cnt[8];
    for (int v = 0; v < 8; ++v) cnt[v] = p.chunks > v ? p.tiles * ((p.chunks - v + 7) / 8) : 0;
    int best_rot = 0, best_max = 1 << 30;
    for (int r = 0; r < 8; ++r) {
      int mx = 0;
      for (int x = 0; x < 8; ++x) mx = std::max(mx, load[x] + cnt[(x + r) & 7]);
      if (mx < best_max) { best_max = mx; best_rot = r; }
    }
    p.rot = best_rot;
    g.qprob[oi] = (unsigned char)order[oi];
    for (int x = 0; x < 8; ++x) {
      p.lane_begin[x] = load[x];
      g.qbegin[x][oi] = load[x];
      load[x] += cnt[(x + best_rot) & 7];
    }
  }
  for (int x = 0; x < 8; ++x) {
    g.qbegin[x][g.n] = load[x];
    for (int t = g.n + 1; t < 16; ++t) g.qbegin[x][t] = 0x7fffffff;
  }
  return *std::max_element(load, load + 8);
}

void TnBatch::launch(hipStream_t s) {
  if (g.n == 0) return;
  const int per_xcd = TN_WGS_PER_XCD;
  const int max_rows = TN_MAX_ROWS;
  int rows[TN_MAX_GROUP];
  // a row count that lives on the device (distinct nodes of a step) is usually a small part of its bound
  for (int i = 0; i < g.n; ++i)
    rows[i] = g.p[i].m_dev == nullptr ? g.p[i].M
              : dev_rows_est > 0      ? std::min(g.p[i].M, dev_rows_est)
                                      : (g.p[i].M + 7) / 8;
  // smallest chunk length (in units of TN_ROWS) whose placement fits the chip at once, by bisection
  int lo = 4, hi = max_rows / TN_ROWS;   // lo: at least four steps per wavefront; hi: taken if nothing smaller fits
  int longest = tn_place(g, rows, hi * TN_ROWS);
  if (longest <= per_xcd) {
    while (lo < hi) {
      const int mid = (lo + hi) / 2;
      if (tn_place(g, rows, mid * TN_ROWS) <= per_xcd) hi = mid; else lo = mid + 1;
    }
    longest = tn_place(g, rows, hi * TN_ROWS);
  }
  const int total_wgs = 8 * longest;
  hipLaunchKernelGGL(gemm_tn_kernel, dim3(total_wgs), dim3(64 * TN_W), 0, s, g);
  g.n = 0;
}

void gemm_tn_acc(const float* D, int ldd, const float* A, int lda, int M, int N, int K, const OutMap& out,
                 hipStream_t s, const int* m_dev) {
  TnBatch b;
  b.add(D, ldd, A, lda, M, N, K, out, m_dev);
  b.launch(s);
}

}  // namespace tgnn
