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

#include "tgnn_internal.h"

namespace tgnn {

typedef float floatx4 __attribute__((ext_vector_type(4)));

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
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, (TN <= 5 ? 4 : 2)))) void gemm_nt_kernel(const float* __restrict__ A, int lda,
                                                      const float* __restrict__ B, int ldb,
                                                      const float* __restrict__ bias, float* __restrict__ C, int ldc,
                                                      int M, int N, int Kp, int n_store, int relu,
                                                      const int* __restrict__ m_dev, int col_tiles) {
  constexpr int BM = 64, BN = 16 * TN;
  // Workgroups are dealt round-robin to the 8 XCDs, each with its own L2.  The column tiles of one row tile
  // read the same rows of A, so they are given consecutive slots of one XCD.
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int row_tile = (slot / col_tiles) * 8 + xcd, col_tile = slot % col_tiles;
  if (m_dev != nullptr) M = min(M, *m_dev);
  if (row_tile * BM >= M) return;   // uniform for the workgroup, before any barrier
  constexpr int A_PER = BM * 8 / 256, B_F4 = BN * 8;  // float4 loads per stage and thread
  constexpr int B_PER = (B_F4 + 255) / 256;
  __shared__ __attribute__((aligned(16))) float As[2][BM * NT_P];
  __shared__ __attribute__((aligned(16))) float Bs[2][BN * NT_P];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane & 15, lg = lane >> 4;
  const int m0 = row_tile * BM, n0 = col_tile * BN;

  floatx4 acc[TN];
#pragma unroll
  for (int b = 0; b < TN; ++b) acc[b] = floatx4{0.f, 0.f, 0.f, 0.f};

  // Row indices are clamped instead of guarded, so the hot loop has no branches: rows >= M and weight
  // rows >= N read valid memory whose products are dropped in the epilogue.
  const float* pa[A_PER];
  const float* pb[B_PER];
#pragma unroll
  for (int u = 0; u < A_PER; ++u) {
    const int f = tid + u * 256;
    pa[u] = A + (size_t)min(m0 + (f >> 3), M - 1) * lda + (f & 7) * 4;
  }
#pragma unroll
  for (int u = 0; u < B_PER; ++u) {
    const int f = min(tid + u * 256, B_F4 - 1);
    pb[u] = B + (size_t)min(n0 + (f >> 3), N - 1) * ldb + (f & 7) * 4;
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
  auto compute = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {  // two 16-wide k slabs per stage
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
  const int nk = Kp / NT_BK;
  gload(r0, 0);
  gload(r1, nk > 1 ? NT_BK : 0);
  sstore(r0, 0);
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
  compute(0);
  if (rem >= 2) {
    sstore(r1, 1);
    __syncthreads();
    compute(1);
    if (rem == 3) {
      sstore(r0, 0);
      __syncthreads();
      compute(0);
    }
  }

#pragma unroll
  for (int b = 0; b < TN; ++b) {
    const int col = n0 + b * 16 + li;
    if (col >= n_store) continue;
    const float bv = (bias != nullptr && col < N) ? bias[col] : 0.f;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int row = m0 + wave * 16 + lg * 4 + v;
      if (row < M) {
        float x = 0.f;
        if (col < N) {
          x = acc[b][v] + bv;
          if (relu) x = fmaxf(x, 0.f);
        }
        C[(size_t)row * ldc + col] = x;
      }
    }
  }
}

template <int TN>
static void launch_nt(const float* A, int lda, const float* B, int ldb, const float* bias, float* C, int ldc, int M,
                      int N, int Kp, int n_store, bool relu, hipStream_t s, const int* m_dev) {
  constexpr int BM = 64, BN = 16 * TN;
  const int col_tiles = (n_store + BN - 1) / BN;
  const int row_tiles8 = ((M + BM - 1) / BM + 7) & ~7;
  hipLaunchKernelGGL((gemm_nt_kernel<TN>), dim3(col_tiles * row_tiles8), dim3(256), 0, s, A, lda, B, ldb, bias, C, ldc, M,
                     N, Kp, n_store, relu ? 1 : 0, m_dev, col_tiles);
}

// ------------------------------------------------------------------------------------------------
// NT with v_mfma_f32_32x32x2_f32 for problems with many rows: lane l supplies A[i = l%32][kk = l/32] and
// B[kk = l/32][j = l%32]; accumulator v of 16 holds D[i = 8*(v/4) + 4*(l/32) + v%4][j = l%32].  Half the LDS
// reads per flop of the 16x16 kernel and a higher sustained issue rate.  A workgroup is 4 waves stacked
// along M (32 rows each, BM = 128) and 32*TNB columns; a stage is 16 k-columns = two 8-wide slabs, of which
// lane half g reads k = 4g .. 4g+3 as one float4.  LDS rows are 16 floats = 4 chunks; chunk c of row r sits at
// c ^ ((r >> 2) & 3), which makes both the operand reads and the stage stores bank-conflict free.
// ------------------------------------------------------------------------------------------------
typedef float floatx16 __attribute__((ext_vector_type(16)));
constexpr int N32_BK = 16;
__device__ __forceinline__ int n32_swz(int row, int chunk) { return row * N32_BK + ((chunk ^ ((row >> 2) & 3)) << 2); }

template <int TNB>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, (TNB <= 2 ? 4 : 2)))) void gemm_nt32_kernel(
    const float* __restrict__ A, int lda, const float* __restrict__ B, int ldb, const float* __restrict__ bias,
    float* __restrict__ C, int ldc, int M, int N, int Kp, int n_store, int relu, const int* __restrict__ m_dev,
    int col_tiles) {
  constexpr int BM = 128, BN = 32 * TNB;
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int row_tile = (slot / col_tiles) * 8 + xcd, col_tile = slot % col_tiles;
  if (m_dev != nullptr) M = min(M, *m_dev);
  if (row_tile * BM >= M) return;
  constexpr int A_PER = BM * 4 / 256, B_F4 = BN * 4;
  constexpr int B_PER = (B_F4 + 255) / 256;
  __shared__ __attribute__((aligned(16))) float As[2][BM * N32_BK];
  __shared__ __attribute__((aligned(16))) float Bs[2][BN * N32_BK];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane & 31, lg = lane >> 5;
  const int m0 = row_tile * BM, n0 = col_tile * BN;

  floatx16 acc[TNB];
#pragma unroll
  for (int b = 0; b < TNB; ++b)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[b][v] = 0.f;

  const float* pa[A_PER];
  const float* pb[B_PER];
#pragma unroll
  for (int u = 0; u < A_PER; ++u) {
    const int f = tid + u * 256;
    pa[u] = A + (size_t)min(m0 + (f >> 2), M - 1) * lda + (f & 3) * 4;
  }
#pragma unroll
  for (int u = 0; u < B_PER; ++u) {
    const int f = min(tid + u * 256, B_F4 - 1);
    pb[u] = B + (size_t)min(n0 + (f >> 2), N - 1) * ldb + (f & 3) * 4;
  }
  struct Regs {
    floatx4 a[A_PER], b[B_PER];
  };
  Regs r0, r1;
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
      *reinterpret_cast<floatx4*>(&As[buf][n32_swz(f >> 2, f & 3)]) = r.a[u];
    }
#pragma unroll
    for (int u = 0; u < B_PER; ++u) {
      const int f = tid + u * 256;
      if (B_F4 % 256 == 0 || f < B_F4) *reinterpret_cast<floatx4*>(&Bs[buf][n32_swz(f >> 2, f & 3)]) = r.b[u];
    }
  };
  auto compute = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {  // two 8-wide k slabs per stage
      const floatx4 a4 = *reinterpret_cast<const floatx4*>(&As[buf][n32_swz(wave * 32 + li, h * 2 + lg)]);
      floatx4 b4[TNB];
#pragma unroll
      for (int b = 0; b < TNB; ++b)
        b4[b] = *reinterpret_cast<const floatx4*>(&Bs[buf][n32_swz(b * 32 + li, h * 2 + lg)]);
#pragma unroll
      for (int b = 0; b < TNB; ++b) acc[b] = __builtin_amdgcn_mfma_f32_32x32x2f32(a4.x, b4[b].x, acc[b], 0, 0, 0);
#pragma unroll
      for (int b = 0; b < TNB; ++b) acc[b] = __builtin_amdgcn_mfma_f32_32x32x2f32(a4.y, b4[b].y, acc[b], 0, 0, 0);
#pragma unroll
      for (int b = 0; b < TNB; ++b) acc[b] = __builtin_amdgcn_mfma_f32_32x32x2f32(a4.z, b4[b].z, acc[b], 0, 0, 0);
#pragma unroll
      for (int b = 0; b < TNB; ++b) acc[b] = __builtin_amdgcn_mfma_f32_32x32x2f32(a4.w, b4[b].w, acc[b], 0, 0, 0);
    }
  };

  const int nk = Kp / N32_BK;
  gload(r0, 0);
  gload(r1, nk > 1 ? N32_BK : 0);
  sstore(r0, 0);
  __syncthreads();
  int kt = 0;
  for (; kt + 3 < nk; kt += 2) {
    gload(r0, (kt + 2) * N32_BK);
    compute(0);
    sstore(r1, 1);
    __syncthreads();
    gload(r1, (kt + 3) * N32_BK);
    compute(1);
    sstore(r0, 0);
    __syncthreads();
  }
  const int rem = nk - kt;
  if (rem == 3) gload(r0, (kt + 2) * N32_BK);
  compute(0);
  if (rem >= 2) {
    sstore(r1, 1);
    __syncthreads();
    compute(1);
    if (rem == 3) {
      sstore(r0, 0);
      __syncthreads();
      compute(0);
    }
  }

#pragma unroll
  for (int b = 0; b < TNB; ++b) {
    const int col = n0 + b * 32 + li;
    if (col >= n_store) continue;
    const float bv = (bias != nullptr && col < N) ? bias[col] : 0.f;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int row = m0 + wave * 32 + 8 * (v >> 2) + 4 * lg + (v & 3);
      if (row < M) {
        float x = 0.f;
        if (col < N) {
          x = acc[b][v] + bv;
          if (relu) x = fmaxf(x, 0.f);
        }
        C[(size_t)row * ldc + col] = x;
      }
    }
  }
}

template <int TNB>
static void launch_nt32(const float* A, int lda, const float* B, int ldb, const float* bias, float* C, int ldc, int M,
                        int N, int Kp, int n_store, bool relu, hipStream_t s, const int* m_dev) {
  constexpr int BM = 128, BN = 32 * TNB;
  const int col_tiles = (n_store + BN - 1) / BN;
  const int row_tiles8 = ((M + BM - 1) / BM + 7) & ~7;
  hipLaunchKernelGGL((gemm_nt32_kernel<TNB>), dim3(col_tiles * row_tiles8), dim3(256), 0, s, A, lda, B, ldb, bias, C, ldc,
                     M, N, Kp, n_store, relu ? 1 : 0, m_dev, col_tiles);
}

void gemm_nt(const float* A, int lda, const float* B, int ldb, const float* bias, float* C, int ldc, int M, int N,
             int Kp, int n_store, bool relu, hipStream_t s, const int* m_dev) {
  if (M <= 0 || N <= 0) return;
  if (n_store < N) n_store = N;
  // Column-tile width in 16-wide MFMA blocks, from sweeps on MI355X: problems of a few thousand rows want the
  // narrowest tiles (many short workgroups, all resident at once), tens of thousands of rows want 2 blocks,
  // and only beyond that do wider tiles (less re-reading of A) pay off.
  const int nb = (n_store + 15) / 16;
  int best = 1;
  if (M > 4096 && M <= 65536) {
    best = 2;
  } else if (M > 65536) {
    float best_cost = 1e30f;
    static const int cand[] = {5, 4, 7, 2};
    for (int c : cand) {
      const float cost = (float)(((nb + c - 1) / c) * c) / nb;   // padded / useful columns
      if (cost < best_cost - 1e-6f) { best_cost = cost; best = c; }
    }
  }
  if (const char* e = getenv("TGNN_NT_TN")) best = atoi(e);
  if (const char* e = getenv("TGNN_NT32")) {   // experiment switch: 32x32x2 kernel with the given column blocks
    const int t = atoi(e);
    if (t == 1) { launch_nt32<1>(A, lda, B, ldb, bias, C, ldc, M, N, Kp, n_store, relu, s, m_dev); return; }
    if (t == 2) { launch_nt32<2>(A, lda, B, ldb, bias, C, ldc, M, N, Kp, n_store, relu, s, m_dev); return; }
    if (t == 4) { launch_nt32<4>(A, lda, B, ldb, bias, C, ldc, M, N, Kp, n_store, relu, s, m_dev); return; }
  }
#define TGNN_NT_CASE(TNV) \
  case TNV: launch_nt<TNV>(A, lda, B, ldb, bias, C, ldc, M, N, Kp, n_store, relu, s, m_dev); break;
  switch (best) {
    TGNN_NT_CASE(10)
    TGNN_NT_CASE(7)
    TGNN_NT_CASE(5)
    TGNN_NT_CASE(4)
    TGNN_NT_CASE(2)
    TGNN_NT_CASE(1)
  }
#undef TGNN_NT_CASE
}

// ------------------------------------------------------------------------------------------------
// TN with accumulation: G[n, k] += sum_m D[m, n] * A[m, k].  Both operands are m-major, so a stage is
// 32 rows of D (64 columns) and 32 rows of A (64 columns); 2 x 2 waves each own a 32 x 32 block of G.
// The reduction over m is split over blockIdx.y; partial results are added with float atomics.
// ------------------------------------------------------------------------------------------------
constexpr int TT = 64;     // output tile edge
constexpr int TN_P = 80;   // stage row pitch: rows 4 apart land 16 banks apart
constexpr int TN_ROWS = 32;

__global__ __launch_bounds__(256) void gemm_tn_kernel(TnGroup grp) {
  // Several independent problems share one launch (all weight gradients of a step): find this workgroup's.
  int pi = 0;
  while (pi + 1 < grp.n && (int)blockIdx.x >= grp.p[pi + 1].wg_begin) ++pi;
  const TnProblem& pr = grp.p[pi];
  const float* __restrict__ D = pr.D;
  const float* __restrict__ A = pr.A;
  const int ldd = pr.ldd, lda = pr.lda, N = pr.N, K = pr.K, k_tiles = pr.k_tiles, tiles = pr.tiles, chunks = pr.chunks;
  int M = pr.M, m_chunk = pr.m_chunk;
  const OutMap& out = pr.out;
  // All output tiles of one m-chunk read the same rows of D and A: keep them on one XCD (one L2).
  const int local = (int)blockIdx.x - pr.wg_begin;
  const int xcd = local & 7, slot = local >> 3;
  const int chunk = (slot / tiles) * 8 + xcd, tile = slot % tiles;
  if (chunk >= chunks) return;
  if (pr.m_dev != nullptr) {  // row count known only on the device: split it evenly over the launched chunks
    M = min(M, *pr.m_dev);
    m_chunk = ((M + chunks - 1) / chunks + TN_ROWS - 1) / TN_ROWS * TN_ROWS;
  }
  if (chunk * m_chunk >= M) return;
  __shared__ __attribute__((aligned(16))) float Ds[2][TN_ROWS * TN_P];
  __shared__ __attribute__((aligned(16))) float Asm[2][TN_ROWS * TN_P];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane & 15, lg = lane >> 4;
  const int wn = wave >> 1, wk = wave & 1;
  const int n0 = (tile / k_tiles) * TT, k0 = (tile % k_tiles) * TT;
  const int m_lo = chunk * m_chunk;
  const int m_hi = min(M, m_lo + m_chunk);
  const bool do_bias = (tile % k_tiles) == 0 && (out.bias[0] != nullptr);

  floatx4 acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b) acc[a][b] = floatx4{0.f, 0.f, 0.f, 0.f};
  float bsum = 0.f;

  // This thread's float4s of a stage: rows lrow and lrow + 16.  Column offsets are clamped into the row
  // (results of clamped columns are dropped at the end); rows >= m_hi are clamped and zeroed by a select.
  const int lrow = tid >> 4, lc4 = (tid & 15) * 4;
  const float* pd = D + min(n0 + lc4, ldd - 4);
  const float* pa = A + min(k0 + lc4, lda - 4);
  struct Regs {
    floatx4 d[2], a[2];
  };
  Regs r0, r1;
  auto gload = [&](Regs& r, int m) __attribute__((always_inline)) {
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int row = m + lrow + u * 16;
      const size_t rr = (size_t)min(row, M - 1);
      const floatx4 vd = *reinterpret_cast<const floatx4*>(pd + rr * ldd);
      const floatx4 va = *reinterpret_cast<const floatx4*>(pa + rr * lda);
      const bool ok = row < m_hi;
      r.d[u] = ok ? vd : floatx4{0.f, 0.f, 0.f, 0.f};
      r.a[u] = va;   // multiplied by the zeros of r.d when the row is out of range
    }
  };
  auto sstore = [&](const Regs& r, int buf) __attribute__((always_inline)) {
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      *reinterpret_cast<floatx4*>(&Ds[buf][(lrow + u * 16) * TN_P + lc4]) = r.d[u];
      *reinterpret_cast<floatx4*>(&Asm[buf][(lrow + u * 16) * TN_P + lc4]) = r.a[u];
    }
  };
  auto compute = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
    for (int q = 0; q < TN_ROWS / 4; ++q) {
      const int mm = q * 4 + lg;
      const float a0 = Ds[buf][mm * TN_P + wn * 32 + li];
      const float a1 = Ds[buf][mm * TN_P + wn * 32 + 16 + li];
      const float b0 = Asm[buf][mm * TN_P + wk * 32 + li];
      const float b1 = Asm[buf][mm * TN_P + wk * 32 + 16 + li];
      acc[0][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(a0, b0, acc[0][0], 0, 0, 0);
      acc[0][1] = __builtin_amdgcn_mfma_f32_16x16x4f32(a0, b1, acc[0][1], 0, 0, 0);
      acc[1][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(a1, b0, acc[1][0], 0, 0, 0);
      acc[1][1] = __builtin_amdgcn_mfma_f32_16x16x4f32(a1, b1, acc[1][1], 0, 0, 0);
    }
    if (do_bias && tid < TT) {
#pragma unroll
      for (int mm = 0; mm < TN_ROWS; ++mm) bsum += Ds[buf][mm * TN_P + tid];
    }
  };

  const int nst = (m_hi - m_lo + TN_ROWS - 1) / TN_ROWS;   // >= 1 by construction of the grid
  gload(r0, m_lo);
  gload(r1, m_lo + TN_ROWS);
  sstore(r0, 0);
  __syncthreads();
  int st = 0;
  for (; st + 3 < nst; st += 2) {
    gload(r0, m_lo + (st + 2) * TN_ROWS);
    compute(0);
    sstore(r1, 1);
    __syncthreads();
    gload(r1, m_lo + (st + 3) * TN_ROWS);
    compute(1);
    sstore(r0, 0);
    __syncthreads();
  }
  const int rem = nst - st;
  if (rem == 3) gload(r0, m_lo + (st + 2) * TN_ROWS);
  compute(0);
  if (rem >= 2) {
    sstore(r1, 1);
    __syncthreads();
    compute(1);
    if (rem == 3) {
      sstore(r0, 0);
      __syncthreads();
      compute(0);
    }
  }

#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      const int k = k0 + wk * 32 + b * 16 + li;
      if (k >= K) continue;
      const int ks = k >= out.k_split ? 1 : 0;
      const int kk = k - (ks ? out.k_split : 0);
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int n = n0 + wn * 32 + a * 16 + lg * 4 + v;
        if (n >= N) continue;
        const int ns = n >= out.n_split ? 1 : 0;
        const int nn = n - (ns ? out.n_split : 0);
        atomicAdd(out.p[ns][ks] + (size_t)nn * out.ld[ns][ks] + kk, acc[a][b][v]);
      }
    }
  if (do_bias && tid < TT) {
    const int n = n0 + tid;
    if (n < N) {
      const int ns = n >= out.n_split ? 1 : 0;
      atomicAdd(out.bias[ns] + (n - (ns ? out.n_split : 0)), bsum);
    }
  }
}

void TnBatch::add(const float* D, int ldd, const float* A, int lda, int M, int N, int K, const OutMap& out,
                  const int* m_dev) {
  if (M <= 0 || N <= 0 || K <= 0 || g.n >= TN_MAX_GROUP) return;
  TnProblem& p = g.p[g.n];
  const int n_tiles = (N + TT - 1) / TT, k_tiles = (K + TT - 1) / TT;
  const int tiles = n_tiles * k_tiles;
  // enough m-chunks to give the chip a few workgroups per CU, at least 64 rows (two stages) each
  int chunks = (1024 + tiles - 1) / tiles;
  const int max_chunks = (M + 63) / 64;
  if (chunks > max_chunks) chunks = max_chunks;
  if (chunks < 1) chunks = 1;
  int m_chunk = ((M + chunks - 1) / chunks + TN_ROWS - 1) / TN_ROWS * TN_ROWS;
  chunks = (M + m_chunk - 1) / m_chunk;
  if (m_dev != nullptr && chunks > 16) chunks = 16;   // the device-side row count is usually far below M
  p.D = D; p.ldd = ldd; p.A = A; p.lda = lda; p.M = M; p.N = N; p.K = K;
  p.m_chunk = m_chunk; p.k_tiles = k_tiles; p.tiles = tiles; p.chunks = chunks;
  p.wg_begin = total_wgs; p.m_dev = m_dev; p.out = out;
  total_wgs += tiles * ((chunks + 7) & ~7);
  g.n++;
}

void TnBatch::launch(hipStream_t s) {
  if (g.n == 0) return;
  hipLaunchKernelGGL(gemm_tn_kernel, dim3(total_wgs), dim3(256), 0, s, g);
  g.n = 0;
  total_wgs = 0;
}

void gemm_tn_acc(const float* D, int ldd, const float* A, int lda, int M, int N, int K, const OutMap& out,
                 hipStream_t s, const int* m_dev) {
  TnBatch b;
  b.add(D, ldd, A, lda, M, N, K, out, m_dev);
  b.launch(s);
}

}  // namespace tgnn
