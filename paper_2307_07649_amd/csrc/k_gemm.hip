// fp32 MFMA GEMMs for the dense contractions of the step: the GRU and attention projections
// (Eq. 3-6), the merge layer, the decoder, and their data / weight gradients.
//
// v_mfma_f32_16x16x4_f32: lane l supplies A[i = l%16][kk = l/16] and B[kk = l/16][j = l%16]; its four
// accumulators hold D[i = 4*(l/16) + v][j = l%16].
#include "tgnn_internal.h"

namespace tgnn {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int BK = 16;     // k-depth of one LDS stage
constexpr int LDS_P = 20;  // row pitch (floats) of an NT stage: 16 lanes * 20 floats hit 16 distinct bank quads

// ------------------------------------------------------------------------------------------------
// NT: C = A * B^T.  One workgroup = 4 waves stacked along M; a wave owns a (16*TM) x (16*TN) tile.
// ------------------------------------------------------------------------------------------------
template <int TM, int TN>
__global__ __launch_bounds__(256) void gemm_nt_kernel(const float* __restrict__ A, int lda,
                                                      const float* __restrict__ B, int ldb,
                                                      const float* __restrict__ bias, float* __restrict__ C, int ldc,
                                                      int M, int N, int Kp, int n_store, int relu) {
  constexpr int BM = 64 * TM, BN = 16 * TN;
  constexpr int A_F4 = BM * 4, B_F4 = BN * 4;  // float4 loads per stage
  constexpr int A_PER = (A_F4 + 255) / 256, B_PER = (B_F4 + 255) / 256;
  __shared__ __attribute__((aligned(16))) float As[2][BM * LDS_P];
  __shared__ __attribute__((aligned(16))) float Bs[2][BN * LDS_P];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane & 15, lg = lane >> 4;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;

  floatx4 acc[TM][TN];
#pragma unroll
  for (int a = 0; a < TM; ++a)
#pragma unroll
    for (int b = 0; b < TN; ++b) acc[a][b] = floatx4{0.f, 0.f, 0.f, 0.f};

  float4 ra[A_PER], rb[B_PER];
  auto gload = [&](int k0) {
#pragma unroll
    for (int u = 0; u < A_PER; ++u) {
      int f = tid + u * 256;
      int row = f >> 2, c4 = (f & 3) * 4;
      ra[u] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (f < A_F4 && m0 + row < M) ra[u] = *reinterpret_cast<const float4*>(A + (size_t)(m0 + row) * lda + k0 + c4);
    }
#pragma unroll
    for (int u = 0; u < B_PER; ++u) {
      int f = tid + u * 256;
      int row = f >> 2, c4 = (f & 3) * 4;
      rb[u] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (f < B_F4 && n0 + row < N) rb[u] = *reinterpret_cast<const float4*>(B + (size_t)(n0 + row) * ldb + k0 + c4);
    }
  };
  auto sstore = [&](int buf) {
#pragma unroll
    for (int u = 0; u < A_PER; ++u) {
      int f = tid + u * 256;
      if (f < A_F4) *reinterpret_cast<float4*>(&As[buf][(f >> 2) * LDS_P + (f & 3) * 4]) = ra[u];
    }
#pragma unroll
    for (int u = 0; u < B_PER; ++u) {
      int f = tid + u * 256;
      if (f < B_F4) *reinterpret_cast<float4*>(&Bs[buf][(f >> 2) * LDS_P + (f & 3) * 4]) = rb[u];
    }
  };

  const int nk = Kp / BK;
  gload(0);
  sstore(0);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < nk) gload((kt + 1) * BK);
    float4 a4[TM];
#pragma unroll
    for (int a = 0; a < TM; ++a)
      a4[a] = *reinterpret_cast<const float4*>(&As[cur][(wave * 16 * TM + a * 16 + li) * LDS_P + lg * 4]);
#pragma unroll
    for (int b = 0; b < TN; ++b) {
      float4 b4 = *reinterpret_cast<const float4*>(&Bs[cur][(b * 16 + li) * LDS_P + lg * 4]);
#pragma unroll
      for (int a = 0; a < TM; ++a) {
        acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x4f32(a4[a].x, b4.x, acc[a][b], 0, 0, 0);
        acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x4f32(a4[a].y, b4.y, acc[a][b], 0, 0, 0);
        acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x4f32(a4[a].z, b4.z, acc[a][b], 0, 0, 0);
        acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x4f32(a4[a].w, b4.w, acc[a][b], 0, 0, 0);
      }
    }
    if (kt + 1 < nk) sstore(cur ^ 1);
    __syncthreads();
  }

#pragma unroll
  for (int b = 0; b < TN; ++b) {
    const int col = n0 + b * 16 + li;
    if (col >= n_store) continue;
    const float bv = (bias != nullptr && col < N) ? bias[col] : 0.f;
#pragma unroll
    for (int a = 0; a < TM; ++a) {
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int row = m0 + wave * 16 * TM + a * 16 + lg * 4 + v;
        if (row < M) {
          float x = 0.f;
          if (col < N) {
            x = acc[a][b][v] + bv;
            if (relu) x = fmaxf(x, 0.f);
          }
          C[(size_t)row * ldc + col] = x;
        }
      }
    }
  }
}

template <int TM, int TN>
static void launch_nt(const float* A, int lda, const float* B, int ldb, const float* bias, float* C, int ldc, int M,
                      int N, int Kp, int n_store, bool relu, hipStream_t s) {
  constexpr int BM = 64 * TM, BN = 16 * TN;
  dim3 grid((n_store + BN - 1) / BN, (M + BM - 1) / BM);
  hipLaunchKernelGGL((gemm_nt_kernel<TM, TN>), grid, dim3(256), 0, s, A, lda, B, ldb, bias, C, ldc, M, N, Kp, n_store,
                     relu ? 1 : 0);
}

void gemm_nt(const float* A, int lda, const float* B, int ldb, const float* bias, float* C, int ldc, int M, int N,
             int Kp, int n_store, bool relu, hipStream_t s) {
  if (M <= 0 || N <= 0) return;
  if (n_store < N) n_store = N;
  // pick the column-tile width (in 16-wide MFMA blocks) that wastes the fewest padded columns
  static const int cand[] = {13, 10, 7, 4, 2, 1};
  const int nb = (n_store + 15) / 16;
  int best = 1, best_cost = 1 << 30;
  for (int c : cand) {
    int tiles = (nb + c - 1) / c;
    int cost = tiles * c;
    if (cost < best_cost) { best_cost = cost; best = c; }
  }
#define TGNN_NT_CASE(TNV) \
  case TNV: launch_nt<1, TNV>(A, lda, B, ldb, bias, C, ldc, M, N, Kp, n_store, relu, s); break;
  switch (best) {
    TGNN_NT_CASE(13)
    TGNN_NT_CASE(10)
    TGNN_NT_CASE(7)
    TGNN_NT_CASE(4)
    TGNN_NT_CASE(2)
    TGNN_NT_CASE(1)
  }
#undef TGNN_NT_CASE
}

// ------------------------------------------------------------------------------------------------
// TN with accumulation: G[n, k] += sum_m D[m, n] * A[m, k].  Both operands are m-major, so a stage is
// 16 rows of D (64 columns) and 16 rows of A (64 columns); 2 x 2 waves each own a 32 x 32 block of G.
// The reduction over m is split over blockIdx.y; partial results are added with float atomics.
// ------------------------------------------------------------------------------------------------
constexpr int TT = 64;     // output tile edge
constexpr int TN_P = 80;   // stage row pitch: rows 4 apart land 16 banks apart

__global__ __launch_bounds__(256) void gemm_tn_kernel(const float* __restrict__ D, int ldd,
                                                      const float* __restrict__ A, int lda, int M, int N, int K,
                                                      int m_chunk, int k_tiles, OutMap out) {
  __shared__ __attribute__((aligned(16))) float Ds[2][16 * TN_P];
  __shared__ __attribute__((aligned(16))) float Asm[2][16 * TN_P];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane & 15, lg = lane >> 4;
  const int wn = wave >> 1, wk = wave & 1;
  const int n0 = (blockIdx.x / k_tiles) * TT, k0 = (blockIdx.x % k_tiles) * TT;
  const int m_lo = blockIdx.y * m_chunk;
  const int m_hi = min(M, m_lo + m_chunk);
  const bool do_bias = (blockIdx.x % k_tiles) == 0 && (out.bias[0] != nullptr);

  floatx4 acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b) acc[a][b] = floatx4{0.f, 0.f, 0.f, 0.f};
  float bsum = 0.f;

  const int lrow = tid >> 4, lc4 = (tid & 15) * 4;  // this thread's float4 of a 16 x 64 stage
  float4 rd, ra;
  auto gload = [&](int m) {
    rd = make_float4(0.f, 0.f, 0.f, 0.f);
    ra = rd;
    if (m + lrow < m_hi) {
      if (n0 + lc4 < ldd) rd = *reinterpret_cast<const float4*>(D + (size_t)(m + lrow) * ldd + n0 + lc4);
      if (k0 + lc4 < lda) ra = *reinterpret_cast<const float4*>(A + (size_t)(m + lrow) * lda + k0 + lc4);
    }
  };
  auto sstore = [&](int buf) {
    *reinterpret_cast<float4*>(&Ds[buf][lrow * TN_P + lc4]) = rd;
    *reinterpret_cast<float4*>(&Asm[buf][lrow * TN_P + lc4]) = ra;
  };

  const int nst = (m_hi - m_lo + 15) / 16;
  if (nst > 0) {
    gload(m_lo);
    sstore(0);
  }
  __syncthreads();
  for (int st = 0; st < nst; ++st) {
    const int cur = st & 1;
    if (st + 1 < nst) gload(m_lo + (st + 1) * 16);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int mm = q * 4 + lg;
      float a0 = Ds[cur][mm * TN_P + wn * 32 + li];
      float a1 = Ds[cur][mm * TN_P + wn * 32 + 16 + li];
      float b0 = Asm[cur][mm * TN_P + wk * 32 + li];
      float b1 = Asm[cur][mm * TN_P + wk * 32 + 16 + li];
      acc[0][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(a0, b0, acc[0][0], 0, 0, 0);
      acc[0][1] = __builtin_amdgcn_mfma_f32_16x16x4f32(a0, b1, acc[0][1], 0, 0, 0);
      acc[1][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(a1, b0, acc[1][0], 0, 0, 0);
      acc[1][1] = __builtin_amdgcn_mfma_f32_16x16x4f32(a1, b1, acc[1][1], 0, 0, 0);
    }
    if (do_bias && tid < TT) {
#pragma unroll
      for (int mm = 0; mm < 16; ++mm) bsum += Ds[cur][mm * TN_P + tid];
    }
    if (st + 1 < nst) sstore(cur ^ 1);
    __syncthreads();
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

void gemm_tn_acc(const float* D, int ldd, const float* A, int lda, int M, int N, int K, const OutMap& out,
                 hipStream_t s) {
  if (M <= 0 || N <= 0 || K <= 0) return;
  const int n_tiles = (N + TT - 1) / TT, k_tiles = (K + TT - 1) / TT;
  const int tiles = n_tiles * k_tiles;
  // enough m-chunks to give the chip ~4 workgroups per CU, at least 64 rows each
  int chunks = (1024 + tiles - 1) / tiles;
  int max_chunks = (M + 63) / 64;
  if (chunks > max_chunks) chunks = max_chunks;
  if (chunks < 1) chunks = 1;
  int m_chunk = ((M + chunks - 1) / chunks + 15) & ~15;
  chunks = (M + m_chunk - 1) / m_chunk;
  hipLaunchKernelGGL(gemm_tn_kernel, dim3(tiles, chunks), dim3(256), 0, s, D, ldd, A, lda, M, N, K, m_chunk, k_tiles,
                     out);
}

}  // namespace tgnn
