// Element-wise part of UPDT = GRU cell (Eq. 3): gates forward (gru_device.h), as a launch of its own.  In the
// training step it rides in the launch that assembles the per-slot attention input instead.  The matrix products
// live in k_gemm.hip; the gates' backward pass is an epilogue of the product that yields the gradient reaching s'.
#include <algorithm>

#include "tgnn_internal.h"
#include "gru_device.h"

namespace tgnn {

__global__ __launch_bounds__(256) void gru_fwd_kernel(GruFwdArgs a) { gru_fwd_block(a, blockIdx.x); }

GruFwdArgs gru_gates_args(const Dims& d, int n, const int* n_dev, const float* gi, const float* gh, const float* Hm,
                          const int32_t* has, float* gates, float* x_out, int ld_x, const float* stat, const int32_t* gid,
                          float* zero_buf, int zero_w, const SortArgs& scan, int launch_rows) {
  GruFwdArgs a;
  if (n <= 0) return a;
  a.n_max = n; a.n_dev = n_dev; a.dm = d.dm; a.ldh = d.ldh; a.ld3 = d.ld3;
  a.gi = gi; a.gh = gh; a.Hm = Hm; a.has = has; a.gates = gates; a.x_out = x_out; a.ld_x = ld_x;
  a.stat = stat; a.ds = d.ds; a.gid = gid; a.N = d.N; a.zero_buf = zero_buf; a.zero_w = zero_w;
  // a row count that lives on the device is usually a small part of its bound: launch for an eighth of it (the
  // threads stride over the elements, so more rows only mean more rounds)
  // (launch_rows: the caller's estimate of the row count, in which case half of it is launched: two rounds)
  const int rows_launched = n_dev == nullptr ? n
                            : launch_rows > 0 ? std::min(n, std::max(512, launch_rows / 2))
                                              : std::min(n, std::max(512, (n + 7) / 8));
  a.gru_blocks = (int)(((long long)rows_launched * d.dm + 255) / 256);
  a.scan = scan;
  return a;
}

void gru_gates_fwd(const GruFwdArgs& a, hipStream_t s) {
  const int blocks = gru_total_blocks(a);
  if (blocks > 0) hipLaunchKernelGGL(gru_fwd_kernel, dim3(blocks), dim3(256), 0, s, a);
}

}  // namespace tgnn
