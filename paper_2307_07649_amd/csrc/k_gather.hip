// Row gathers (Sec. 3.2.1: fetch node memory and cached mails of root and supporting nodes) fused with
// the time encoding of the mail (Eq. 1-2), and the assembly of the attention inputs (Eq. 4-6).
// One wavefront moves one row: 16-byte (or 8-byte) vector loads, every row a contiguous burst.
#include "tgnn_internal.h"
#include "device_math.h"

namespace tgnn {

template <int VEC>
__global__ __launch_bounds__(256) void gather_kernel(GatherArgs a) {
  const int lane = threadIdx.x & 63;
  const int wpb = blockDim.x >> 6;
  const int n_slots = a.n_dev ? min(a.n_slots, *a.n_dev) : a.n_slots;
  for (int s = blockIdx.x * wpb + (threadIdx.x >> 6); s < n_slots; s += gridDim.x * wpb) {
    int gid = a.slot_gid ? a.slot_gid[s] : s;
    if (gid >= 0) gid += a.gid_add;
    float* o_mem = a.o_mem + (size_t)s * a.p_mem;
    float* o_mail = a.o_mail + (size_t)s * a.p_mail;
    float* o_ef = a.o_ef ? a.o_ef + (size_t)s * a.p_ef : nullptr;
    float* o_phi = a.o_phi ? a.o_phi + (size_t)s * a.p_phi : nullptr;
    int me = -1;
    double mem_ts = 0.0, mail_ts = 0.0;
    if (gid >= 0) {
      me = a.mail_eid ? a.mail_eid[gid] : (a.has_in[gid] ? gid : -1);
      mem_ts = a.mem_ts[gid];
      mail_ts = a.mail_ts[gid];
      wave_copy<VEC>(o_mem, a.mem + (size_t)gid * a.dm, a.dm, a.z_mem, lane);
      wave_copy<VEC>(o_mail, a.mail + (size_t)gid * 2 * a.dm, 2 * a.dm, a.z_mail, lane);
    } else {
      wave_zero(o_mem, a.dm + a.z_mem, lane);
      wave_zero(o_mail, 2 * a.dm + a.z_mail, lane);
    }
    const bool has = me >= 0;
    if (o_ef) {
      if (has) wave_copy<VEC>(o_ef, a.efeat + (size_t)me * a.de, a.de, a.z_ef, lane);
      else wave_zero(o_ef, a.de + a.z_ef, lane);
    }
    const double delta = has ? mail_ts - mem_ts : 0.0;
    if (o_phi) {
      float* o_ms = a.o_msin ? a.o_msin + (size_t)s * a.p_msin : nullptr;
      for (int c = lane; c < a.dt; c += 64) {
        float sn, cs;
        sincos_reduced(fma((double)a.time_w[c], delta, (double)a.time_b[c]), sn, cs);
        o_phi[c] = cs;
        if (o_ms) o_ms[c] = -sn;
      }
      for (int c = lane; c < a.z_phi; c += 64) o_phi[a.dt + c] = 0.f;
    }
    if (lane == 0) {
      if (a.o_has) a.o_has[s] = has ? 1 : 0;
      if (a.o_mem_ts) a.o_mem_ts[s] = mem_ts;
      if (a.o_mail_ts) a.o_mail_ts[s] = mail_ts;
      if (a.o_tau) a.o_tau[s] = has ? mail_ts : mem_ts;
      if (a.o_delta) a.o_delta[s] = delta;
    }
  }
}

static int pick_vec(std::initializer_list<long long> vals) {
  int v = 4;
  for (long long x : vals) {
    while (v > 1 && (x % v) != 0) v >>= 1;
  }
  return v;
}

void gather_rows(const GatherArgs& a, hipStream_t s) {
  if (a.n_slots <= 0) return;
  const int vec = pick_vec({a.dm, a.de, a.p_mem, a.p_mail, a.p_ef, (long long)((uintptr_t)a.o_mem / 4),
                            (long long)((uintptr_t)a.o_mail / 4), (long long)((uintptr_t)a.o_ef / 4),
                            (long long)((uintptr_t)a.mem / 4), (long long)((uintptr_t)a.mail / 4),
                            (long long)((uintptr_t)a.efeat / 4)});
  const int blocks = (a.n_slots + 3) / 4;
  if (vec == 4) hipLaunchKernelGGL(gather_kernel<4>, dim3(blocks), dim3(256), 0, s, a);
  else if (vec == 2) hipLaunchKernelGGL(gather_kernel<2>, dim3(blocks), dim3(256), 0, s, a);
  else hipLaunchKernelGGL(gather_kernel<1>, dim3(blocks), dim3(256), 0, s, a);
}

// Rows 0 .. R*k-1: key/value input {s'_w | static_w | e_vw | Phi(dt)} of neighbour slot (r, j);
// rows R*k .. R*k+R-1: query input {s'_v | static_v | Phi(0)} and the x_v half of the merge input.
template <int VEC>
__global__ __launch_bounds__(256) void attn_assemble_kernel(AttnAssembleArgs a) {
  const int lane = threadIdx.x & 63;
  const int wpb = blockDim.x >> 6;
  const int RK = a.R * a.k;
  const int dx = a.dm + a.ds, dkv = dx + a.de + a.dt;
  for (int row = blockIdx.x * wpb + (threadIdx.x >> 6); row < RK + a.R; row += gridDim.x * wpb) {
    if (row < RK) {
      const int r = row / a.k, j = row - r * a.k;
      float* out = a.Cmat + (size_t)row * a.ldc;
      if (j >= a.cnt[r]) {
        wave_zero(out, a.ldc, lane);
        if (lane == 0) a.dtk[row] = 0.0;
        continue;
      }
      const int srow = a.slot_row ? a.slot_row[a.R + row] : row;
      wave_copy<VEC>(out, a.s_nbr + (size_t)srow * a.p_s, a.dm, 0, lane);
      if (a.ds) wave_copy<VEC>(out + a.dm, a.stat + (size_t)a.nbr[row] * a.ds, a.ds, 0, lane);
      if (a.de) wave_copy<VEC>(out + dx, a.efeat + (size_t)(a.neid ? a.neid[row] : row) * a.de, a.de, 0, lane);
      const double delta = a.dt_in ? a.dt_in[row]
                                   : a.root_t[r] - (a.dt_source == 0 ? a.tau_nbr[srow] : a.nts[row]);
      float* phi = out + dx + a.de;
      float* ms = a.msin + (size_t)row * a.p_msin;
      for (int c = lane; c < a.dt; c += 64) {
        float sn, cs;
        sincos_reduced(fma((double)a.time_w[c], delta, (double)a.time_b[c]), sn, cs);
        phi[c] = cs;
        ms[c] = -sn;
      }
      for (int c = dkv + lane; c < a.ldc; c += 64) out[c] = 0.f;
      if (lane == 0) a.dtk[row] = delta;
    } else {
      const int r = row - RK;
      const int v = a.ds ? a.root_node[r] : 0;
      float* qi = a.Qin + (size_t)r * a.ldq;
      float* mi = a.Min + (size_t)r * a.ldm + a.dO;
      const float* sv = a.s_root + (size_t)(a.slot_row ? a.slot_row[r] : r) * a.p_s;
      wave_copy<VEC>(qi, sv, a.dm, 0, lane);
      wave_copy<VEC>(mi, sv, a.dm, 0, lane);
      if (a.ds) {
        wave_copy<VEC>(qi + a.dm, a.stat + (size_t)v * a.ds, a.ds, 0, lane);
        wave_copy<VEC>(mi + a.dm, a.stat + (size_t)v * a.ds, a.ds, 0, lane);
      }
      for (int c = lane; c < a.dt; c += 64) qi[dx + c] = time_enc(0.0, a.time_w[c], a.time_b[c]);
      for (int c = dx + a.dt + lane; c < a.ldq; c += 64) qi[c] = 0.f;
      for (int c = a.dO + dx + lane; c < a.ldm; c += 64) a.Min[(size_t)r * a.ldm + c] = 0.f;
    }
  }
}

void attn_assemble(const AttnAssembleArgs& a, hipStream_t s) {
  const int rows = a.R * a.k + a.R;
  if (rows <= 0) return;
  const int vec = pick_vec({a.dm, a.ds ? a.ds : 4, a.de ? a.de : 4, a.dm + a.ds + a.de, a.dO, a.p_s,
                            (long long)((uintptr_t)a.stat / 4), (long long)((uintptr_t)a.efeat / 4),
                            (long long)((uintptr_t)a.s_root / 4), (long long)((uintptr_t)a.s_nbr / 4)});
  const int blocks = (rows + 3) / 4;
  if (vec == 4) hipLaunchKernelGGL(attn_assemble_kernel<4>, dim3(blocks), dim3(256), 0, s, a);
  else if (vec == 2) hipLaunchKernelGGL(attn_assemble_kernel<2>, dim3(blocks), dim3(256), 0, s, a);
  else hipLaunchKernelGGL(attn_assemble_kernel<1>, dim3(blocks), dim3(256), 0, s, a);
}

}  // namespace tgnn
