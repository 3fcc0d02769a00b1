// Row gathers (Sec. 3.2.1: fetch node memory and cached mails of root and supporting nodes) fused with
// the time encoding of the mail (Eq. 1-2), and the assembly of the per-slot attention inputs (Eq. 5-6).
// One wavefront moves one row: 16-byte (or 8-byte) vector loads, every row a contiguous burst.
#include <algorithm>

#include "tgnn_internal.h"
#include "unique_device.h"
#include "gru_device.h"
#include "device_math.h"

namespace tgnn {

template <int VEC>
__global__ __launch_bounds__(256) void gather_kernel(GatherArgs a) {
  if (a.epoch_bump != nullptr && blockIdx.x == 0 && threadIdx.x == 0) *a.epoch_bump += 1ull;   // nothing here reads it
  int block = blockIdx.x, n_blocks = gridDim.x;
  if (a.map.ucnt != nullptr) {   // the first blocks are passengers: the slot -> row map
    const int map_blocks = uniq_blocks(a.map.S);
    if (block < map_blocks) {
      uniq_map_block(a.map, block);
      return;
    }
    block -= map_blocks; n_blocks -= map_blocks;
  }
  const int lane = threadIdx.x & 63;
  const int wpb = blockDim.x >> 6;
  const int n_slots = a.n_dev ? min(a.n_slots, *a.n_dev) : a.n_slots;
  typedef float vecf __attribute__((ext_vector_type(VEC)));
  // rows that fit a few vector registers per lane are moved in three round trips: the row's ids, then memory, mail
  // and their times together, then the mail's edge-feature row; all stores come last (a store issued between two
  // loads would make the later load wait for it)
  constexpr int RM = 2, RL = 4, RE = 4;   // vectors per lane: memory, mail, edge-feature row
  const bool fits = a.dm <= RM * 64 * VEC && 2 * a.dm <= RL * 64 * VEC && a.de <= RE * 64 * VEC && a.o_phi != nullptr &&
                    a.o_ef != nullptr && a.mail_eid != nullptr;
  for (int s = block * wpb + (threadIdx.x >> 6); s < n_slots; s += n_blocks * wpb) {
    int gid = a.slot_gid ? a.slot_gid[s] : s;
    if (gid >= 0) gid += a.gid_add;
    float* o_mem = a.o_mem + (size_t)s * a.p_mem;
    float* o_mail = a.o_mail + (size_t)s * a.p_mail;
    float* o_ef = a.o_ef ? a.o_ef + (size_t)s * a.p_ef : nullptr;
    float* o_phi = a.o_phi ? a.o_phi + (size_t)s * a.p_phi : nullptr;
    if (fits && gid >= 0) {
      const int nm = a.dm / VEC, nl = 2 * a.dm / VEC, ne = a.de / VEC;
      const int me = a.mail_eid[gid];
      const double mem_ts = a.mem_ts[gid], mail_ts = a.mail_ts[gid];
      vecf rm[RM], rl[RL], re[RE];
      const vecf* pm = reinterpret_cast<const vecf*>(a.mem + (size_t)gid * a.dm);
      const vecf* pl = reinterpret_cast<const vecf*>(a.mail + (size_t)gid * 2 * a.dm);
#pragma unroll
      for (int u = 0; u < RM; ++u) rm[u] = pm[min(lane + 64 * u, nm - 1)];
#pragma unroll
      for (int u = 0; u < RL; ++u) rl[u] = pl[min(lane + 64 * u, nl - 1)];
      const bool has = me >= 0;
      if (has && ne > 0) {
        const vecf* pe = reinterpret_cast<const vecf*>(a.efeat + (size_t)me * a.de);
#pragma unroll
        for (int u = 0; u < RE; ++u) re[u] = pe[min(lane + 64 * u, ne - 1)];
      } else {
#pragma unroll
        for (int u = 0; u < RE; ++u) re[u] = vecf(0.f);
      }
      const double delta = has ? mail_ts - mem_ts : 0.0;
      float phi[2];   // the first 128 time columns (the rest, if any, are written directly below)
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int c = lane + 64 * u;
        phi[u] = c < a.dt ? time_enc(delta, a.time_w[c], a.time_b[c]) : 0.f;
      }
      // stores
#pragma unroll
      for (int u = 0; u < RM; ++u)
        if (lane + 64 * u < nm) reinterpret_cast<vecf*>(o_mem)[lane + 64 * u] = rm[u];
      for (int i = lane; i < a.z_mem; i += 64) o_mem[a.dm + i] = 0.f;
#pragma unroll
      for (int u = 0; u < RL; ++u)
        if (lane + 64 * u < nl) reinterpret_cast<vecf*>(o_mail)[lane + 64 * u] = rl[u];
      for (int i = lane; i < a.z_mail; i += 64) o_mail[2 * a.dm + i] = 0.f;
#pragma unroll
      for (int u = 0; u < RE; ++u)
        if (lane + 64 * u < ne) reinterpret_cast<vecf*>(o_ef)[lane + 64 * u] = re[u];
      for (int i = lane; i < a.z_ef; i += 64) o_ef[a.de + i] = 0.f;
#pragma unroll
      for (int u = 0; u < 2; ++u)
        if (lane + 64 * u < a.dt) o_phi[lane + 64 * u] = phi[u];
      for (int c = 128 + lane; c < a.dt; c += 64) o_phi[c] = time_enc(delta, a.time_w[c], a.time_b[c]);
      for (int c = lane; c < a.z_phi; c += 64) o_phi[a.dt + c] = 0.f;
      if (lane == 0) {
        if (a.o_has) a.o_has[s] = has ? 1 : 0;
        if (a.o_mem_ts) a.o_mem_ts[s] = mem_ts;
        if (a.o_mail_ts) a.o_mail_ts[s] = mail_ts;
        if (a.o_tau) a.o_tau[s] = has ? mail_ts : mem_ts;
        if (a.o_delta) a.o_delta[s] = delta;
      }
      continue;
    }
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
      for (int c = lane; c < a.dt; c += 64) o_phi[c] = time_enc(delta, a.time_w[c], a.time_b[c]);
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
  // a row count that lives on the device is usually a small part of its bound: launch for a quarter of it (the
  // waves stride over the rows, so more rows only mean more rounds)
  const int rows_launched = a.n_dev == nullptr ? a.n_slots
                            : a.launch_rows > 0 ? std::min(a.n_slots, a.launch_rows)
                                                : std::min(a.n_slots, std::max(512, (a.n_slots + 3) / 4));
  const int blocks = (rows_launched + 3) / 4 + (a.map.ucnt != nullptr ? uniq_blocks(a.map.S) : 0);
  if (vec == 4) hipLaunchKernelGGL(gather_kernel<4>, dim3(blocks), dim3(256), 0, s, a);
  else if (vec == 2) hipLaunchKernelGGL(gather_kernel<2>, dim3(blocks), dim3(256), 0, s, a);
  else hipLaunchKernelGGL(gather_kernel<1>, dim3(blocks), dim3(256), 0, s, a);
}

// Xrow[r] = x_root[r] (r < R); Xrow[R + r k + j] = x_nbr[r k + j] for j < cnt[r], zero otherwise; pad columns zero.
__global__ __launch_bounds__(256) void stage_x_rows_kernel(int R, int k, int dx, const float* __restrict__ x_root,
                                                           const float* __restrict__ x_nbr,
                                                           const int32_t* __restrict__ cnt, float* __restrict__ Xrow,
                                                           int ldxr) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= R + R * k) return;
  const float* src;
  if (row < R) {
    src = x_root + (size_t)row * dx;
  } else {
    const int sl = row - R, r = sl / k, j = sl - r * k;
    src = j < cnt[r] ? x_nbr + (size_t)sl * dx : nullptr;
  }
  float* out = Xrow + (size_t)row * ldxr;
  for (int c = lane; c < ldxr; c += 64) out[c] = (src != nullptr && c < dx) ? src[c] : 0.f;
}

void stage_x_rows(int R, int k, int dx, const float* x_root, const float* x_nbr, const int32_t* cnt, float* Xrow,
                  int ldxr, hipStream_t s) {
  const int rows = R + R * k;
  if (rows <= 0) return;
  hipLaunchKernelGGL(stage_x_rows_kernel, dim3((rows + 3) / 4), dim3(256), 0, s, R, k, dx, x_root, x_nbr, cnt, Xrow, ldxr);
}

}  // namespace tgnn
