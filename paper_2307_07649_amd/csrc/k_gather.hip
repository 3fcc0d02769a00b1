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
    const int map_blocks = (a.map.S + (int)blockDim.x - 1) / (int)blockDim.x;
    if (block < map_blocks) {
      uniq_map_block(a.map, block);
      return;
    }
    block -= map_blocks; n_blocks -= map_blocks;
  }
  const int lane = threadIdx.x & 63;
  const int wpb = blockDim.x >> 6;
  const int n_slots = a.n_dev ? min(a.n_slots, *a.n_dev) : a.n_slots;
  for (int s = block * wpb + (threadIdx.x >> 6); s < n_slots; s += n_blocks * wpb) {
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
  const int rows_launched = a.n_dev != nullptr ? std::min(a.n_slots, std::max(512, (a.n_slots + 3) / 4)) : a.n_slots;
  const int blocks = (rows_launched + 3) / 4 + (a.map.ucnt != nullptr ? (a.map.S + 255) / 256 : 0);
  if (vec == 4) hipLaunchKernelGGL(gather_kernel<4>, dim3(blocks), dim3(256), 0, s, a);
  else if (vec == 2) hipLaunchKernelGGL(gather_kernel<2>, dim3(blocks), dim3(256), 0, s, a);
  else hipLaunchKernelGGL(gather_kernel<1>, dim3(blocks), dim3(256), 0, s, a);
}

// Per neighbour slot (r, j): the slot's own part of the key/value input of Eq. 5-6, {e_vw | Phi(dt)}.  The
// node part {s'_w | static_w} is projected once per distinct node elsewhere, so it is not copied here.
// A block takes CE_ROWS consecutive slot rows.  Their indices and time differences are fetched first by a
// few lanes and shared through LDS, so that the row loads of a wave (CE_ROWS / 4 rows, all issued before
// any is consumed) do not each wait behind their own chain of dependent index loads.  Each output row is put
// together in LDS and leaves as one contiguous run of 16-byte stores.
constexpr int CE_ROWS = 16;
template <int VEC>
__global__ __launch_bounds__(256) void assemble_ce_kernel(CeArgs a) {
  extern __shared__ __attribute__((aligned(16))) float ce_lds[];   // [CE_ROWS][ldce] staging rows
  __shared__ int s_eid[CE_ROWS];       // edge-feature row, -1: absent neighbour
  __shared__ double s_delta[CE_ROWS];
  int block = blockIdx.x;
  {
    const int gru_blocks = gru_total_blocks(a.gru);   // the first blocks are passengers: the GRU gates
    if (block < gru_blocks) {
      gru_fwd_block(a.gru, block);
      return;
    }
    block -= gru_blocks;
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int RK = a.R * a.k;
  const int row0 = block * CE_ROWS;
  if (threadIdx.x < CE_ROWS) {
    const int row = row0 + threadIdx.x;
    int e = -1;
    double delta = 0.0;
    if (row < RK) {
      const int r = row / a.k, j = row - r * a.k;
      if (j < a.cnt[r]) {
        e = a.neid ? a.neid[row] : row;
        if (a.dt_in) delta = a.dt_in[row];
        else if (a.dt_source != 0) delta = a.root_t[r] - a.nts[row];
        else delta = a.root_t[r] - a.tau_nbr[a.slot_row ? a.slot_row[a.R + row] : row];
      }
      a.dtk[row] = delta;
    }
    s_eid[threadIdx.x] = e;
    s_delta[threadIdx.x] = delta;
  }
  __syncthreads();
  constexpr int PER = CE_ROWS / 4;   // rows per wave: local rows wave * PER + i
  float* stage = ce_lds + (size_t)wave * PER * a.ldce;
  // edge features: the loads of all PER rows of a pass are in flight together
  constexpr int EW = VEC == 4 ? 4 : 1;   // floats per lane and load (d_e % EW == 0)
  const int e_units = a.de / EW;
  for (int u0 = 0; u0 < e_units; u0 += 64) {
    const int u = u0 + lane;
    float4 v4[PER];
    float v1[PER];
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int e = s_eid[wave * PER + i];
      v4[i] = make_float4(0.f, 0.f, 0.f, 0.f);
      v1[i] = 0.f;
      if (e >= 0 && u < e_units) {
        if (VEC == 4) v4[i] = reinterpret_cast<const float4*>(a.efeat + (size_t)e * a.de)[u];
        else v1[i] = a.efeat[(size_t)e * a.de + u];
      }
    }
    if (u < e_units) {
#pragma unroll
      for (int i = 0; i < PER; ++i) {
        if (VEC == 4) reinterpret_cast<float4*>(stage + (size_t)i * a.ldce)[u] = v4[i];
        else stage[(size_t)i * a.ldce + u] = v1[i];
      }
    }
  }
  // time encoding and row padding
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    const bool present = s_eid[wave * PER + i] >= 0;
    const double delta = s_delta[wave * PER + i];
    float* srow = stage + (size_t)i * a.ldce;
    for (int c = lane; c < a.dt; c += 64) srow[a.de + c] = present ? time_enc(delta, a.time_w[c], a.time_b[c]) : 0.f;
    for (int c = a.de + a.dt + lane; c < a.ldce; c += 64) srow[c] = 0.f;
  }
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0): this wave's LDS writes are visible to all its lanes
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    const int row = row0 + wave * PER + i;
    if (row >= RK) break;
    float4* out = reinterpret_cast<float4*>(a.CE + (size_t)row * a.ldce);
    const float4* srow = reinterpret_cast<const float4*>(stage + (size_t)i * a.ldce);
    for (int q = lane; q < a.ldce / 4; q += 64) out[q] = srow[q];
  }
}

// Fallback for rows too wide to stage CE_ROWS of them in LDS: one wavefront per row, direct stores.
template <int VEC>
__global__ __launch_bounds__(256) void assemble_ce_wide_kernel(CeArgs a) {
  int block = blockIdx.x, n_blocks = gridDim.x;
  {
    const int gru_blocks = gru_total_blocks(a.gru);   // the first blocks are passengers: the GRU gates
    if (block < gru_blocks) {
      gru_fwd_block(a.gru, block);
      return;
    }
    block -= gru_blocks; n_blocks -= gru_blocks;
  }
  const int lane = threadIdx.x & 63;
  const int wpb = blockDim.x >> 6;
  const int RK = a.R * a.k;
  for (int row = block * wpb + (threadIdx.x >> 6); row < RK; row += n_blocks * wpb) {
    const int r = row / a.k, j = row - r * a.k;
    float* out = a.CE + (size_t)row * a.ldce;
    if (j >= a.cnt[r]) {
      wave_zero(out, a.ldce, lane);
      if (lane == 0) a.dtk[row] = 0.0;
      continue;
    }
    if (a.de) wave_copy<VEC>(out, a.efeat + (size_t)(a.neid ? a.neid[row] : row) * a.de, a.de, 0, lane);
    double delta;
    if (a.dt_in) delta = a.dt_in[row];
    else if (a.dt_source != 0) delta = a.root_t[r] - a.nts[row];
    else delta = a.root_t[r] - a.tau_nbr[a.slot_row ? a.slot_row[a.R + row] : row];
    for (int c = lane; c < a.dt; c += 64) out[a.de + c] = time_enc(delta, a.time_w[c], a.time_b[c]);
    for (int c = a.de + a.dt + lane; c < a.ldce; c += 64) out[c] = 0.f;
    if (lane == 0) a.dtk[row] = delta;
  }
}

void assemble_ce(const CeArgs& a, hipStream_t s) {
  const int rows = a.R * a.k;
  if (rows <= 0) {
    gru_gates_fwd(a.gru, s);
    return;
  }
  const int vec = pick_vec({a.de ? a.de : 4, (long long)((uintptr_t)a.efeat / 4)});
  const size_t lds = (size_t)CE_ROWS * a.ldce * sizeof(float);
  if (lds <= 48 * 1024) {
    const int blocks = (rows + CE_ROWS - 1) / CE_ROWS + gru_total_blocks(a.gru);
    if (vec == 4) hipLaunchKernelGGL(assemble_ce_kernel<4>, dim3(blocks), dim3(256), lds, s, a);
    else hipLaunchKernelGGL(assemble_ce_kernel<1>, dim3(blocks), dim3(256), lds, s, a);
  } else {
    const int blocks = (rows + 3) / 4 + gru_total_blocks(a.gru);
    if (vec == 4) hipLaunchKernelGGL(assemble_ce_wide_kernel<4>, dim3(blocks), dim3(256), 0, s, a);
    else hipLaunchKernelGGL(assemble_ce_wide_kernel<1>, dim3(blocks), dim3(256), 0, s, a);
  }
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
