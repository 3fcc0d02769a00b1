// tgnn_memory_writeback_noalloc: the last-event-wins write-back for callers that cannot allocate device memory
// (code under HIP graph capture, tight serving loops).  Same kernels as tgnn_memory_writeback; the arbitration
// words, the step counter and the batch descriptor live in a file-scope device array instead of a context's
// workspace.  Every GPU the library runs on holds its own copy of the array until the process ends.
#include <string.h>

#include <mutex>

#include "tgnn_internal.h"
#include "writeback_device.h"

namespace tgnn {

struct StaticScratch {
  unsigned long long winkey[TGNN_NOALLOC_MAX_NODES];   // arbitration word per node
  unsigned long long epoch;                            // the key prefix the kernels expect (constant here)
  BatchSet bs;                                         // device copy of the call's batch descriptor
};
// In host code this name is only a handle for hipGetSymbolAddress; the device address is looked up once per device.
static __device__ __align__(256) unsigned char scratch[sizeof(StaticScratch)];

constexpr int MAX_DEVICES = 64;
static std::mutex g_mu;
static StaticScratch* g_scratch[MAX_DEVICES] = {};

// Device address of this device's copy of the array (the device must be current).
static int scratch_of_current_device(StaticScratch** out) {
  int dev = -1;
  TGNN_HIP_CHECK(hipGetDevice(&dev));
  if (dev < 0 || dev >= MAX_DEVICES) return set_error(TGNN_E_OUT_OF_RANGE, "device ordinal %d outside [0, %d)", dev, MAX_DEVICES);
  std::lock_guard<std::mutex> lock(g_mu);
  if (g_scratch[dev] == nullptr) {
    void* p = nullptr;
    TGNN_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (p == nullptr) return set_error(TGNN_E_HIP, "hipGetSymbolAddress returned a null address");
    g_scratch[dev] = static_cast<StaticScratch*>(p);
  }
  *out = g_scratch[dev];
  return TGNN_OK;
}

// The array keeps what the last call left: the words of this call's node range are cleared, the descriptor and
// the key prefix are rewritten.  (A fill kernel rather than a memset node, so that the call can be captured.)
__global__ void noalloc_setup_kernel(StaticScratch* sc, BatchSet bs, int n_nodes) {
  const int stride = gridDim.x * blockDim.x;
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n_nodes; i += stride) sc->winkey[i] = 0ull;
  if (blockIdx.x == 0) {
    const int* src = reinterpret_cast<const int*>(&bs);
    int* dst = reinterpret_cast<int*>(&sc->bs);
    for (int i = threadIdx.x; i < (int)(sizeof(BatchSet) / sizeof(int)); i += blockDim.x) dst[i] = src[i];
    if (threadIdx.x == 0) sc->epoch = 1ull;
  }
}

}  // namespace tgnn

using namespace tgnn;

extern "C" int32_t tgnn_memory_writeback_noalloc(int32_t n_nodes, int32_t d_mem, tgnn_state* st, const int32_t* src,
                                                 const int32_t* dst, const int32_t* eid, const double* t,
                                                 int32_t n_events, const float* s_new_src, const float* s_new_dst,
                                                 const double* tau_src, const double* tau_dst, int32_t* out_winner,
                                                 void* stream) {
  if (n_nodes <= 0 || n_nodes > TGNN_NOALLOC_MAX_NODES)
    return set_error(TGNN_E_OUT_OF_RANGE, "n_nodes = %d outside [1, %d] (size of the static scratch array)", n_nodes,
                     TGNN_NOALLOC_MAX_NODES);
  if (d_mem <= 0 || d_mem > 256) return set_error(TGNN_E_UNSUPPORTED_DIM, "d_mem = %d outside [1, 256]", d_mem);
  if (n_events < 0 || n_events > TGNN_NOALLOC_MAX_EVENTS)
    return set_error(TGNN_E_OUT_OF_RANGE, "n_events = %d outside [0, %d]", n_events, TGNN_NOALLOC_MAX_EVENTS);
  if (st == nullptr) return set_error(TGNN_E_NULL_PTR, "state is NULL");
  const void* req[] = {st->mem, st->mem_ts, st->mail, st->mail_ts, st->mail_eid, src, dst, eid, t, s_new_src, s_new_dst,
                       tau_src, tau_dst};
  static const char* names[] = {"state.mem", "state.mem_ts", "state.mail", "state.mail_ts", "state.mail_eid", "src", "dst",
                                "eid", "t", "s_new_src", "s_new_dst", "tau_src", "tau_dst"};
  for (int i = 0; i < 13; ++i) {
    if (req[i] == nullptr) return set_error(TGNN_E_NULL_PTR, "%s is NULL", names[i]);
    if ((reinterpret_cast<uintptr_t>(req[i]) & 15u) != 0) return set_error(TGNN_E_MISALIGNED, "%s is not 16-byte aligned", names[i]);
  }
  if (out_winner != nullptr && (reinterpret_cast<uintptr_t>(out_winner) & 15u) != 0)
    return set_error(TGNN_E_MISALIGNED, "out_winner is not 16-byte aligned");
  if (n_events == 0) return TGNN_OK;
  StaticScratch* sc = nullptr;
  if (int rc = scratch_of_current_device(&sc)) return rc;
  BatchSet bs;
  memset(&bs, 0, sizeof(bs));
  bs.b[0] = BatchDesc{src, dst, nullptr, eid, t, n_events, 0, 0};
  bs.nb = 1; bs.total = n_events;
  Dims d;
  memset(&d, 0, sizeof(d));
  d.N = n_nodes; d.dm = d_mem;
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  const int blocks = (n_nodes + 255) / 256 < 1024 ? (n_nodes + 255) / 256 : 1024;
  hipLaunchKernelGGL(noalloc_setup_kernel, dim3(blocks), dim3(256), 0, s, sc, bs, n_nodes);
  writeback_mark(d, &sc->bs, n_events, sc->winkey, &sc->epoch, s);
  writeback_scatter(d, &sc->bs, n_events, st, sc->winkey, &sc->epoch, nullptr, d_mem, nullptr, nullptr, s_new_src, s_new_dst,
                    tau_src, tau_dst, out_winner, s);
  TGNN_LAUNCH_CHECK();
  return TGNN_OK;
}
