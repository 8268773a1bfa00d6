// monarch_attn_fwd_noalloc: the forward call on the library's own scratch memory, for callers
// that cannot allocate.  The scratch array lives in this file's device image (one copy per GPU);
// host code only ever uses the address hipGetSymbolAddress returns for the current device.
#include <mutex>

#include "mrt_internal.hpp"

namespace {

constexpr size_t kScratchBytes = size_t(128) << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

// Address of this device's copy of the array, looked up once per device with that device current.
hipError_t scratch_address(void** out) {
  static std::mutex mu;
  static void* ptr[64] = {nullptr};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lk(mu);
  if (!ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    ptr[dev] = p;
  }
  *out = ptr[dev];
  return hipSuccess;
}

}  // namespace

extern "C" mrt_status monarch_attn_fwd_noalloc(const void* Q, const void* K, const void* V, void* O,
                                               const mrt_problem* p, int b1, int b2, int tile, int iters,
                                               int causal_chunk, void* hip_stream) {
  // argument checks first (no GPU call for an invalid request)
  mrt_status st = monarch_attn_check(p, b1, b2, tile, iters, causal_chunk);
  if (st != MRT_OK) return st;
  const size_t need = monarch_attn_workspace_min_bytes(p, b1, b2, tile, iters);
  if (need == 0 || need > kScratchBytes) {
    mrt::set_error("monarch_attn_fwd_noalloc: one query tile row of one (batch, head) needs %zu bytes of "
                   "intermediates, the built-in scratch holds %zu; use monarch_attn_fwd with a workspace",
                   need, kScratchBytes);
    return MRT_ERR_WORKSPACE;
  }
  if (!Q || !K || !V || !O) { mrt::set_error("Q, K, V and O must be non-NULL"); return MRT_ERR_NULL; }
  void* ws = nullptr;
  const hipError_t e = scratch_address(&ws);
  if (e != hipSuccess) {
    mrt::set_error("address of the built-in scratch: %s", hipGetErrorString(e));
    return MRT_ERR_HIP;
  }
  return mrt::fwd_run(Q, K, V, O, p, b1, b2, tile, iters, causal_chunk, ws, kScratchBytes, hip_stream, true);
}
