// The entry point for callers that cannot allocate (code under graph capture, tight serving loops, harnesses
// that forbid hipMalloc): disco_loss_fwd_bwd with its workspace in a static device array of this library.
#include "common.h"

#include <mutex>

using namespace disco;

namespace {

static __device__ __align__(256) unsigned char scratch[DISCO_STATIC_SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[MAX_DEVICES] = {};      // device address of `scratch` on each device, looked up once

// Address of this device's copy of `scratch` (every device holds its own), or nullptr on failure.
void* scratch_on_current_device() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}

}  // namespace

extern "C" size_t disco_static_scratch_bytes(void) { return DISCO_STATIC_SCRATCH_BYTES; }

extern "C" int disco_loss_fwd_bwd_static(const void* I, const void* T, int64_t B, int64_t d, int32_t rank, int32_t N,
                                         float s, int dtype, int path, int accumulate, float* loss, float* gI,
                                         float* gT, float* gs, void* hip_stream) {
  if (!I || !T || !loss || !gI || !gT || !gs) return DISCO_ERR_NULL;
  const int r = disco_resolve_path(B, d, N, dtype, path);
  if (r < 0) return -r;
  if (rank < 0 || rank >= N) return DISCO_ERR_SHAPE;
  const size_t need = disco_workspace_bytes(B, d, N, dtype, r);
  if (need == 0 || need > DISCO_STATIC_SCRATCH_BYTES) return DISCO_ERR_WORKSPACE;
  void* ws = scratch_on_current_device();
  if (!ws) return DISCO_ERR_HIP;
  return disco_loss_fwd_bwd(I, T, B, d, rank, N, s, dtype, r, accumulate, loss, gI, gT, gs, ws, DISCO_STATIC_SCRATCH_BYTES,
                            hip_stream);
}

