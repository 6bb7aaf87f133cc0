// Host side of libdisco: argument validation, path selection, workspace checks, dispatch.
// No allocation, no synchronisation, no HIP call before validation has passed.
#include "common.h"

#include <atomic>

using namespace disco;

namespace {
std::atomic<void**> g_stage_events{nullptr};
std::atomic<int> g_stage_count{0};
}  // namespace

namespace disco {
void stage_mark(hipStream_t st, int k) {
  void** ev = g_stage_events.load(std::memory_order_acquire);
  if (ev && k < g_stage_count.load(std::memory_order_acquire) && ev[k]) (void)hipEventRecord(static_cast<hipEvent_t>(ev[k]), st);
}
}  // namespace disco

extern "C" int disco_set_stage_events(void** events, int count) {
  if (count < 0) return DISCO_ERR_SHAPE;
  g_stage_count.store(events ? count : 0, std::memory_order_release);
  g_stage_events.store(events, std::memory_order_release);
  return DISCO_OK;
}

namespace {

int check_shape(int64_t B, int64_t d, int32_t N) {
  if (B <= 0 || d <= 0 || N <= 0) return DISCO_ERR_SHAPE;
  if (B % N != 0) return DISCO_ERR_SHAPE;
  // tile indices and row offsets are kept in 32-bit registers inside the kernels
  if (B > (int64_t)1 << 24 || d > (int64_t)1 << 16) return DISCO_ERR_SHAPE;
  // the fp32 path walks the rank's rows in 64-row tiles along a grid dimension limited to 65535 workgroups
  if (B / N > (int64_t)65535 * 64) return DISCO_ERR_SHAPE;
  return DISCO_OK;
}

// smallest b x B block for which DISCO_PATH_AUTO sends a ragged bf16 share to the tile kernels
constexpr int64_t RAGGED_MIN_BLOCK = (int64_t)256 * 1024;

// 16-byte alignment of the feature matrices: the bf16 tile kernels fetch them in 16-byte pieces
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int resolve(int64_t B, int64_t d, int32_t N, int dtype, int path, int variant = LOSS_CLIP) {
  int st = check_shape(B, d, N);
  if (st != DISCO_OK) return -st;
  if (variant == LOSS_NTXENT && B % 2 != 0) return -DISCO_ERR_SHAPE;       // two views of B/2 samples
  if (dtype != DISCO_F32 && dtype != DISCO_BF16) return -DISCO_ERR_UNSUPPORTED;
  const bool tiles = mfma_supported(B, d, N, dtype, variant);          // the bf16 tile kernels can take it
  const bool whole = tiles && mfma_whole_tiles(B, N);                  // without padding the share to 256-row tiles
  switch (path) {
    case DISCO_PATH_AUTO: {
      const int fast = N == 1 && variant == LOSS_CLIP ? DISCO_PATH_SYMMETRIC : DISCO_PATH_MATERIALIZED;
      if (whole) return fast;
      // a ragged share is padded to whole tiles: worth it once the padded block is more than a few tiles of work
      // (below that the call is launch-bound on either path and the fp32 one has fewer launches)
      return tiles && (B / N) * B >= RAGGED_MIN_BLOCK ? fast : DISCO_PATH_NAIVE;
    }
    case DISCO_PATH_NAIVE:
      return DISCO_PATH_NAIVE;
    case DISCO_PATH_MATERIALIZED:
      return tiles ? DISCO_PATH_MATERIALIZED : -DISCO_ERR_UNSUPPORTED;
    case DISCO_PATH_FUSED:
      return tiles ? DISCO_PATH_FUSED : -DISCO_ERR_UNSUPPORTED;
    case DISCO_PATH_SYMMETRIC:
      return N == 1 && variant == LOSS_CLIP && tiles ? DISCO_PATH_SYMMETRIC : -DISCO_ERR_UNSUPPORTED;
    default:
      return -DISCO_ERR_UNSUPPORTED;
  }
}

size_t workspace_need(int r, int64_t B, int64_t d, int32_t N, int variant) {
  if (r == DISCO_PATH_NAIVE) return naive_workspace_bytes(B, d, N, variant);
  // (the bf16 paths lay their workspace out for two blocks; the one-block loss uses the first half of each part)
  if (r == DISCO_PATH_MATERIALIZED) return mfma_stored_workspace_bytes(B, d, N, variant);
  if (r == DISCO_PATH_FUSED) return mfma_fused_workspace_bytes(B, d, N, variant);
  if (r == DISCO_PATH_SYMMETRIC) return mfma_sym_workspace_bytes(B, d);
  return 0;
}

}  // namespace

extern "C" int disco_resolve_path(int64_t B, int64_t d, int32_t N, int dtype, int path) {
  return resolve(B, d, N, dtype, path);
}

extern "C" size_t disco_workspace_bytes(int64_t B, int64_t d, int32_t N, int dtype, int path) {
  const int r = resolve(B, d, N, dtype, path);
  return r > 0 ? workspace_need(r, B, d, N, LOSS_CLIP) : 0;
}

extern "C" int disco_loss_fwd_bwd(const void* I, const void* T, int64_t B, int64_t d, int32_t rank, int32_t N,
                                  float s, int dtype, int path, int accumulate, float* loss, float* gI, float* gT,
                                  float* gs, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!I || !T || !loss || !gI || !gT || !gs) return DISCO_ERR_NULL;
  int r = resolve(B, d, N, dtype, path);
  if (r < 0) return -r;
  if (rank < 0 || rank >= N) return DISCO_ERR_SHAPE;
  const size_t need = workspace_need(r, B, d, N, LOSS_CLIP);
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0 || workspace_bytes < need)
    return DISCO_ERR_WORKSPACE;
  if (r != DISCO_PATH_NAIVE && !(aligned16(I) && aligned16(T) && aligned16(gI) && aligned16(gT))) return DISCO_ERR_UNSUPPORTED;

  Problem p;
  p.variant = LOSS_CLIP;
  p.I = I; p.T = T; p.B = B; p.d = d; p.rank = rank; p.N = N; p.b = B / N; p.s = s; p.dtype = dtype;
  p.accumulate = accumulate ? 1 : 0;
  p.loss = loss; p.gI = gI; p.gT = gT; p.gs = gs;
  p.ws = workspace; p.ws_bytes = workspace_bytes;
  p.stream = static_cast<hipStream_t>(hip_stream);
  if (r == DISCO_PATH_NAIVE) return naive_run(p);
  if (r == DISCO_PATH_SYMMETRIC) return mfma_sym_run(p);
  return r == DISCO_PATH_MATERIALIZED ? mfma_stored_run(p) : mfma_fused_run(p);
}

extern "C" int clip_loss_fwd_bwd(const void* I, const void* T, int64_t B, int64_t d, float s, int dtype, int path,
                                 float* loss, float* gI, float* gT, float* gs, void* workspace,
                                 size_t workspace_bytes, void* hip_stream) {
  return disco_loss_fwd_bwd(I, T, B, d, 0, 1, s, dtype, path, 0, loss, gI, gT, gs, workspace, workspace_bytes,
                            hip_stream);
}

// ---- the self-supervised (two-view) contrastive loss on the same kernels -------------------------------------
extern "C" int ntxent_resolve_path(int64_t B, int64_t d, int32_t N, int dtype, int path) {
  return resolve(B, d, N, dtype, path, LOSS_NTXENT);
}

extern "C" size_t ntxent_workspace_bytes(int64_t B, int64_t d, int32_t N, int dtype, int path) {
  const int r = resolve(B, d, N, dtype, path, LOSS_NTXENT);
  return r > 0 ? workspace_need(r, B, d, N, LOSS_NTXENT) : 0;
}

extern "C" int ntxent_loss_fwd_bwd(const void* Z, int64_t B, int64_t d, int32_t rank, int32_t N, float s, int dtype,
                                   int path, int accumulate, float* loss, float* gZ, float* gs, void* workspace,
                                   size_t workspace_bytes, void* hip_stream) {
  if (!Z || !loss || !gZ || !gs) return DISCO_ERR_NULL;
  const int r = resolve(B, d, N, dtype, path, LOSS_NTXENT);
  if (r < 0) return -r;
  if (rank < 0 || rank >= N) return DISCO_ERR_SHAPE;
  const size_t need = workspace_need(r, B, d, N, LOSS_NTXENT);
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0 || workspace_bytes < need)
    return DISCO_ERR_WORKSPACE;
  if (r != DISCO_PATH_NAIVE && !(aligned16(Z) && aligned16(gZ))) return DISCO_ERR_UNSUPPORTED;
  Problem p;
  p.variant = LOSS_NTXENT;
  p.I = Z; p.T = Z; p.B = B; p.d = d; p.rank = rank; p.N = N; p.b = B / N; p.s = s; p.dtype = dtype;
  p.accumulate = accumulate ? 1 : 0;
  p.loss = loss; p.gI = gZ; p.gT = gZ; p.gs = gs;
  p.ws = workspace; p.ws_bytes = workspace_bytes;
  p.stream = static_cast<hipStream_t>(hip_stream);
  if (r == DISCO_PATH_NAIVE) return naive_run(p);
  return r == DISCO_PATH_MATERIALIZED ? mfma_stored_run(p) : mfma_fused_run(p);
}

extern "C" const char* disco_status_string(int status) {
  switch (status) {
    case DISCO_OK: return "ok";
    case DISCO_ERR_NULL: return "a required pointer is NULL";
    case DISCO_ERR_SHAPE: return "invalid shape: need B, d, N > 0, B % N == 0, 0 <= rank < N";
    case DISCO_ERR_UNSUPPORTED: return "dtype/path value unknown, path does not support this shape and dtype, or a bf16 MFMA path was given a matrix that is not 16-byte aligned";
    case DISCO_ERR_WORKSPACE: return "workspace NULL, not 256-byte aligned, or smaller than disco_workspace_bytes() (static entry point: the call needs more than disco_static_scratch_bytes())";
    case DISCO_ERR_HIP: return "a HIP kernel launch failed";
    default: return "unknown status";
  }
}
