// Internal declarations shared by the host dispatch and the kernel files of libdisco.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/disco.h"

namespace disco {

// One of the two logit blocks of a rank (Sec. 4.1 Eq. 6).  Block A: X = I_r, Y = T, query-side
// gradient goes to gI rows R_r and key-side gradient to all rows of gT; block C is the mirror image.
struct Problem {
  const void* I;
  const void* T;
  int64_t B, d;
  int32_t rank, N;
  int64_t b;          // B / N
  float s;
  int dtype;
  int accumulate;
  float* loss;
  float* gI;
  float* gT;
  float* gs;
  void* ws;
  size_t ws_bytes;
  hipStream_t stream;
  int variant;        // LOSS_CLIP: two blocks, label = own row.  LOSS_NTXENT: I = T = Z (one matrix, one block,
                      // gI = gT = gZ), label = the other view's row, the self-similarity is left out
};

enum { LOSS_CLIP = 0, LOSS_NTXENT = 1 };

// Global row of the positive of global row g, and the column that is left out of row g's softmax (-1: none).
__host__ __device__ inline int64_t label_row(int64_t g, int64_t B, int variant) {
  if (variant == LOSS_NTXENT) return g + B / 2 < B ? g + B / 2 : g - B / 2;
  return g;
}
__host__ __device__ inline int64_t masked_col(int64_t g, int variant) { return variant == LOSS_NTXENT ? g : -1; }
__host__ __device__ inline int loss_blocks(int variant) { return variant == LOSS_NTXENT ? 1 : 2; }
// Normalisation: 1/(2B) for the two directions of the CLIP loss, 1/B for the single one of the two-view loss.
__host__ __device__ inline float loss_norm(int64_t B, int variant) { return (variant == LOSS_NTXENT ? 1.0f : 0.5f) / (float)B; }

// Benchmark stage timing (see disco_set_stage_events): records events[k] on `st` if it exists.
void stage_mark(hipStream_t st, int k);

inline size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }

size_t naive_workspace_bytes(int64_t B, int64_t d, int32_t N, int variant = LOSS_CLIP);
int naive_run(const Problem& p);

// the bf16 tile kernels can take the shape (materialized path; a rank share that is not a whole number of 256-row
// tiles is zero-padded in the workspace) / the share is whole tiles (what the fused and symmetric paths need too)
bool mfma_supported(int64_t B, int64_t d, int32_t N, int dtype, int variant = LOSS_CLIP);
bool mfma_whole_tiles(int64_t B, int32_t N);
size_t mfma_stored_workspace_bytes(int64_t B, int64_t d, int32_t N, int variant = LOSS_CLIP);
int mfma_stored_run(const Problem& p);
size_t mfma_fused_workspace_bytes(int64_t B, int64_t d, int32_t N, int variant = LOSS_CLIP);
int mfma_fused_run(const Problem& p);
size_t mfma_sym_workspace_bytes(int64_t B, int64_t d);
int mfma_sym_run(const Problem& p);      // N = 1, the CLIP loss only

}  // namespace disco
