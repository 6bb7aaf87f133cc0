/*
 * disco.h - C ABI of the decomposed CLIP contrastive loss for one MI355X (gfx950).
 *
 * The operation is the second segment of the paper's Alg. 1 (Sec. 4.2): given the
 * all-gathered image and text features I, T (B x d), the rank r of N and the logit
 * multiplier s (Alg. 1's `t`), rank r forms only the two b x B logit blocks
 *     A = s * I_r * T^T        C = s * T_r * I^T            (b = B/N, Sec. 4.1 Eq. 6)
 * takes the row-wise softmax cross-entropy of each against the global diagonal
 * (label of local row i is column r*b + i, Alg. 1 `labels = arange(b) + b*rank`),
 * and back-propagates: the intra-rank gradient lands in rows R_r = [r*b, (r+1)*b)
 * and the inter-rank gradient in ALL B rows of gI and gT (Sec. 4.1 Eq. 4, 5).  The
 * all_reduce of Eq. 7 is replaced by adding the N simulated ranks' outputs into the
 * same device buffers (`accumulate`).
 *
 * Normalisation: Alg. 1's mean over b rows, the /2 and the all_reduce(AVG) compose
 * to the factor c = 1/(2B).  Every per-rank output carries c, so the SUM over
 * r = 0..N-1 of (loss, gI, gT, gs) equals the loss and gradients of the original
 * non-distributed CLIP loss (Eq. 1, Eq. 3).
 *
 * Pointers: every data pointer is a DEVICE pointer owned by the caller; the library
 * allocates and frees nothing and keeps no pointer after the call returns.  All work
 * is enqueued on `hip_stream` (a hipStream_t passed as void*, NULL = default stream)
 * and the call returns without synchronising.  I and T are read-only and must not
 * overlap any output or the workspace.
 *
 * Errors are return codes.  On any status other than DISCO_OK and DISCO_ERR_HIP
 * nothing was launched and no output was touched.
 *
 * Stream capture: the calls enqueue kernels only (no allocation, no memset, no
 * synchronisation), so a caller may capture them in a HIP graph.  The first call of a
 * process on one of the bf16 MFMA paths also raises the dynamic-LDS limit of its kernels
 * (hipFuncSetAttribute), which is not a stream operation: make one call outside any
 * capture first.
 *
 * Inputs: any finite values.  The features are expected L2-normalised (what CLIP feeds
 * the loss) and that is the fast case; rows of other norms, positives that are not the
 * row maximum, duplicate and all-zero rows give the same results as the definition, and
 * on the bf16 MFMA paths a row whose every logit lies more than about 110 below its
 * Cauchy-Schwarz bound s*|x_i|*max_j|y_j| is recomputed on a slower path (its query tile of
 * 256 rows is redone).  NaN or infinity in I, T or s propagates to the outputs.
 */
#ifndef DISCO_H
#define DISCO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DISCO_API __attribute__((visibility("default")))

typedef enum {
  DISCO_OK = 0,
  DISCO_ERR_NULL = 1,        /* a required pointer is NULL */
  DISCO_ERR_SHAPE = 2,       /* B<=0, d<=0, N<=0, B % N != 0, rank outside [0,N), B > 2^24, d > 2^16, B/N > 65535*64 */
  DISCO_ERR_UNSUPPORTED = 3, /* unknown dtype/path value, the path cannot run this shape/dtype, or a bf16 MFMA
                                path was handed I, T, gI or gT that is not 16-byte aligned */
  DISCO_ERR_WORKSPACE = 4,   /* workspace NULL/misaligned or smaller than disco_workspace_bytes() */
  DISCO_ERR_HIP = 5          /* a kernel launch failed; outputs are undefined */
} disco_status;

/* dtype of I and T only.  Outputs and all accumulation are fp32. */
typedef enum { DISCO_F32 = 0, DISCO_BF16 = 1 } disco_dtype;

/*
 * DISCO_PATH_NAIVE        fp32 arithmetic (fp32 matrix instruction for fp32 features, vector-ALU FMA for
 *                         part of the bf16 case), fp32 logit blocks kept in the workspace (2*b*B*4
 *                         bytes: the paper's 2B^2/N memory model, Sec. 4.1).  Any B, d, N; either dtype.
 * DISCO_PATH_MATERIALIZED bf16 MFMA tiles.  The logit blocks are computed once; the un-normalised
 *                         softmax numerators are kept in bf16 (2*b*B*2 bytes) and feed the two
 *                         gradient contractions (12*b*B*d flop).  Needs dtype bf16, d % 64 == 0,
 *                         B <= 2^23.  A share b that is not a whole number of 256-row tiles is rounded up
 *                         to one inside the workspace (zero-padded copies of I, T and the rank's rows,
 *                         2*(B+b)*d*2 more bytes; the padding takes part in no softmax, sum or output),
 *                         so the call costs what the rounded-up shape costs.
 * DISCO_PATH_FUSED        bf16 MFMA tiles, streaming: a forward pass keeps the row sums on chip and
 *                         writes nothing of size b x B; the backward pass recomputes the logits one
 *                         key panel (at most 16384 keys) at a time and contracts each panel while
 *                         it is cache-resident (16*b*B*d flop, workspace 2*b*W*2 bytes for panel
 *                         width W).  Shape limits of MATERIALIZED (ragged shares padded as there).
 * DISCO_PATH_SYMMETRIC    bf16 MFMA tiles, N = 1 only (the non-decomposed loss, Eq. 1 / Fig. 1): the B x B
 *                         similarity matrix is computed once and serves both directions (text -> image is
 *                         its transpose); one matrix of numerators (B*B*2 bytes) against one exponent
 *                         reference, turned in place into the combined gradient matrix, then one contraction
 *                         per feature gradient: 6*B^2*d flop instead of 12.  Shape limits of MATERIALIZED
 *                         (a batch that is not whole 256-row tiles is padded in the workspace as there).  Inputs whose rows' or columns' largest logits lie more than about
 *                         60 (base 2) under the largest positive-pair logit are handed over, inside the same
 *                         call, to the MATERIALIZED kernels, so the workspace is sized for those as well.
 * DISCO_PATH_AUTO         the fastest path that supports the arguments: SYMMETRIC (N = 1) or
 *                         MATERIALIZED when their shape limits hold, else NAIVE.  Feature widths that are not
 *                         a multiple of 64, fp32 inputs, and ragged shares of blocks smaller than
 *                         b*B = 2^18 logits (launch-bound either way) therefore run on the vector ALUs, for
 *                         large shapes an order of magnitude slower; disco_resolve_path tells which path a
 *                         call takes.
 */
typedef enum {
  DISCO_PATH_AUTO = 0,
  DISCO_PATH_NAIVE = 1,
  DISCO_PATH_MATERIALIZED = 2,
  DISCO_PATH_FUSED = 3,
  DISCO_PATH_SYMMETRIC = 4
} disco_path;

/* The concrete path (1..4) that `path` resolves to for these arguments, or a negative
 * disco_status (e.g. -DISCO_ERR_UNSUPPORTED) if the arguments are invalid for it.  Host only. */
DISCO_API int disco_resolve_path(int64_t B, int64_t d, int32_t N, int dtype, int path);

/* Bytes of device workspace the call needs (256-byte aligned pointer).  0 on invalid arguments.
 * Host only, no HIP call. */
DISCO_API size_t disco_workspace_bytes(int64_t B, int64_t d, int32_t N, int dtype, int path);

/*
 * One rank's forward + backward (Alg. 1 lines "scaled dot product similarities" to
 * "loss backward"; Sec. 4.1 Eq. 4-6).
 *
 *   I, T        device, row-major B x d, contiguous, dtype `dtype` (bf16 = raw 16-bit patterns),
 *               16-byte aligned for the bf16 MFMA paths (as gI and gT).
 *               Expected L2-normalised by the caller; gradients are w.r.t. the arrays as given.
 *   B, d        global batch and feature width.   rank, N: 0 <= rank < N, B % N == 0.
 *   s           logit multiplier (1/temperature).
 *   accumulate  0: loss, gI, gT, gs are overwritten (all B rows of gI and gT are defined);
 *               1: the rank's results are added to what the buffers hold.
 *   loss, gs    device, one fp32 each.      gI, gT: device, row-major B x d fp32.
 *   workspace   device scratch of at least disco_workspace_bytes(...) bytes, 256-byte aligned;
 *               contents before and after the call are unspecified.
 */
DISCO_API int disco_loss_fwd_bwd(const void* I, const void* T, int64_t B, int64_t d, int32_t rank, int32_t N,
                       float s, int dtype, int path, int accumulate,
                       float* loss, float* gI, float* gT, float* gs,
                       void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * The original non-distributed CLIP loss (Eq. 1, Fig. 1): the whole B x B similarity matrix on
 * one device.  Equal in value to disco_loss_fwd_bwd(rank = 0, N = 1, accumulate = 0) and the same call
 * (DISCO_PATH_AUTO resolves to DISCO_PATH_SYMMETRIC when the shape allows); the workspace size is
 * disco_workspace_bytes(B, d, 1, dtype, path).
 */
DISCO_API int clip_loss_fwd_bwd(const void* I, const void* T, int64_t B, int64_t d, float s, int dtype, int path,
                      float* loss, float* gI, float* gT, float* gs,
                      void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * The self-supervised contrastive loss on the same decomposition (Sec. 4.1, last sentence, and the Conclusion say
 * that it applies; the paper prints no formula, so the loss is SimCLR's).  Z (B x d, B = 2M even) holds two views of
 * M samples, view one in rows 0..M-1 and view two in rows M..2M-1; the positive of row i is row (i + M) mod B and a
 * row is never its own negative:
 *     l_i = log sum_{k != i} exp(s <z_i, z_k>) - s <z_i, z_p(i)>,      L = (1/B) sum_i l_i.
 * Rank r of N owns rows [r*b, (r+1)*b), b = B/N, forms its b x B block of logits and returns, each carrying 1/B so
 * that the SUM over ranks is the full result: loss_r, gs_r = d loss_r / d s, and gZ_r (B x d fp32): the query-side
 * gradient in the rank's own rows plus the key-side gradient in all B rows (the part Eq. 5 / Eq. 7 would send to
 * the other ranks).  Arguments, ownership, errors, paths, `accumulate`, stream and capture rules are those of
 * disco_loss_fwd_bwd, with one matrix Z for I and T and one gradient gZ; B odd is DISCO_ERR_SHAPE; there is no
 * symmetric path for this loss.  ntxent_workspace_bytes / ntxent_resolve_path are this entry's
 * counterparts of disco_workspace_bytes / disco_resolve_path.
 */
DISCO_API int ntxent_resolve_path(int64_t B, int64_t d, int32_t N, int dtype, int path);
DISCO_API size_t ntxent_workspace_bytes(int64_t B, int64_t d, int32_t N, int dtype, int path);
DISCO_API int ntxent_loss_fwd_bwd(const void* Z, int64_t B, int64_t d, int32_t rank, int32_t N, float s, int dtype, int path,
                                  int accumulate, float* loss, float* gZ, float* gs,
                                  void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * disco_loss_fwd_bwd for callers that cannot allocate device memory or keep a workspace of their own: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and
 * status codes as disco_loss_fwd_bwd without the workspace pair: the workspace is a static device array of
 * DISCO_STATIC_SCRATCH_BYTES inside the library (every GPU the library runs on holds its own copy until the
 * process ends).  The call allocates and frees nothing; on its first use on a device it looks the array's
 * address up once (not a stream operation: make one call outside any capture first, as for the MFMA paths).
 * Returns DISCO_ERR_WORKSPACE, before any launch, when the arguments need more than the array holds
 * (disco_workspace_bytes(...) > disco_static_scratch_bytes()), DISCO_ERR_HIP when the address lookup fails.
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different streams or
 * threads) race on it and must be serialised by the caller; nothing in it needs to start at zero, each call
 * overwrites what it reads.
 */
#define DISCO_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
DISCO_API size_t disco_static_scratch_bytes(void);
DISCO_API int disco_loss_fwd_bwd_static(const void* I, const void* T, int64_t B, int64_t d, int32_t rank, int32_t N,
                                        float s, int dtype, int path, int accumulate,
                                        float* loss, float* gI, float* gT, float* gs, void* hip_stream);

/*
 * Stage timing for benchmarks (measurement only; the paper reports per-operator times in Table 4).
 * `events` is a caller-owned array of `count` hipEvent_t handles (created with timing enabled), or
 * NULL to switch stage timing off (the default).  The setting is process-wide: it is meant for a
 * benchmark that owns the process, not for use next to other callers of the library.  While set, every
 * disco_loss_fwd_bwd / clip_loss_fwd_bwd call made from any thread records events[0] on its stream before its first
 * kernel and events[k] after stage k, for as many stages as fit in `count` (NULL entries are skipped, so that a
 * caller can bracket one stage alone and leave the others undisturbed); the caller synchronises
 * and reads the intervals with hipEventElapsedTime.  The library keeps the pointer until it is
 * replaced.  Stages of DISCO_PATH_MATERIALIZED (DISCO_STAGES_MATERIALIZED = 6):
 *   1 row norms + positive-pair logits   2 logit tiles + softmax numerators   3 row merge + scaled transpose
 *   4 key-side gradient GEMM             5 query-side split GEMM              6 query finalize + scalars
 * Stages of DISCO_PATH_NAIVE (DISCO_STAGES_NAIVE = 5): similarity, row softmax, scalars, key grad, query grad.
 * Stages of DISCO_PATH_FUSED (DISCO_STAGES_FUSED = 5): row norms + positive-pair logits, streaming forward
 *   (row sums only), row merge + scaled transpose, all key panels (recompute + both gradient GEMMs),
 *   query finalize + scalars.
 * Stages of DISCO_PATH_SYMMETRIC (DISCO_STAGES_SYMMETRIC = 7): row norms + positive-pair logits + reference, logit
 *   tiles with row and column sums, both merges + transpose, combining pass, key-side GEMM, query-side split GEMM,
 *   finalize + scalars.
 * Returns DISCO_OK, or DISCO_ERR_SHAPE if count < 0.
 */
#define DISCO_STAGES_MATERIALIZED 6
#define DISCO_STAGES_NAIVE 5
#define DISCO_STAGES_FUSED 5
#define DISCO_STAGES_SYMMETRIC 7
DISCO_API int disco_set_stage_events(void** events, int count);

/*
 * Measurement only: `workgroups` workgroups of 8 waves each issue `iters` x 8 bf16 MFMA 32x32x16 instructions per
 * wave (32768 flop each) from registers, with no memory traffic: what the matrix cores sustain once the clock
 * management has settled, the ceiling under the published peak that a tile kernel works against.  varied != 0: the
 * operands differ in sign, exponent and mantissa from element to element (as real data does); 0: in the mantissa
 * only, which draws less power.  sink: one device
 * float (never written); clocks: two device uint64, filled by workgroup 0 with its elapsed shader-clock ticks and
 * its elapsed ticks of the fixed 100 MHz counter (their ratio is the shader clock in units of 100 MHz).
 */
DISCO_API int disco_mfma_probe(int workgroups, int iters, int varied, float* sink, unsigned long long* clocks, void* hip_stream);

/*
 * Feature preparation on either side of the loss.  In Alg. 1 the encoders hand the features to the loss
 * and take the feature gradients back; the paper prints neither the row normalisation nor the
 * parametrisation of `t`.  Reading taken (CLIP's convention): unit-norm rows, u = x / max(|x|, 1e-12),
 * and s = min(exp(theta), s_max).  All pointers are device pointers owned by the caller; work is enqueued
 * on hip_stream; nothing is allocated; errors are status codes returned before anything is launched.
 *
 * disco_normalize_fwd: X rows x d raw features (row-major, contiguous, dtype x_dtype), U rows x d normalised
 *   rows (dtype u_dtype: DISCO_BF16 feeds the MFMA path), inv_norm rows fp32 = 1 / max(|x|, 1e-12), kept for
 *   the backward.  Norms and scaling in fp32; bf16 output rounded to nearest even.  X and U may be the same
 *   buffer when the dtypes are equal.
 * disco_normalize_bwd: G rows x d fp32 = d loss / d u (rows of gI or gT), X and inv_norm as in the forward,
 *   DX rows x d fp32 = (G - <G, u> u) inv_norm, or G inv_norm where the 1e-12 cap was active.  DX may be G.
 */
DISCO_API int disco_normalize_fwd(const void* X, int64_t rows, int64_t d, int x_dtype, void* U, int u_dtype, float* inv_norm,
                                  void* hip_stream);
DISCO_API int disco_normalize_bwd(const float* G, const void* X, int x_dtype, const float* inv_norm, int64_t rows, int64_t d,
                                  float* DX, void* hip_stream);

/*
 * Logit multiplier on the device: *s = min(exp(*theta), s_max) and, given *gs = d loss / d s (the gs output of
 * the loss entry points, summed over ranks), *gtheta (+)= *gs exp(*theta) where exp(*theta) <= s_max, else 0.
 * One fp32 each.  (The loss entry points take s by value: read *s back, or keep theta on the host.)
 */
DISCO_API int disco_logit_scale_fwd(const float* theta, float s_max, float* s, void* hip_stream);
DISCO_API int disco_logit_scale_bwd(const float* theta, float s_max, const float* gs, float* gtheta, int accumulate,
                                    void* hip_stream);

/* Static, NUL-terminated description of a status code. */
DISCO_API const char* disco_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* DISCO_H */
