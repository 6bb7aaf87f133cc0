// Reference-grade GPU path: fp32 FMA arithmetic on the vector ALUs, any shape, either input dtype.
// The two b x B blocks of raw similarities live in the workspace in fp32 (the 2B^2/N memory model
// of Sec. 4.1) and are turned in place into (softmax - onehot); the four gradient contractions of
// Eq. 4-6 are plain tiled products.  Everything is deterministic (no float atomics).
#include "common.h"

namespace disco {
namespace {


__device__ __forceinline__ float load_feat(const void* base, int dtype, int64_t idx) {
  if (dtype == DISCO_BF16) {
    uint32_t u = static_cast<const uint16_t*>(base)[idx];
    return __uint_as_float(u << 16);
  }
  return static_cast<const float*>(base)[idx];
}

// Generic tiled product  out(m,n) = sum_k A(m,k) * Bm(k,n)  for one TM x TN output tile (TM, TN: 64 or 128).
// A and Bm are accessor functors (any layout, any dtype); entries outside the ranges count as 0.  256 threads as
// 16 x 16; a thread owns (TM/16) x (TN/16) outputs in pieces of 4: rows ty*4 + u (+ 64 for the second piece), columns
// tx*4 + v (+ 64), so that its LDS reads are 16-byte vectors, a wave's column reads are 256 contiguous bytes and
// its row reads 4 broadcast pieces: one LDS read per 8 (128 x 128: 16) multiply-adds.
// TK: reduction step.  AK / BK: the reduction index is the contiguous one in the memory behind A(m, k) / Bm(k, n);
// the fill loops run consecutive threads along it, otherwise along m / n, so that the loads coalesce either way.
// PREFETCH: fetch the next reduction step's operand pieces into registers while the current one
// is multiplied: pays where few workgroups share a compute unit (the query-side product), costs occupancy where
// many do.
template <int TM, int TN, int TK, bool AK, bool BK, bool PREFETCH, class FA, class FB, class FOut>
__device__ __forceinline__ void tile_product(int64_t M, int64_t Nn, int64_t K, int64_t m0, int64_t n0,
                                             FA A, FB Bm, FOut out) {
  typedef __attribute__((ext_vector_type(4))) float f32x4;
  constexpr int PM = TM / 64, PN = TN / 64;             // pieces of 4 rows / columns per thread
  __shared__ __attribute__((aligned(16))) float As[TK][TM + 4];
  __shared__ __attribute__((aligned(16))) float Bs[TK][TN + 4];
  const int tid = threadIdx.x;
  const int tx = tid % 16, ty = tid / 16;
  float acc[PM * 4][PN * 4] = {};
  constexpr int NA = TM * TK / 256, NB = TN * TK / 256;
  float ra[NA], rb[NB];
  auto fetch = [&](int64_t k0) {
#pragma unroll
    for (int r = 0; r < NA; ++r) {
      const int e = tid + r * 256, kk = AK ? e % TK : e / TM, mm = AK ? e / TK : e % TM;
      const int64_t m = m0 + mm, k = k0 + kk;
      ra[r] = (m < M && k < K) ? A(m, k) : 0.f;
    }
#pragma unroll
    for (int r = 0; r < NB; ++r) {
      const int e = tid + r * 256, kk = BK ? e % TK : e / TN, nn = BK ? e / TK : e % TN;
      const int64_t n = n0 + nn, k = k0 + kk;
      rb[r] = (n < Nn && k < K) ? Bm(k, n) : 0.f;
    }
  };
  if constexpr (PREFETCH) fetch(0);
  for (int64_t k0 = 0; k0 < K; k0 += TK) {
    if constexpr (PREFETCH) {
#pragma unroll
      for (int r = 0; r < NA; ++r) {
        const int e = tid + r * 256;
        As[AK ? e % TK : e / TM][AK ? e / TK : e % TM] = ra[r];
      }
#pragma unroll
      for (int r = 0; r < NB; ++r) {
        const int e = tid + r * 256;
        Bs[BK ? e % TK : e / TN][BK ? e / TK : e % TN] = rb[r];
      }
    } else {
      for (int e = tid; e < TM * TK; e += 256) {
        const int kk = AK ? e % TK : e / TM, mm = AK ? e / TK : e % TM;
        const int64_t m = m0 + mm, k = k0 + kk;
        As[kk][mm] = (m < M && k < K) ? A(m, k) : 0.f;
      }
      for (int e = tid; e < TK * TN; e += 256) {
        const int kk = BK ? e % TK : e / TN, nn = BK ? e / TK : e % TN;
        const int64_t n = n0 + nn, k = k0 + kk;
        Bs[kk][nn] = (n < Nn && k < K) ? Bm(k, n) : 0.f;
      }
    }
    __syncthreads();
    if constexpr (PREFETCH) { if (k0 + TK < K) fetch(k0 + TK); }
#pragma unroll
    for (int kk = 0; kk < TK; ++kk) {
      f32x4 a[PM], bb[PN];
#pragma unroll
      for (int p = 0; p < PM; ++p) a[p] = *reinterpret_cast<const f32x4*>(&As[kk][p * 64 + ty * 4]);
#pragma unroll
      for (int p = 0; p < PN; ++p) bb[p] = *reinterpret_cast<const f32x4*>(&Bs[kk][p * 64 + tx * 4]);
#pragma unroll
      for (int u = 0; u < PM * 4; ++u)
#pragma unroll
        for (int v = 0; v < PN * 4; ++v) acc[u][v] = fmaf(a[u / 4][u % 4], bb[v / 4][v % 4], acc[u][v]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int u = 0; u < PM * 4; ++u)
#pragma unroll
    for (int v = 0; v < PN * 4; ++v) {
      int64_t m = m0 + (u / 4) * 64 + ty * 4 + u % 4, n = n0 + (v / 4) * 64 + tx * 4 + v % 4;
      if (m < M && n < Nn) out(m, n, acc[u][v]);
    }
}

// Output tile edges of the three products: 128 x 128 where the grid is large (b x B similarities, B x d key-side
// gradient), 64 x 64 for the b x d query-side gradient, whose grid would not fill the chip otherwise (it prefetches
// the next reduction step while it multiplies).  Reduction step 16 everywhere.
constexpr int TS = 128;
constexpr int TQ = 64;

struct BlockView {
  const void* X;   // b x d local rows (already offset to the rank's first row)
  const void* Y;   // B x d
  float* W;        // b x B fp32: raw similarities, later softmax - onehot
};

__device__ __forceinline__ BlockView block_view(const void* I, const void* T, int dtype, int64_t b, int64_t B,
                                                int64_t d, int rank, float* ws, int z) {
  size_t esz = dtype == DISCO_BF16 ? 2 : 4;
  const char* Ir = static_cast<const char*>(I) + (size_t)rank * b * d * esz;
  const char* Tr = static_cast<const char*>(T) + (size_t)rank * b * d * esz;
  BlockView v;
  v.X = z == 0 ? Ir : Tr;
  v.Y = z == 0 ? T : I;
  v.W = ws + (size_t)z * b * B;
  return v;
}

// Step 1 (Alg. 1 "scaled dot product similarities", without the multiplier): W[i][j] = <X_i, Y_j>.
__global__ __launch_bounds__(256) void naive_similarity(const void* I, const void* T, int dtype, int64_t b,
                                                         int64_t B, int64_t d, int rank, float* ws) {
  BlockView v = block_view(I, T, dtype, b, B, d, rank, ws, blockIdx.z);
  int64_t m0 = (int64_t)blockIdx.y * TS, n0 = (int64_t)blockIdx.x * TS;
  tile_product<TS, TS, 16, true, true, false>(
      b, B, d, m0, n0, [&](int64_t m, int64_t k) { return load_feat(v.X, dtype, m * d + k); },
      [&](int64_t k, int64_t n) { return load_feat(v.Y, dtype, n * d + k); },
      [&](int64_t m, int64_t n, float a) { v.W[m * B + n] = a; });
}

__device__ __forceinline__ float block_reduce(float v, bool is_max, float* red) {
  for (int o = 32; o > 0; o >>= 1) {
    float w = __shfl_xor(v, o);
    v = is_max ? fmaxf(v, w) : v + w;
  }
  int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
  __syncthreads();
  if (lane == 0) red[wave] = v;
  __syncthreads();
  float r = red[0];
  for (int w = 1; w < (int)(blockDim.x / 64); ++w) r = is_max ? fmaxf(r, red[w]) : r + red[w];
  return r;
}

// Step 2 (Alg. 1 cross_entropy_loss, and the softmax gradient of loss.backward()).  One workgroup per
// local row: lse_i = m + log(sum exp(z - m)) over z = s * W[i][:], ce_i = lse_i - z[label], then
// W[i][j] <- P_ij - [j = label].  The off-label mass is summed on its own so that P_label - 1 is
// formed as -(sum of the other terms)/(total) without cancellation.  Also the row's share of
// d/ds:  sum_j (P_ij - [j=label]) * W_ij.
// variant LOSS_NTXENT: the positive is the other view's row and column `self` (the row itself) takes no part:
// it is left out of the maximum and the sums and its gradient entry is 0.
__global__ __launch_bounds__(256) void naive_row_softmax(float* ws, int64_t b, int64_t B, int rank, float s,
                                                          float* row_ce, float* row_ds, int variant) {
  __shared__ float red[4];
  const int z = blockIdx.y;
  const int64_t i = blockIdx.x;
  float* w = ws + ((size_t)z * b + i) * B;
  const int64_t label = label_row((int64_t)rank * b + i, B, variant);
  const int64_t self = masked_col((int64_t)rank * b + i, variant);
  float mx = -INFINITY;
  for (int64_t j = threadIdx.x; j < B; j += 256)
    if (j != self) mx = fmaxf(mx, s * w[j]);
  mx = block_reduce(mx, true, red);
  float off = 0.f;
  for (int64_t j = threadIdx.x; j < B; j += 256)
    if (j != label && j != self) off += expf(s * w[j] - mx);
  off = block_reduce(off, false, red);
  const float zl = s * w[label];
  const float el = expf(zl - mx);
  const float tot = off + el;
  const float inv = 1.f / tot;
  float ds = 0.f;
  for (int64_t j = threadIdx.x; j < B; j += 256) {
    float cs = w[j];
    float g = (j == label) ? -off * inv : (j == self) ? 0.f : expf(s * cs - mx) * inv;
    ds = fmaf(g, cs, ds);
    w[j] = g;
  }
  ds = block_reduce(ds, false, red);
  if (threadIdx.x == 0) {
    // ce = log(tot) - (zl - mx).  When the label holds most of the mass this is log1p(off/el), which
    // keeps relative accuracy for a saturated softmax (s = 100) where the plain difference cancels.
    row_ce[(size_t)z * b + i] = (el > 0.5f * tot) ? log1pf(off / el) : logf(tot) - (zl - mx);
    row_ds[(size_t)z * b + i] = ds;
  }
}

// Step 3: loss_r = c * sum ce, gs_r = c * sum ds  (Alg. 1 `(loss_i + loss_t)/2` with c = 1/(2B)).
// One workgroup, fixed summation order.
__global__ __launch_bounds__(256) void naive_scalars(const float* row_ce, const float* row_ds, int64_t n, float c,
                                                      int accumulate, float* loss, float* gs) {
  __shared__ float red[4];
  float a = 0.f, g = 0.f;
  for (int64_t i = threadIdx.x; i < n; i += 256) { a += row_ce[i]; g += row_ds[i]; }
  a = block_reduce(a, false, red);
  g = block_reduce(g, false, red);
  if (threadIdx.x == 0) {
    *loss = (accumulate ? *loss : 0.f) + c * a;
    *gs = (accumulate ? *gs : 0.f) + c * g;
  }
}

// Step 4, key side (inter-rank term of Eq. 5 plus the key-side intra term): for every global row j
//   gT[j] (+)= c s sum_i G^A[i][j] I_r[i]      (z = 0)
//   gI[j] (+)= c s sum_i G^C[i][j] T_r[i]      (z = 1)
__global__ __launch_bounds__(256) void naive_key_grad(const void* I, const void* T, int dtype, int64_t b, int64_t B,
                                                       int64_t d, int rank, float* ws, float cs, int accumulate,
                                                       float* gI, float* gT) {
  const int z = blockIdx.z;
  BlockView v = block_view(I, T, dtype, b, B, d, rank, ws, z);
  float* out = z == 0 ? gT : gI;
  // the B key rows run along grid.x (up to 2^31 - 1 workgroups), the feature columns along grid.y
  int64_t m0 = (int64_t)blockIdx.x * TS, n0 = (int64_t)blockIdx.y * TS;
  tile_product<TS, TS, 16, true, false, false>(
      B, d, b, m0, n0, [&](int64_t m, int64_t k) { return v.W[k * B + m]; },
      [&](int64_t k, int64_t n) { return load_feat(v.X, dtype, k * d + n); },
      [&](int64_t m, int64_t n, float a) {
        float prev = accumulate ? out[m * d + n] : 0.f;
        out[m * d + n] = prev + cs * a;
      });
}

// Step 5, query side (the intra-rank terms of Eq. 4 that land in the rank's own rows):
//   gI[R_r][i] += c s sum_j G^A[i][j] T[j]     (z = 0)
//   gT[R_r][i] += c s sum_j G^C[i][j] I[j]     (z = 1)
// Runs after naive_key_grad on the same stream, so the rows already hold the key-side part.
__global__ __launch_bounds__(256) void naive_query_grad(const void* I, const void* T, int dtype, int64_t b,
                                                         int64_t B, int64_t d, int rank, float* ws, float cs,
                                                         float* gI, float* gT) {
  const int z = blockIdx.z;
  BlockView v = block_view(I, T, dtype, b, B, d, rank, ws, z);
  float* out = (z == 0 ? gI : gT) + (size_t)rank * b * d;
  int64_t m0 = (int64_t)blockIdx.y * TQ, n0 = (int64_t)blockIdx.x * TQ;
  tile_product<TQ, TQ, 16, true, false, true>(
      b, d, B, m0, n0, [&](int64_t m, int64_t k) { return v.W[m * B + k]; },
      [&](int64_t k, int64_t n) { return load_feat(v.Y, dtype, k * d + n); },
      [&](int64_t m, int64_t n, float a) { out[m * d + n] += cs * a; });
}

inline unsigned cdiv(int64_t a, int64_t b) { return (unsigned)((a + b - 1) / b); }

}  // namespace

size_t naive_workspace_bytes(int64_t B, int64_t d, int32_t N, int variant) {
  (void)d;
  int64_t b = B / N;
  const size_t nb = (size_t)loss_blocks(variant);
  return align_up(nb * b * B * sizeof(float)) + 2 * align_up(nb * b * sizeof(float));
}

int naive_run(const Problem& p) {
  const int64_t b = p.b, B = p.B, d = p.d;
  float* W = static_cast<float*>(p.ws);
  char* base = static_cast<char*>(p.ws);
  const unsigned nb = (unsigned)loss_blocks(p.variant);
  float* row_ce = reinterpret_cast<float*>(base + align_up((size_t)nb * b * B * sizeof(float)));
  float* row_ds = reinterpret_cast<float*>(reinterpret_cast<char*>(row_ce) + align_up((size_t)nb * b * sizeof(float)));
  const float c = loss_norm(B, p.variant);
  const float cs = c * p.s;

  stage_mark(p.stream, 0);
  naive_similarity<<<dim3(cdiv(B, TS), cdiv(b, TS), nb), 256, 0, p.stream>>>(p.I, p.T, p.dtype, b, B, d, p.rank, W);
  stage_mark(p.stream, 1);
  naive_row_softmax<<<dim3((unsigned)b, nb), 256, 0, p.stream>>>(W, b, B, p.rank, p.s, row_ce, row_ds, p.variant);
  stage_mark(p.stream, 2);
  naive_scalars<<<1, 256, 0, p.stream>>>(row_ce, row_ds, (int64_t)nb * b, c, p.accumulate, p.loss, p.gs);
  stage_mark(p.stream, 3);
  naive_key_grad<<<dim3(cdiv(B, TS), cdiv(d, TS), nb), 256, 0, p.stream>>>(p.I, p.T, p.dtype, b, B, d, p.rank, W, cs,
                                                                          p.accumulate, p.gI, p.gT);
  stage_mark(p.stream, 4);
  naive_query_grad<<<dim3(cdiv(d, TQ), cdiv(b, TQ), nb), 256, 0, p.stream>>>(p.I, p.T, p.dtype, b, B, d, p.rank, W, cs,
                                                                            p.gI, p.gT);
  stage_mark(p.stream, 5);
  return hipGetLastError() == hipSuccess ? DISCO_OK : DISCO_ERR_HIP;
}

}  // namespace disco
