// Reference-grade GPU path: fp32 arithmetic (fp32 matrix instruction or vector-ALU FMA), any shape, either input dtype.
// The two b x B blocks of raw similarities live in the workspace in fp32 (the 2B^2/N memory model
// of Sec. 4.1) and are turned in place into (softmax - onehot); the four gradient contractions of
// Eq. 4-6 are plain tiled products.  Everything is deterministic (no float atomics).
#include "common.h"

namespace disco {
namespace {


// DT: DISCO_F32 or DISCO_BF16, a template argument of the product kernels so that no load sits behind a branch
// (the fill loops then issue all their loads before they wait for the first).
template <int DT>
__device__ __forceinline__ float load_feat(const void* base, int64_t idx) {
  if (DT == DISCO_BF16) {
    uint32_t u = static_cast<const uint16_t*>(base)[idx];
    return __uint_as_float(u << 16);
  }
  return static_cast<const float*>(base)[idx];
}

// Generic tiled product  out(m,n) = sum_k A(m,k) * Bm(k,n)  for one TM x TN output tile (TM, TN: 64 or 128), on the
// vector ALUs.  A and Bm are accessor functors (any layout, any dtype); entries outside the ranges count as 0.
// 256 threads as 16 x 16; a thread owns (TM/16) x (TN/16) outputs in pieces of 4: rows ty*4 + u (+ 64 for the second
// piece), columns tx*4 + v (+ 64), so that its LDS reads are 16-byte vectors, a wave's column reads are 256
// contiguous bytes and its row reads 4 broadcast pieces: one LDS read per 8 (128 x 128: 16) multiply-adds.
// TK: reduction step.  AK / BK: the reduction index is the contiguous one in the memory behind A(m, k) / Bm(k, n);
// the fill loops run consecutive threads along it, otherwise along m / n, so that the loads coalesce either way.
template <int TM, int TN, int TK, bool AK, bool BK, class FA, class FB, class FOut>
__device__ __forceinline__ void tile_product_valu(int64_t M, int64_t Nn, int64_t K, int64_t m0, int64_t n0,
                                                  FA A, FB Bm, FOut out) {
  typedef __attribute__((ext_vector_type(4))) float f32x4;
  constexpr int PM = TM / 64, PN = TN / 64;             // pieces of 4 rows / columns per thread
  __shared__ __attribute__((aligned(16))) float As[TK][TM + 4];
  __shared__ __attribute__((aligned(16))) float Bs[TK][TN + 4];
  const int tid = threadIdx.x;
  const int tx = tid % 16, ty = tid / 16;
  float acc[PM * 4][PN * 4] = {};
  for (int64_t k0 = 0; k0 < K; k0 += TK) {
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
    __syncthreads();
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

// The same product on the matrix cores in fp32 (v_mfma_f32_32x32x2_f32: fp32 products, fp32 sums).  256 threads as
// 2 x 2 waves, each wave a (TM/2) x (TN/2) part of the tile in 32 x 32 accumulator blocks.  One instruction takes
// A[32 rows][2 k] and B[2 k][32 columns], one value per lane: lane l supplies row (column) l % 32 of reduction index
// l / 32, and holds of the 32 x 32 result the entries (row 8 (r / 4) + 4 (l / 32) + r % 4, column l % 32), r < 16.
// The fill fetches a whole reduction step into registers before it writes any of it to LDS (all loads in flight at
// once; the accumulators live in the other half of the register file, so there is room).  LDS row pitch TM + 1: a
// k-contiguous fill writes 32 consecutive k of one row, all banks once; an operand read takes 32 consecutive floats.
template <int TM, int TN, int TK, bool AK, bool BK, class FA, class FB, class FOut>
__device__ __forceinline__ void tile_product_mfma(int64_t M, int64_t Nn, int64_t K, int64_t m0, int64_t n0,
                                                  FA A, FB Bm, FOut out) {
  typedef __attribute__((ext_vector_type(16))) float f32x16;
  constexpr int WM = TM / 2, WN = TN / 2, NBM = WM / 32, NBN = WN / 32;
  __shared__ float As[TK][TM + 1];
  __shared__ float Bs[TK][TN + 1];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wr = wave >> 1, wc = wave & 1, l32 = lane & 31, lh = lane >> 5;
  f32x16 acc[NBM][NBN];
#pragma unroll
  for (int u = 0; u < NBM; ++u)
#pragma unroll
    for (int v = 0; v < NBN; ++v)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[u][v][r] = 0.f;
  for (int64_t k0 = 0; k0 < K; k0 += TK) {
    {
      constexpr int NA = TM * TK / 256, NB = TN * TK / 256;
      float ra[NA], rb[NB];
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
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < TK; kk += 2) {
      float a[NBM], bb[NBN];
#pragma unroll
      for (int u = 0; u < NBM; ++u) a[u] = As[kk + lh][wr * WM + u * 32 + l32];
#pragma unroll
      for (int v = 0; v < NBN; ++v) bb[v] = Bs[kk + lh][wc * WN + v * 32 + l32];
#pragma unroll
      for (int u = 0; u < NBM; ++u)
#pragma unroll
        for (int v = 0; v < NBN; ++v) acc[u][v] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u], bb[v], acc[u][v], 0, 0, 0);
    }
    __syncthreads();
  }
#pragma unroll
  for (int u = 0; u < NBM; ++u)
#pragma unroll
    for (int v = 0; v < NBN; ++v)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int64_t m = m0 + wr * WM + u * 32 + (r >> 2) * 8 + lh * 4 + (r & 3), n = n0 + wc * WN + v * 32 + l32;
        if (m < M && n < Nn) out(m, n, acc[u][v][r]);
      }
}

// Which product runs where (measured at B = 32768, d = 512, b = 4096; ms for the two logit blocks):
//  * fp32 features: the matrix-core product everywhere (similarities 2.6 against 4.0 on the vector ALUs, key side 2.6
//    against 4.4, query side 3.2 against 4.6);
//  * bf16 features (the widths the MFMA path does not take): their 2-byte loads make the batched fill slow, and the
//    vector-ALU product with its element-by-element fill wins for the similarities (3.5 against 5.0) and the key
//    side (4.3 against 5.2); the query side, whose left operand is the fp32 matrix in the workspace, stays on the
//    matrix cores (5.0 against 5.4).
// Output tiles: 128 x 128 where the grid is large (b x B similarities, B x d key-side gradient), 64 x 64 for the
// b x d query-side gradient, whose grid would not fill the chip otherwise.
constexpr int TS = 128;
constexpr int TQ = 64;

// AKV: the left operand's fill order on the vector-ALU variant (the key side runs 8 % faster there with consecutive
// threads along the reduction index although its left operand is contiguous along m)
template <int DT, int TM, int TN, bool AK, bool BK, bool AKV, class FA, class FB, class FOut>
__device__ __forceinline__ void tile_product(int64_t M, int64_t Nn, int64_t K, int64_t m0, int64_t n0, FA A, FB Bm, FOut out) {
  if constexpr (DT == DISCO_F32) tile_product_mfma<TM, TN, 16, AK, BK>(M, Nn, K, m0, n0, A, Bm, out);
  else tile_product_valu<TM, TN, 16, AKV, BK>(M, Nn, K, m0, n0, A, Bm, out);
}

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
template <int DT>
__global__ __launch_bounds__(256) void naive_similarity(const void* I, const void* T, int dtype, int64_t b,
                                                         int64_t B, int64_t d, int rank, float* ws) {
  BlockView v = block_view(I, T, dtype, b, B, d, rank, ws, blockIdx.z);
  int64_t m0 = (int64_t)blockIdx.y * TS, n0 = (int64_t)blockIdx.x * TS;
  tile_product<DT, TS, TS, true, true, true>(
      b, B, d, m0, n0, [&](int64_t m, int64_t k) { return load_feat<DT>(v.X, m * d + k); },
      [&](int64_t k, int64_t n) { return load_feat<DT>(v.Y, n * d + k); },
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

// One pass of a workgroup over a row of B floats: x <- f(j, x) for every column j (stored back if WRITE).  The row
// starts at any float offset of a 256-byte aligned buffer: `head` (0..3) columns up to the first 16-byte boundary,
// then 16-byte pieces, then up to 3 columns; the at most six odd columns go one per thread.
template <bool WRITE, class F>
__device__ __forceinline__ void row_visit(float* w, int64_t B, int head, F f) {
  typedef __attribute__((ext_vector_type(4))) float f32x4;
  const int64_t nvec = (B - head) >> 2;
  for (int64_t q = threadIdx.x; q < nvec; q += 256) {
    f32x4* p = reinterpret_cast<f32x4*>(w + head) + q;
    f32x4 v = *p;
    const int64_t j = head + q * 4;
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] = f(j + e, v[e]);
    if (WRITE) *p = v;
  }
  const int64_t t0 = head + nvec * 4;
  const int nrest = head + (int)(B - t0);
  if ((int)threadIdx.x < nrest) {
    const int64_t j = (int)threadIdx.x < head ? (int64_t)threadIdx.x : t0 + ((int)threadIdx.x - head);
    const float x = f(j, w[j]);
    if (WRITE) w[j] = x;
  }
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
  const int64_t row0 = ((int64_t)z * b + i) * B;
  float* w = ws + row0;
  const int64_t to_boundary = (4 - (row0 & 3)) & 3;
  const int head = (int)(to_boundary < B ? to_boundary : B);
  const int64_t label = label_row((int64_t)rank * b + i, B, variant);
  const int64_t self = masked_col((int64_t)rank * b + i, variant);
  float mx = -INFINITY;
  row_visit<false>(w, B, head, [&](int64_t j, float x) {
    if (j != self) mx = fmaxf(mx, s * x);
    return x;
  });
  mx = block_reduce(mx, true, red);
  float off = 0.f;
  row_visit<false>(w, B, head, [&](int64_t j, float x) {
    if (j != label && j != self) off += expf(s * x - mx);
    return x;
  });
  off = block_reduce(off, false, red);
  const float zl = s * w[label];
  const float el = expf(zl - mx);
  const float tot = off + el;
  const float inv = 1.f / tot;
  float ds = 0.f;
  row_visit<true>(w, B, head, [&](int64_t j, float x) {
    const float g = (j == label) ? -off * inv : (j == self) ? 0.f : expf(s * x - mx) * inv;
    ds = fmaf(g, x, ds);
    return g;
  });
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
template <int DT>
__global__ __launch_bounds__(256) void naive_key_grad(const void* I, const void* T, int dtype, int64_t b, int64_t B,
                                                       int64_t d, int rank, float* ws, float cs, int accumulate,
                                                       float* gI, float* gT) {
  const int z = blockIdx.z;
  BlockView v = block_view(I, T, dtype, b, B, d, rank, ws, z);
  float* out = z == 0 ? gT : gI;
  // the B key rows run along grid.x (up to 2^31 - 1 workgroups), the feature columns along grid.y
  int64_t m0 = (int64_t)blockIdx.x * TS, n0 = (int64_t)blockIdx.y * TS;
  tile_product<DT, TS, TS, false, false, true>(
      B, d, b, m0, n0, [&](int64_t m, int64_t k) { return v.W[k * B + m]; },
      [&](int64_t k, int64_t n) { return load_feat<DT>(v.X, k * d + n); },
      [&](int64_t m, int64_t n, float a) {
        float prev = accumulate ? out[m * d + n] : 0.f;
        out[m * d + n] = prev + cs * a;
      });
}

// Step 5, query side (the intra-rank terms of Eq. 4 that land in the rank's own rows):
//   gI[R_r][i] += c s sum_j G^A[i][j] T[j]     (z = 0)
//   gT[R_r][i] += c s sum_j G^C[i][j] I[j]     (z = 1)
// Runs after naive_key_grad on the same stream, so the rows already hold the key-side part.
template <int DT>
__global__ __launch_bounds__(256) void naive_query_grad(const void* I, const void* T, int dtype, int64_t b,
                                                         int64_t B, int64_t d, int rank, float* ws, float cs,
                                                         float* gI, float* gT) {
  const int z = blockIdx.z;
  BlockView v = block_view(I, T, dtype, b, B, d, rank, ws, z);
  float* out = (z == 0 ? gI : gT) + (size_t)rank * b * d;
  int64_t m0 = (int64_t)blockIdx.y * TQ, n0 = (int64_t)blockIdx.x * TQ;
  tile_product_mfma<TQ, TQ, 32, true, false>(
      b, d, B, m0, n0, [&](int64_t m, int64_t k) { return v.W[m * B + k]; },
      [&](int64_t k, int64_t n) { return load_feat<DT>(v.Y, k * d + n); },
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
  const bool bf = p.dtype == DISCO_BF16;
  const dim3 sim_grid(cdiv(B, TS), cdiv(b, TS), nb);
  if (bf) naive_similarity<DISCO_BF16><<<sim_grid, 256, 0, p.stream>>>(p.I, p.T, p.dtype, b, B, d, p.rank, W);
  else naive_similarity<DISCO_F32><<<sim_grid, 256, 0, p.stream>>>(p.I, p.T, p.dtype, b, B, d, p.rank, W);
  stage_mark(p.stream, 1);
  naive_row_softmax<<<dim3((unsigned)b, nb), 256, 0, p.stream>>>(W, b, B, p.rank, p.s, row_ce, row_ds, p.variant);
  stage_mark(p.stream, 2);
  naive_scalars<<<1, 256, 0, p.stream>>>(row_ce, row_ds, (int64_t)nb * b, c, p.accumulate, p.loss, p.gs);
  stage_mark(p.stream, 3);
  const dim3 key_grid(cdiv(B, TS), cdiv(d, TS), nb);
  if (bf) naive_key_grad<DISCO_BF16><<<key_grid, 256, 0, p.stream>>>(p.I, p.T, p.dtype, b, B, d, p.rank, W, cs, p.accumulate, p.gI, p.gT);
  else naive_key_grad<DISCO_F32><<<key_grid, 256, 0, p.stream>>>(p.I, p.T, p.dtype, b, B, d, p.rank, W, cs, p.accumulate, p.gI, p.gT);
  stage_mark(p.stream, 4);
  const dim3 query_grid(cdiv(d, TQ), cdiv(b, TQ), nb);
  if (bf) naive_query_grad<DISCO_BF16><<<query_grid, 256, 0, p.stream>>>(p.I, p.T, p.dtype, b, B, d, p.rank, W, cs, p.gI, p.gT);
  else naive_query_grad<DISCO_F32><<<query_grid, 256, 0, p.stream>>>(p.I, p.T, p.dtype, b, B, d, p.rank, W, cs, p.gI, p.gT);
  stage_mark(p.stream, 5);
  return hipGetLastError() == hipSuccess ? DISCO_OK : DISCO_ERR_HIP;
}

}  // namespace disco
