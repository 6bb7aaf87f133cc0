// bf16 MFMA path ("materialized"): the two b x B logit blocks are computed once on the matrix cores,
// their un-normalised softmax numerators are kept in bf16, and the two gradient contractions of each
// block (Eq. 4-6) are MFMA GEMMs over those numerators.  12*b*B*d executed flops per call.
//
// For one block with query rows X (b x d, the rank's rows) and key rows Y (B x d):
//   z_ij   = s <x_i, y_j>                      z2 = z * log2(e)   (all exponentials are base 2)
//   ref2_i = z2 of the positive pair (i, label_i), lifted where needed so that no z2_ij - ref2_i
//            exceeds 100 (overflow guard from the row norms, Cauchy-Schwarz)
//   E_ij   = exp2(z2_ij - ref2_i)  for j != label_i, stored as bf16 (b x B);  E_i,label = 0 in the
//            store and kept separately in fp32 as e_i
//   tot_i  = sum_j E_ij + e_i,  beta_i = 1/tot_i,  P_ij = beta_i E_ij,
//   ce_i   = log(tot_i / e_i),  P_i,label - 1 = -(sum_j E_ij)/tot_i       (no cancellation)
//   query-side gradient  gX_i = c s [ beta_i (E Y)_i + (P_i,label - 1) y_label ]
//   key-side gradient    gY_j = c s [ sum_i E_ij beta_i x_i  (+ (P_i,label - 1) x_i  if j = label_i) ]
//   d/ds share           c <gX_i / (c s), x_i>  summed over i   (sum_ij G_ij S_ij = <G Y, X>)
// Since lse_i >= z_i,label, every E_ij that underflows is negligible against the row total.  Where the guard
// lifts ref2_i so far above every logit of the row that the row total itself falls below 2^-60 (rows of large
// norm whose cosines are all small, positives far below the Cauchy-Schwarz bound), k_row_merge flags the row's
// query tile and k_logit_repair redoes that tile with the true row maximum as its reference (a slow path for
// inputs that are not CLIP-like; it returns at once when nothing is flagged).
//
// One 256x256x64 NT tile main loop (mfma_tile.h: 8 waves, each 128x64 = 4x2 MFMA 32x32x16 blocks, operands
// loaded global -> LDS directly into a ring of five units) serves all three contractions; operands whose
// reduction index is not the contiguous one in memory are read from LDS with transposing loads.
#include "common.h"
#include "mfma_tile.h"

namespace disco {
namespace {

using namespace tile;

constexpr float LOG2E = 1.4426950408889634f;
constexpr float REF_HEADROOM = 100.f;                    // largest exponent (base 2) a stored numerator may reach

constexpr int E_ROW_BYTES = BM * 2;                      // row of the bf16 tile copy in LDS (swizzled, not padded)
constexpr int E_TILE_BYTES = BN * E_ROW_BYTES;            // 128 KiB
constexpr int LOGIT_SMEM_BYTES = E_TILE_BYTES > SMEM_BYTES ? E_TILE_BYTES : SMEM_BYTES;
constexpr int GEMM_SMEM_BYTES = OUT_SMEM_BYTES > SMEM_BYTES ? OUT_SMEM_BYTES : SMEM_BYTES;

// Workgroup id -> tile, keeping the workgroups that share an XCD's L2 on neighbouring tiles.
// Workgroups are dealt round-robin to the 8 XCDs; XCD x takes the x-th contiguous eighth of the
// (padded) tile list.  Returns false for padding.
__device__ __forceinline__ bool xcd_linear(int total, int& lin) {
  const int w = blockIdx.x;
  const int chunk = (total + 7) / 8;
  lin = (w & 7) * chunk + (w >> 3);
  return (w >> 3) < chunk && lin < total;
}

// Tile (it, jt) at position lin of the walk over super-blocks of sbi query tiles x sbj key tiles: bands of sbj key
// tiles one after the other, inside a band the super-blocks along the query tiles, inside a super-block the query
// tile runs fastest.  The last super-block of either direction may be partial.
__device__ __forceinline__ void superblock_tile(int lin, int nI, int nJ, int sbi, int sbj, int& it, int& jt) {
  const int band = sbj * nI;
  const int jb = lin / band, r = lin - jb * band;
  const int hj = nJ - jb * sbj < sbj ? nJ - jb * sbj : sbj;
  const int ib = r / (sbi * hj), r2 = r - ib * sbi * hj;
  const int wi = nI - ib * sbi < sbi ? nI - ib * sbi : sbi;
  it = ib * sbi + r2 % wi;
  jt = jb * sbj + r2 / wi;
}

// ------------------------------------------------------------------------------------------------
struct BlockPtrs {
  const uint16_t* X;     // b x d, the rank's rows (zero rows past the real ones)
  const uint16_t* Y;     // B x d (zero rows past the real ones)
  uint16_t* E;           // b x W stored numerators of one key panel, in 16-byte atoms (e_index)
  float* lpart;          // (B/128) x b partial row sums (label column excluded)
  float* ediag;          // b: numerator of the label column
  float* zd2;            // b: z2 of the positive pair
  float* xnorm;          // b: |x_i|
  float* ref2;           // b: exponent reference of the row (written by the statistics pass, replaced by a repair)
  int* tileflag;         // b / 256: set when a row of that query tile has lost its row total to underflow
  const float* ymax_parts; // NORM_BLOCKS partial maxima of |y_j|^2
  float* beta;           // b
  float* gdiag;          // b: P_label - 1
  float* ce;             // b
  float* rowds;          // b
  uint16_t* Xs;          // d x b: (beta_i x_i)^T in bf16
  float* part;           // splitK x b x d partial query-side products
  float* gq;             // query-side gradient destination (gI for block A, gT for block C), B x d
  float* gk;             // key-side gradient destination, B x d
};
struct Blocks {
  BlockPtrs z[2];
  int variant;           // LOSS_CLIP or LOSS_NTXENT (label and left-out column of a row, see common.h)
  int nblk;              // blocks in use: 2 for the CLIP loss, 1 for the two-view loss and for the symmetric full loss
  const int* gate;       // nullptr: the kernel always runs; else it runs only while *gate == gate_value (the symmetric
  int gate_value;        // full-loss path hands over to the two-block path through this flag)
  int64_t rows, keys;    // the rank's rows and the batch as the caller has them.  The kernels' own b / B arguments are
                         // these rounded up to whole 256-row tiles; where they differ (a ragged share), X and Y are
                         // zero-padded copies, query rows >= rows and key columns >= keys are padding
};

__device__ __forceinline__ bool gated_off(const Blocks& bl) { return bl.gate != nullptr && *bl.gate != bl.gate_value; }

__device__ __forceinline__ float wave_sum(float v) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// Exponent reference (base 2) of a row: its positive-pair logit, lifted to the row's Cauchy-Schwarz bound minus the
// headroom where that is larger.  One explicit fma, so that every kernel that forms it gets the same bits.
__device__ __forceinline__ float row_reference(float zd2, float xnorm, float ymax, float s2) {
  return fmaxf(zd2, __fmaf_rn(fabsf(s2) * xnorm, ymax, -REF_HEADROOM));
}

constexpr int NORM_BLOCKS = 512;     // workgroups per matrix that take row norms = partial maxima per matrix
static_assert(NORM_BLOCKS == NTHREADS, "the logit kernel folds the partial maxima one per thread");

// Preparation, two kinds of workgroup in one launch (they are independent of each other):
//  * blockIdx.x < 2 NORM_BLOCKS: partial maximum over rows of |row|^2 of I (first NORM_BLOCKS workgroups) or T,
//    for the overflow guard, to wgmax[which * NORM_BLOCKS + index].  A wave takes 8 rows at a time (one 16-byte
//    load per lane and row in flight, d is a multiple of 8) and reduces the 8 row sums with interleaved
//    butterflies.  No atomics: the consumers fold the partial maxima (max is exact, so order does not matter).
//  * the rest: positive-pair logit and query norm of every local row, one wave per (block, row); the first of
//    these workgroups also clears the query-tile repair flags of both blocks.  The positive of local row i is
//    key row label_row(rank b + i): the same global row for the CLIP loss, the other view's row for the two-view loss.
//    B, b: the real sizes; bp: b rounded up to whole tiles (the padding rows get a zero logit and a zero norm).
__global__ __launch_bounds__(256) void k_prep(Blocks bl, const uint16_t* I, const uint16_t* T, int64_t B, int64_t b, int64_t bp, int64_t d,
                                              int rank, float s2, float* wgmax) {
  if (gated_off(bl)) return;
  __shared__ float red[4];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (blockIdx.x < 2 * NORM_BLOCKS) {
    const int which = blockIdx.x / NORM_BLOCKS, idx = blockIdx.x % NORM_BLOCKS;
    const uint16_t* M = which == 0 ? I : T;
    float best = 0.f;
    for (int64_t row0 = ((int64_t)idx * 4 + wave) * 8; row0 < B; row0 += (int64_t)NORM_BLOCKS * 32) {
      float a[8];
#pragma unroll
      for (int r = 0; r < 8; ++r) a[r] = 0.f;
      for (int64_t k = lane * 8; k < d; k += 512) {
        u32x4 v[8];
#pragma unroll
        for (int r = 0; r < 8; ++r) {
          const int64_t row = row0 + r < B ? row0 + r : B - 1;     // clamp: a repeated row does not change the max
          v[r] = *reinterpret_cast<const u32x4*>(M + row * d + k);
        }
#pragma unroll
        for (int r = 0; r < 8; ++r)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            a[r] = fmaf(bf16_lo(v[r][q]), bf16_lo(v[r][q]), a[r]);
            a[r] = fmaf(bf16_hi(v[r][q]), bf16_hi(v[r][q]), a[r]);
          }
      }
#pragma unroll
      for (int o = 32; o > 0; o >>= 1)
#pragma unroll
        for (int r = 0; r < 8; ++r) a[r] += __shfl_xor(a[r], o);
#pragma unroll
      for (int r = 0; r < 8; ++r) best = fmaxf(best, a[r]);
    }
    if (lane == 0) red[wave] = best;
    __syncthreads();
    if (threadIdx.x == 0) wgmax[which * NORM_BLOCKS + idx] = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    return;
  }
  const int64_t rb = (bp + 3) / 4;                      // row workgroups per block
  const int64_t q = (int64_t)blockIdx.x - 2 * NORM_BLOCKS;
  if (q == 0)
    for (int64_t it = threadIdx.x; it < bp / BN; it += 256) { bl.z[0].tileflag[it] = 0; bl.z[1].tileflag[it] = 0; }
  const BlockPtrs& p = bl.z[q / rb];
  const int64_t i = (q % rb) * 4 + wave;
  if (i >= bp) return;
  if (i >= b) {
    if (lane == 0) { p.zd2[i] = 0.f; p.xnorm[i] = 0.f; }
    return;
  }
  const uint16_t* x = p.X + i * d;
  const uint16_t* y = p.Y + label_row((int64_t)rank * b + i, B, bl.variant) * d;
  float dot = 0.f, nn = 0.f;
  for (int64_t k = lane * 8; k < d; k += 512) {          // 16-byte pieces (d is a multiple of 8, the rows are 16-byte aligned)
    const u32x4 xw = *reinterpret_cast<const u32x4*>(x + k), yw = *reinterpret_cast<const u32x4*>(y + k);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const float x0 = bf16_lo(xw[q]), x1 = bf16_hi(xw[q]);
      dot = fmaf(x0, bf16_lo(yw[q]), dot);
      dot = fmaf(x1, bf16_hi(yw[q]), dot);
      nn = fmaf(x0, x0, nn);
      nn = fmaf(x1, x1, nn);
    }
  }
  dot = wave_sum(dot);
  nn = wave_sum(nn);
  if (lane == 0) { p.zd2[i] = s2 * dot; p.xnorm[i] = sqrtf(nn); }
}

// Operands of a ragged share (the rank's rows or the batch are not whole 256-row tiles): zero-padded copies of I and T
// (Bp rows each) and of the rank's rows of both (bp rows each), so that the tile kernels read whole tiles of
// memory that exists and the padding contributes exact zeros to every contraction.  16-byte pieces, grid-stride.
__global__ __launch_bounds__(256) void k_pad_operands(const uint16_t* I, const uint16_t* T, int64_t B, int64_t Bp, int64_t b, int64_t bp,
                                                      int64_t d, int rank, uint16_t* Ipad, uint16_t* Tpad, uint16_t* XI, uint16_t* XT) {
  const int64_t cpr = d >> 3;                              // 16-byte pieces per row
  const int64_t nY = Bp * cpr, nX = bp * cpr;
  for (int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x; c < 2 * (nY + nX); c += (int64_t)gridDim.x * 256) {
    const int seg = c < nY ? 0 : c < 2 * nY ? 1 : c < 2 * nY + nX ? 2 : 3;
    const int64_t w = c - (seg == 0 ? 0 : seg == 1 ? nY : seg == 2 ? 2 * nY : 2 * nY + nX);
    const int64_t row = w / cpr, piece = w - row * cpr;
    const uint16_t* src = (seg & 1) ? T : I;
    uint16_t* dst = seg == 0 ? Ipad : seg == 1 ? Tpad : seg == 2 ? XI : XT;
    const bool there = seg < 2 ? row < B : row < b;
    const int64_t srow = seg < 2 ? row : (int64_t)rank * b + row;
    u32x4 v = {0u, 0u, 0u, 0u};
    if (there) v = *reinterpret_cast<const u32x4*>(src + srow * d + piece * 8);
    *reinterpret_cast<u32x4*>(dst + row * d + piece * 8) = v;
  }
}

// Element (i, jl) of a stored numerator panel of width W: 16-byte atoms of 8 consecutive keys, by groups of 64 query
// rows, inside a group key piece by key piece (formats FMT_KA / FMT_RA of mfma_tile.h).
// (The definition of the layout; the epilogue below forms the same address piecewise, which the compiler turns into
// a percent faster code than a call of this function.)
[[maybe_unused]] __device__ __forceinline__ int64_t e_index(int64_t i, int64_t jl, int64_t W) {
  return ((i >> 6) * (W >> 3) + (jl >> 3)) * 512 + (i & 63) * 8 + (jl & 7);
}

// Epilogue of one logit tile: numerators from the accumulators, row sums, the bf16 numerators to memory.
// Each lane holds, per accumulator quad, 4 consecutive key columns of one query row, lanes l and l + 32 the two
// halves of 8 consecutive keys; one v_permlane32_swap per register pair gives the lower lane the whole atom of an
// even key piece and the upper lane that of the odd piece next to it, and the 32 lanes of a half-wave (32
// consecutive query rows) then store 512 contiguous bytes of the panel (see e_index): no LDS, no barrier, so
// the waves of a workgroup need not meet between the main loops of consecutive tiles.
// MASK_DIAG: the tile contains label columns, which are stored as 0 and kept in fp32 in ediag.
// Local query row i is global row g0 + i; its label is key row label_row(g0 + i), and for the two-view loss its own
// key row g0 + i is left out of its softmax (stored as 0, in no sum), and so are the padding columns from key row
// nkeys (the batch size) on (MASK_EDGE only:
// the caller takes that variant for the tiles they fall into).  LOCAL (with STATS): the row sums and the label numerators
// are added into rs / kept in ed (registers of the lane, indexed like ref2) instead of being written to lpart / ediag.
// jl0: first key column of the tile relative to the panel of width W that p.E holds.  STREAM: streaming stores
// (written once, read by later kernels: keeps the operand tiles in L2).  STAGE: also leave the bf16 tile in LDS,
// row-major 256 x 256 (8-byte granules XOR-swizzled with the row: conflict-free 8-byte writes and 16-byte reads),
// for a caller that wants sums down its columns.
constexpr int64_t NO_SELF = -((int64_t)1 << 40);

// Do label columns or left-out columns of the 256 query rows from global row g on fall among key rows [j0, j0 + BM)?
// (Only such tiles pay for finding those columns.  The rows of a tile of the two-view loss may lie in both views.)
__device__ __forceinline__ bool tile_has_marked_columns(int64_t g, int64_t B, int variant, int64_t j0) {
  auto hits = [&](int64_t lo, int64_t hi) { return lo < j0 + BM && j0 < hi; };      // key rows [lo, hi)
  if (variant != LOSS_NTXENT) return hits(g, g + BN);
  const int64_t M = B / 2;
  bool h = hits(g, g + BN);                                                          // the rows' own columns
  const int64_t hi1 = g + BN < M ? g + BN : M;                                       // rows of view one: label g' + M
  if (g < hi1) h = h || hits(g + M, hi1 + M);
  const int64_t lo2 = g > M ? g : M;                                                 // rows of view two: label g' - M
  if (lo2 < g + BN) h = h || hits(lo2 - M, g + BN - M);
  return h;
}

enum { MASK_NONE = 0, MASK_DIAG = 1, MASK_EDGE = 2 };     // MASK_EDGE: label / left-out columns and padding columns

template <bool STATS, bool STORE, int MASK, bool LOCAL = false, bool STAGE = false, bool STREAM = true>
__device__ __forceinline__ void logit_epilogue(const BlockPtrs& p, f32x16 (&acc)[4][2], char* smem, int64_t b, float s2, int64_t i0,
                                               int64_t j0, int64_t g0, int variant, int64_t nkeys, const float (&ref2)[2],
                                               int64_t jl0, int64_t W, float* rs = nullptr, float* ed = nullptr) {
  constexpr bool DIAG = MASK != MASK_NONE, EDGE = MASK == MASK_EDGE;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave >> 2, wn = wave & 3, half = lane >> 5;
#pragma unroll
  for (int bn = 0; bn < 2; ++bn) {
    const int il = wn * 64 + bn * 32 + (lane & 31);
    const int64_t i = i0 + il;
    const float ref = ref2[bn];
    // label column of row i, relative to this lane's first key column of the tile (any value outside
    // [0, 128) means the label is not among this lane's columns)
    const int64_t dl64 = (DIAG ? label_row(g0 + i, nkeys, variant) : 0) - (j0 + wm * 128 + half * 4);
    const int dl = dl64 >= 0 && dl64 < 128 ? (int)dl64 : -1;
    const int64_t dm64 = (variant == LOSS_NTXENT ? g0 + i : NO_SELF) - (j0 + wm * 128 + half * 4);
    const int dm = dm64 >= 0 && dm64 < 128 ? (int)dm64 : -1;
    // first padding column, relative like dl (128: none among this lane's columns)
    const int64_t jl64 = nkeys - (j0 + wm * 128 + half * 4);
    const int jlim = jl64 >= 128 ? 128 : jl64 > 0 ? (int)jl64 : 0;
    float rowsum = 0.f;
    char* lrow = smem + il * E_ROW_BYTES;
    // this lane's atom of the wave's first key piece pair: row i, key piece (jl0 + 128 wm) / 8 + half
    uint16_t* erow = STORE ? p.E + ((i >> 6) * (W >> 3) + ((jl0 + wm * 128) >> 3) + half) * 512 + (i & 63) * 8 : nullptr;
#pragma unroll
    for (int bm = 0; bm < 4; ++bm) {
      const int jl = wm * 128 + bm * 32 + half * 4;
      u32x2 pk[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        float e[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) e[r] = __builtin_amdgcn_exp2f(fmaf(acc[bm][bn][q * 4 + r], s2, -ref));
        if (DIAG) {
#pragma unroll
          for (int r = 0; r < 4; ++r)
            if (dl == bm * 32 + q * 8 + r) {
              if (STATS && LOCAL) ed[bn] = e[r];
              else if (STATS) p.ediag[i] = e[r];
              e[r] = 0.f;
            }
#pragma unroll
          for (int r = 0; r < 4; ++r)
            if (dm == bm * 32 + q * 8 + r || (EDGE && bm * 32 + q * 8 + r >= jlim)) e[r] = 0.f;
        }
        if (STATS) rowsum += (e[0] + e[1]) + (e[2] + e[3]);
        if (STORE || STAGE) {
          bf16x4 v;
#pragma unroll
          for (int r = 0; r < 4; ++r) v[r] = (__bf16)e[r];
          pk[q] = __builtin_bit_cast(u32x2, v);
          // 8-byte granule g of row il lives at granule g ^ (il & 31): the 32 rows of a half-wave (same g)
          // then cover all 64 banks once
          if (STAGE) *reinterpret_cast<u32x2*>(lrow + ((((jl >> 2) + q * 2) ^ (il & 31)) << 3)) = pk[q];
        }
      }
      if (STORE) {
#pragma unroll
        for (int qp = 0; qp < 2; ++qp) {
          // lanes 32..63 of the even piece's registers <-> lanes 0..31 of the odd piece's
          const auto w0 = __builtin_amdgcn_permlane32_swap(pk[2 * qp][0], pk[2 * qp + 1][0], false, false);
          const auto w1 = __builtin_amdgcn_permlane32_swap(pk[2 * qp][1], pk[2 * qp + 1][1], false, false);
          const u32x4 atom = {w0[0], w1[0], w0[1], w1[1]};
          u32x4* dst = reinterpret_cast<u32x4*>(erow + (bm * 4 + qp * 2) * 512);
          if (STREAM) __builtin_nontemporal_store(atom, dst);
          else *dst = atom;
        }
      }
    }
    if (STATS && LOCAL) {
      rs[bn] += rowsum;
    } else if (STATS) {
      rowsum += __shfl_xor(rowsum, 32);
      if (half == 0) p.lpart[((j0 >> 7) + wm) * b + i] = rowsum;
    }
  }
}

// Logit tile + softmax numerators for the key panel [jp0, jp0 + W).  Tile rows (MFMA M side) are key rows
// j, tile columns (N side) are query rows i, so that each lane holds 4 consecutive j of one query row per
// accumulator quad: 8-byte pieces of an E row and an in-lane row sum.
//   STATS: write the partial row sums and the label-column numerator (forward statistics);
//   STORE: write the bf16 numerators to E (panel-relative columns, atom storage, see e_index).
// materialized path: STATS and STORE, one panel = all keys.  fused path: a STATS-only pass over all
// keys (nothing of size b x B is written), then STORE-only passes that recompute one panel at a time.
// A STATS pass derives the rows' exponent references (row_reference; k_row_merge records the same values in ref2);
// a pass without STATS reads them from ref2, so that it sees the references a repair has replaced.
// b: the rank's rows rounded up to whole tiles; B: the key rows that exist (the panel widths cover them rounded up to
// whole tiles); g0: global row of the rank's first row.  RAGGED: the last key tile may hold padding columns (the
// instance without it keeps the tile walk free of that variant of the epilogue and of the registers it costs).
template <bool STATS, bool STORE, bool RAGGED = false>
__global__ __launch_bounds__(NTHREADS) void k_logit_tiles(Blocks bl, int64_t b, int64_t B, int64_t d, int64_t g0, float s2,
                                                          int64_t jp0, int64_t W, int sbi, int sbj, int nblk) {
  if (gated_off(bl)) return;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  // Persistent workgroups (one per compute unit) walk the tile lists of the nblk blocks in bl, one after the
  // other, with a stride of the grid size: a wave ends only when all its stores are acknowledged, so ending a
  // workgroup per tile would expose that latency and the launch of the next workgroup once per tile; here a
  // tile's stores drain while the next tile's operands are fetched.  gridDim.x is a multiple of 8, so a
  // workgroup stays on one XCD's contiguous eighth of the tile list.  The list runs over super-blocks of
  // sbi query tiles x sbj key tiles (sbi sbj <= 32; 8 x 4 where the shape allows, see superblock_tile): the
  // workgroups an XCD runs at one time then share sbi + sbj operand tiles in its L2.
  const int nI = (int)(b / BN), nJ = (int)(W / BM);
  const int total = nI * nJ;
  const int chunk = (total + 7) >> 3, padded = chunk << 3;
  const int lane = threadIdx.x & 63, wn = (threadIdx.x >> 6) & 3;
  // max_j |y_j| of each block's key matrix, folded from the partial maxima (one per thread)
  float ymax_z[2];
  {
    float* red = reinterpret_cast<float*>(smem);
#pragma unroll
    for (int z = 0; z < 2; ++z) {
      float m = bl.z[z].ymax_parts[threadIdx.x];
      for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
      if (lane == 0) red[z * 8 + (threadIdx.x >> 6)] = m;
    }
    __syncthreads();
#pragma unroll
    for (int z = 0; z < 2; ++z) {
      float m = red[z * 8];
#pragma unroll
      for (int w = 1; w < 8; ++w) m = fmaxf(m, red[z * 8 + w]);
      ymax_z[z] = sqrtf(m);
    }
    __syncthreads();
  }
  for (int v = blockIdx.x; v < nblk * padded; v += gridDim.x) {
    const int z = v >= padded ? 1 : 0;
    const int u = v - z * padded;
    const BlockPtrs& p = bl.z[z];
    const int lin = (u & 7) * chunk + (u >> 3);
    if ((u >> 3) >= chunk || lin >= total) continue;                  // padding of the eighths (workgroup-uniform)
    int it, jt;
    superblock_tile(lin, nI, nJ, sbi, sbj, it, jt);
    const int64_t i0 = (int64_t)it * BN, j0 = jp0 + (int64_t)jt * BM;

    // exponent reference of this lane's two query rows, fetched before the main loop so that the loads are
    // not waited for in the epilogue
    float ref2[2];
    {
      const float ymax = z ? ymax_z[1] : ymax_z[0];
#pragma unroll
      for (int bn = 0; bn < 2; ++bn) {
        const int64_t i = i0 + wn * 64 + bn * 32 + (lane & 31);
        ref2[bn] = STATS ? row_reference(p.zd2[i], p.xnorm[i], ymax, s2) : p.ref2[i];
      }
    }
    f32x16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    mainloop<FMT_K, FMT_K, true>(p.Y + j0 * d, d, p.X + i0 * d, d, (int)(d / BK), smem, acc);

    // Only the tiles that the label diagonal (or the left-out diagonal) crosses, or that hold padding columns, pay
    // for finding those columns.
    const bool diag = tile_has_marked_columns(g0 + i0, B, bl.variant, j0);
    if (diag || (RAGGED && j0 + BM > B)) logit_epilogue<STATS, STORE, RAGGED ? MASK_EDGE : MASK_DIAG>(p, acc, smem, b, s2, i0, j0, g0, bl.variant, B, ref2, j0 - jp0, W);
    else logit_epilogue<STATS, STORE, MASK_NONE>(p, acc, smem, b, s2, i0, j0, g0, bl.variant, B, ref2, j0 - jp0, W);
  }
}

constexpr float LN2 = 0.6931471805599453f;
constexpr float ROW_TOTAL_FLOOR = 0x1p-60f;

// beta, P_label - 1 and the cross-entropy of row i from its off-label sum, its label numerator and their total.
// ce = log(tot / ed); when the label numerator does not dominate it is taken from the exponents,
// log(tot) - (z2_label - ref2) ln 2, which stays finite when ed itself has underflowed.  Returns beta.
__device__ __forceinline__ float row_outputs(const BlockPtrs& p, int64_t i, float off, float ed, float tot) {
  const float beta = 1.f / tot;
  p.beta[i] = beta;
  p.gdiag[i] = -off / tot;
  p.ce[i] = (ed > 0.5f * tot) ? log1pf(off / ed) : logf(tot) - (p.zd2[i] - p.ref2[i]) * LN2;
  return beta;
}

// Xs[k][i] = bf16(scale_i x_ik) for the nrows (a multiple of 64) rows from i0 on, scale = the nrows floats at `scale`
// in LDS (nullptr: 1): the key-side contraction's right operand, with its reduction index contiguous.  All NTH threads
// of the workgroup (512 or 1024), 64 x 64 pieces through `tile` (64 x 65 floats of LDS).  The pieces of up to eight
// 64-feature tiles are fetched before the first is turned round, so that their loads are in flight together.
template <int NTH>
__device__ __forceinline__ void scale_transpose_rows(const BlockPtrs& p, int64_t b, int64_t d, int64_t i0, int nrows, const float* scale,
                                                     float (*tile)[65]) {
  constexpr int NPT = 1024 / NTH, AHEAD = 8;              // pieces of 4 features per thread and tile; tiles per batch
  const int t = threadIdx.x;
  for (int r0 = 0; r0 < nrows; r0 += 64)
    for (int64_t kc = 0; kc < d; kc += 64 * AHEAD) {
      u32x2 w[AHEAD][NPT];
#pragma unroll
      for (int a = 0; a < AHEAD; ++a)
        if (kc + a * 64 < d)
#pragma unroll
          for (int q = 0; q < NPT; ++q) {                 // 64 rows x 16 pieces of 4 features
            const int e = t + q * NTH, r = e >> 4, c4 = (e & 15) * 4;
            w[a][q] = *reinterpret_cast<const u32x2*>(p.X + (i0 + r0 + r) * d + kc + a * 64 + c4);
          }
#pragma unroll
      for (int a = 0; a < AHEAD; ++a) {
        const int64_t k0 = kc + a * 64;
        if (k0 >= d) break;
        __syncthreads();                                  // the tile's previous contents have been read
#pragma unroll
        for (int q = 0; q < NPT; ++q) {
          const int e = t + q * NTH, r = e >> 4, c4 = (e & 15) * 4;
          const float sc = scale ? scale[r0 + r] : 1.f;
          tile[r][c4 + 0] = sc * bf16_lo(w[a][q][0]);
          tile[r][c4 + 1] = sc * bf16_hi(w[a][q][0]);
          tile[r][c4 + 2] = sc * bf16_lo(w[a][q][1]);
          tile[r][c4 + 3] = sc * bf16_hi(w[a][q][1]);
        }
        __syncthreads();
#pragma unroll
        for (int q = 0; q < NPT; ++q) {                   // 64 features x 16 pieces of 4 rows
          const int e = t + q * NTH, k = e >> 4, i4 = (e & 15) * 4;
          bf16x4 v;
#pragma unroll
          for (int j = 0; j < 4; ++j) v[j] = (__bf16)tile[i4 + j][k];
          *reinterpret_cast<bf16x4*>(p.Xs + (k0 + k) * b + i0 + r0 + i4) = v;
        }
      }
    }
}

// Row totals -> beta, P_label - 1, cross-entropy.  A workgroup takes 64 rows; its 16 waves each add a
// sixteenth of the column parts (lane = row, so the reads are coalesced), combined in fixed order.
// nparts0 / nparts1: number of partial sums per row of block 0 / block 1.  global_ref (symmetric full loss): the one
// exponent reference every row shares; bad_flag: where that path records that a row or column total was lost
// (the per-rank paths flag the row's query tile for repair instead).  d > 0: the workgroup goes on to write its
// rows of Xs = (beta x)^T (a query tile that is repaired afterwards rewrites its rows there); d = 0: not.
__global__ __launch_bounds__(1024) void k_row_merge(Blocks bl, int64_t b, int nparts0, int nparts1, float s2,
                                                    const float* global_ref, int* bad_flag, int64_t d) {
  if (gated_off(bl)) return;
  const int nparts = blockIdx.y ? nparts1 : nparts0;
  __shared__ float red[16][64];
  __shared__ float ymax_w[8];
  __shared__ float beta_s[64];
  __shared__ float tile[64][65];
  const BlockPtrs& p = bl.z[blockIdx.y];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  // max_j |y_j| folded from the partial maxima exactly as k_logit_tiles folds it (max is exact in any order)
  if (threadIdx.x < NORM_BLOCKS) {
    float m = p.ymax_parts[threadIdx.x];
    for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
    if (lane == 0) ymax_w[wave] = m;
  }
  const int64_t i = (int64_t)blockIdx.x * 64 + lane;
  float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
  if (i < b) {
    int q = wave;
    for (; q + 112 < nparts; q += 128) {                 // eight loads in flight
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = p.lpart[(int64_t)(q + 16 * u) * b + i];
      a0 += v[0]; a1 += v[1]; a2 += v[2]; a3 += v[3];
      a0 += v[4]; a1 += v[5]; a2 += v[6]; a3 += v[7];
    }
    for (; q + 48 < nparts; q += 64) {
      a0 += p.lpart[(int64_t)q * b + i];
      a1 += p.lpart[(int64_t)(q + 16) * b + i];
      a2 += p.lpart[(int64_t)(q + 32) * b + i];
      a3 += p.lpart[(int64_t)(q + 48) * b + i];
    }
    for (; q < nparts; q += 16) a0 += p.lpart[(int64_t)q * b + i];
  }
  red[wave][lane] = (a0 + a1) + (a2 + a3);
  __syncthreads();
  if (wave == 0 && i < b) {
    if (i >= bl.rows) {                                 // a padding row: no weight anywhere, no flag
      p.ref2[i] = 0.f; p.beta[i] = 0.f; p.gdiag[i] = 0.f; p.ce[i] = 0.f;
      beta_s[lane] = 0.f;
    } else {
      float off = 0.f;
#pragma unroll
      for (int w = 0; w < 16; w += 4) off += (red[w][lane] + red[w + 1][lane]) + (red[w + 2][lane] + red[w + 3][lane]);
      float ym = ymax_w[0];
#pragma unroll
      for (int w = 1; w < 8; ++w) ym = fmaxf(ym, ymax_w[w]);
      p.ref2[i] = global_ref ? *global_ref : row_reference(p.zd2[i], p.xnorm[i], sqrtf(ym), s2);   // what the statistics pass used
      const float ed = p.ediag[i];
      const float tot = off + ed;
      beta_s[lane] = row_outputs(p, i, off, ed, tot);
      // The guard lifted the reference so far above every logit of this row that its total is (next to) lost:
      // the row's query tile is redone against the true row maximum.  Also catches non-finite totals.
      if (!(tot >= ROW_TOTAL_FLOOR)) {
        if (bad_flag) *bad_flag = 1;
        else p.tileflag[i >> 8] = 1;
      }
    }
  }
  if (d > 0 && (int64_t)blockIdx.x * 64 + 64 <= b) scale_transpose_rows<1024>(p, b, d, (int64_t)blockIdx.x * 64, 64, beta_s, tile);
}

// The statistics kernels of a flagged query tile, redone by one workgroup per (block, query tile): a first
// sweep over all keys finds every row's true maximum logit, which becomes its exponent reference (ref2), a
// second sweep forms the numerators (stored to E when STORE) and the row sums against it, and the rows'
// beta, P_label - 1 and cross-entropy are written directly.  Workgroups of tiles that are not flagged return
// at once, which is the normal case: the kernel then costs one launch.
template <bool STORE>
__global__ __launch_bounds__(NTHREADS) void k_logit_repair(Blocks bl, int64_t b, int64_t B, int64_t d, int rank, float s2) {
  if (gated_off(bl)) return;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int nI = (int)(b / BN), nJ = (int)(B / BM);
  const int z = blockIdx.x / nI, it = blockIdx.x % nI;
  const BlockPtrs& p = bl.z[z];
  if (p.tileflag[it] == 0) return;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, wm = wave >> 2, wn = wave & 3, half = lane >> 5;
  const int64_t i0 = (int64_t)it * BN;
  const int64_t g0 = (int64_t)rank * bl.rows;             // global row of the rank's first row
  float* red = reinterpret_cast<float*>(smem);            // [2][256] exchange between the two key halves
  f32x16 acc[4][2];
  float ref2[2] = {-INFINITY, -INFINITY};
  for (int jt = 0; jt < nJ; ++jt) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    mainloop<FMT_K, FMT_K, true>(p.Y + (int64_t)jt * BM * d, d, p.X + i0 * d, d, (int)(d / BK), smem, acc);
    const int64_t j0 = (int64_t)jt * BM;
    // the left-out column and the padding columns take no part in the maximum
    const bool has_self = bl.variant == LOSS_NTXENT && (g0 + i0 < j0 + BM) && (j0 < g0 + i0 + BN);
    const int64_t jl64 = bl.keys - (j0 + wm * 128 + half * 4);
    const int jlim = jl64 >= 128 ? 128 : jl64 > 0 ? (int)jl64 : 0;
#pragma unroll
    for (int bn = 0; bn < 2; ++bn) {
      const int64_t dm64 = g0 + i0 + wn * 64 + bn * 32 + (lane & 31) - (j0 + wm * 128 + half * 4);
#pragma unroll
      for (int bm = 0; bm < 4; ++bm)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int jl = bm * 32 + (e >> 2) * 8 + (e & 3);
          const bool skip = (has_self && dm64 == jl) || jl >= jlim;
          ref2[bn] = skip ? ref2[bn] : fmaxf(ref2[bn], acc[bm][bn][e] * s2);
        }
    }
  }
#pragma unroll
  for (int bn = 0; bn < 2; ++bn) {
    ref2[bn] = fmaxf(ref2[bn], __shfl_xor(ref2[bn], 32));
    if (half == 0) red[wm * 256 + wn * 64 + bn * 32 + lane] = ref2[bn];
  }
  __syncthreads();
#pragma unroll
  for (int bn = 0; bn < 2; ++bn) {
    const int il = wn * 64 + bn * 32 + (lane & 31);
    ref2[bn] = fmaxf(red[il], red[256 + il]);
    if (wm == 0 && half == 0) p.ref2[i0 + il] = ref2[bn];
  }
  __syncthreads();                                         // red is read before the main loop reuses the LDS

  float rs[2] = {0.f, 0.f}, ed[2] = {0.f, 0.f};
  for (int jt = 0; jt < nJ; ++jt) {
    const int64_t j0 = (int64_t)jt * BM;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    mainloop<FMT_K, FMT_K, true>(p.Y + j0 * d, d, p.X + i0 * d, d, (int)(d / BK), smem, acc);
    const bool diag = tile_has_marked_columns(g0 + i0, bl.keys, bl.variant, j0) || j0 + BM > bl.keys;
    if (diag) logit_epilogue<true, STORE, MASK_EDGE, true>(p, acc, smem, b, s2, i0, j0, g0, bl.variant, bl.keys, ref2, j0, B, rs, ed);
    else logit_epilogue<true, STORE, MASK_NONE, true>(p, acc, smem, b, s2, i0, j0, g0, bl.variant, bl.keys, ref2, j0, B, rs, ed);
  }
  // row totals: the four lanes (two key halves x two lane halves) that share a row; exactly one of them met the label
  __syncthreads();
#pragma unroll
  for (int bn = 0; bn < 2; ++bn) {
    rs[bn] += __shfl_xor(rs[bn], 32);
    ed[bn] += __shfl_xor(ed[bn], 32);
    if (half == 0) {
      red[wm * 256 + wn * 64 + bn * 32 + lane] = rs[bn];
      red[512 + wm * 256 + wn * 64 + bn * 32 + lane] = ed[bn];
    }
  }
  __syncthreads();
  if (wm == 0 && half == 0) {
#pragma unroll
    for (int bn = 0; bn < 2; ++bn) {
      const int il = wn * 64 + bn * 32 + lane;
      const float off = red[il] + red[256 + il], e = red[512 + il] + red[768 + il];
      p.ediag[i0 + il] = e;
      float beta = 0.f;
      if (i0 + il < bl.rows) beta = row_outputs(p, i0 + il, off, e, off + e);
      else { p.beta[i0 + il] = 0.f; p.gdiag[i0 + il] = 0.f; p.ce[i0 + il] = 0.f; }
      red[1024 + il] = beta;
    }
  }
  // the rows' share of Xs = (beta x)^T, written by k_row_merge with the betas that have just been replaced
  scale_transpose_rows<NTHREADS>(p, b, d, i0, BN, red + 1024, reinterpret_cast<float (*)[65]>(red + 1280));
}

// Xs = X^T for one block without any scaling (the symmetric full loss folds both normalisations into the stored
// matrix instead): a workgroup per 64 rows.
__global__ __launch_bounds__(1024) void k_transpose(Blocks bl, int64_t b, int64_t d) {
  if (gated_off(bl)) return;
  __shared__ float tile[64][65];
  scale_transpose_rows<1024>(bl.z[0], b, d, (int64_t)blockIdx.x * 64, 64, nullptr, tile);
}

// Key-side gradient without its label-column term: gk[j][k] (+)= cs * sum_i E[i][j] Xs[k][i].
// (The term [j = label_i] gdiag_i x_ik is added by k_query_finalize, which owns the rank's rows.)
// GEMM M = key rows j (operand E read transposed), N = feature index k, reduction over the rank's rows.
template <bool ACCUMULATE>
__global__ __launch_bounds__(NTHREADS) void k_key_grad(Blocks bl, int64_t b, int64_t d, float cs, int64_t jp0, int64_t W,
                                                       int nM, int nN) {
  if (gated_off(bl)) return;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const BlockPtrs& p = bl.z[blockIdx.y];
  int lin;
  if (!xcd_linear(nM * nN, lin)) return;
  const int nt = lin % nN, mt = lin / nN;
  const int64_t jl0 = (int64_t)mt * BM, k0 = (int64_t)nt * BN;     // key rows jp0 + jl0 .. of the panel
  f32x16 acc[4][2];
  const int ncols = d - k0 < BN ? (int)(d - k0) : BN;              // the last column tile may be partial (d % 64 == 0)
  mainloop<FMT_RA, FMT_K, false, true>(p.E + (jl0 >> 6) * 4096, (W >> 6) * 4096, p.Xs + k0 * b, b, (int)(b / BK), smem, acc, ncols);
  const int64_t left = bl.keys - (jp0 + jl0);                      // key rows that exist from this tile's first one on
  store_tile_f32<ACCUMULATE>(acc, smem, p.gk + (jp0 + jl0) * d + k0, d, cs, ncols, left < BM ? (int)left : BM);
}

// Query-side products, split over the key index: part[ks][i][k] = sum_{j in split ks} E[i][j] y_jk.
// GEMM M = query rows i, N = feature index k (operand Y read transposed), reduction over key rows.
// One-dimensional grid over (block z, split ks, row tile mt, column tile nt).  A "slice" is one (z, ks): all
// its workgroups read the same rows of Y, so slices are pinned to XCDs (workgroups are dealt round-robin to
// the 8 XCDs): with S = 2 splitk slices, either S/8 slices per XCD one after the other (S a multiple of 8), or
// 8/S XCDs per slice sharing its tiles (S divides 8).  Then Y comes in from the fabric once per slice instead
// of once per XCD.  Any other S falls back to slices laid out contiguously.
template <bool ACCUMULATE>
__global__ __launch_bounds__(NTHREADS) void k_query_partial(Blocks bl, int64_t b, int64_t d, int64_t jp0, int64_t W, int nM,
                                                            int nN, int splitk, int ktiles_per_split) {
  if (gated_off(bl)) return;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int T = nM * nN, S = bl.nblk * splitk;
  const int w = blockIdx.x, xcd = w & 7, r = w >> 3;
  int slice, tile;
  if (S % 8 == 0) {
    slice = xcd + 8 * (r / T);
    tile = r % T;
  } else if (8 % S == 0) {
    const int G = 8 / S;
    slice = xcd % S;
    tile = xcd / S + G * r;
  } else {
    slice = w / T;
    tile = w % T;
  }
  if (slice >= S || tile >= T) return;
  const BlockPtrs& p = bl.z[slice / splitk];
  const int ks = slice % splitk;
  const int nt = tile % nN, mt = tile / nN;
  const int64_t i0 = (int64_t)mt * BM, k0 = (int64_t)nt * BN;
  const int kt_total = (int)(W / BK);
  const int kt0 = ks * ktiles_per_split;
  int kts = kt_total - kt0;
  if (kts > ktiles_per_split) kts = ktiles_per_split;
  f32x16 acc[4][2];
  const int ncols = d - k0 < BN ? (int)(d - k0) : BN;              // the last column tile may be partial (d % 64 == 0)
  // (kts >= 1: the plan's split count is the number of splits that hold at least one K-step)
  mainloop<FMT_KA, FMT_R, false, true>(p.E + ((i0 >> 6) * (W >> 6) + kt0) * 4096, (W >> 6) * 4096,
                                   p.Y + (jp0 + (int64_t)kt0 * BK) * d + k0, d, kts, smem, acc, ncols);
  store_tile_f32<ACCUMULATE>(acc, smem, p.part + (int64_t)ks * b * d + i0 * d + k0, d, 1.0f, ncols);
}

// Sum over the split-K slices ks0, ks0 + step, ... (< splitk), in that order, of the 16-byte piece of row i at feature
// k of each slice (part[(ks * pitch + i) * d + k]); four loads in flight at a time (a plain loop waits for every load).
__device__ __forceinline__ f32x4 sum_slices(const float* part, int64_t pitch, int64_t i, int64_t d, int64_t k, int ks0, int step,
                                            int splitk) {
  auto piece = [&](int ks) { return *reinterpret_cast<const f32x4*>(part + ((int64_t)ks * pitch + i) * d + k); };
  f32x4 u = {0.f, 0.f, 0.f, 0.f};
  int ks = ks0;
  for (; ks + 3 * step < splitk; ks += 4 * step) {
    const f32x4 v0 = piece(ks), v1 = piece(ks + step), v2 = piece(ks + 2 * step), v3 = piece(ks + 3 * step);
    u += v0; u += v1; u += v2; u += v3;
  }
  for (; ks < splitk; ks += step) u += piece(ks);
  return u;
}

// Everything that lands in the rank's own rows, for both blocks at once.  With lab = label of local row i:
//   gI[lab] += cs (beta^A_i sum_ks part^A + gdiag^A_i T[lab])    query side of block A (Eq. 4)
//            + cs gdiag^C_i T[lab]                                label-column term of block C's key side
//   gT[lab] += cs (beta^C_i sum_ks part^C + gdiag^C_i I[lab]) + cs gdiag^A_i I[lab]
// and the rows' shares of d/ds, <query-side vector, x_i>, per block.  Fixed summation order.  One wave per row; ROWWG
// (small shares, where rows / 4 workgroups would leave most of the chip idle while each wave walks all the split-K
// slices): one workgroup per row, its four waves each add every fourth slice and wave 0 combines them.
// b: the real rows; bp: row pitch of the partial products.
template <bool ROWWG>
__global__ __launch_bounds__(256) void k_query_finalize(Blocks bl, int64_t b, int64_t bp, int64_t d, int rank, float cs, int splitk) {
  if (gated_off(bl)) return;
  __shared__ f32x4 others[ROWWG ? 3 : 1][2][64];
  const BlockPtrs& pa = bl.z[0];
  const BlockPtrs& pc = bl.z[1];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t i = ROWWG ? (int64_t)blockIdx.x : (int64_t)blockIdx.x * 4 + wave;
  if (i >= b) return;                                   // ROWWG: the whole workgroup
  const int64_t lab = (int64_t)rank * b + i;
  const float beta_a = pa.beta[i], gd_a = pa.gdiag[i], beta_c = pc.beta[i], gd_c = pc.gdiag[i];
  float dot_a = 0.f, dot_c = 0.f;
  for (int64_t kc = 0; kc < d; kc += 256) {
    const int64_t k = kc + lane * 4;
    const bool on = k < d;
    f32x4 ua = {0.f, 0.f, 0.f, 0.f}, uc = {0.f, 0.f, 0.f, 0.f};
    if (on) {
      ua = sum_slices(pa.part, bp, i, d, k, ROWWG ? wave : 0, ROWWG ? 4 : 1, splitk);
      uc = sum_slices(pc.part, bp, i, d, k, ROWWG ? wave : 0, ROWWG ? 4 : 1, splitk);
    }
    if (ROWWG) {
      if (wave > 0) { others[wave - 1][0][lane] = ua; others[wave - 1][1][lane] = uc; }
      __syncthreads();
      if (wave == 0)
#pragma unroll
        for (int w = 0; w < 3; ++w) { ua += others[w][0][lane]; uc += others[w][1][lane]; }
      __syncthreads();                                  // read before the next piece overwrites it
      if (wave > 0) continue;
    }
    if (!on) continue;
    const u32x2 iw = *reinterpret_cast<const u32x2*>(pa.X + i * d + k);        // I[lab]
    const u32x2 tw = *reinterpret_cast<const u32x2*>(pc.X + i * d + k);        // T[lab]
    const float iv[4] = {bf16_lo(iw[0]), bf16_hi(iw[0]), bf16_lo(iw[1]), bf16_hi(iw[1])};
    const float tv[4] = {bf16_lo(tw[0]), bf16_hi(tw[0]), bf16_lo(tw[1]), bf16_hi(tw[1])};
    f32x4 gi = *reinterpret_cast<f32x4*>(pa.gq + lab * d + k);
    f32x4 gt = *reinterpret_cast<f32x4*>(pc.gq + lab * d + k);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float ga = fmaf(beta_a, ua[e], gd_a * tv[e]);
      const float gc = fmaf(beta_c, uc[e], gd_c * iv[e]);
      gi[e] = fmaf(cs * gd_c, tv[e], fmaf(cs, ga, gi[e]));
      gt[e] = fmaf(cs * gd_a, iv[e], fmaf(cs, gc, gt[e]));
      dot_a = fmaf(ga, iv[e], dot_a);
      dot_c = fmaf(gc, tv[e], dot_c);
    }
    *reinterpret_cast<f32x4*>(pa.gq + lab * d + k) = gi;
    *reinterpret_cast<f32x4*>(pc.gq + lab * d + k) = gt;
  }
  if (ROWWG && wave > 0) return;
  dot_a = wave_sum(dot_a);
  dot_c = wave_sum(dot_c);
  if (lane == 0) { pa.rowds[i] = dot_a; pc.rowds[i] = dot_c; }
}

// shares up to this many rows finalize with one workgroup per row
constexpr int64_t FINALIZE_ROWWG_MAX = 1024;

// The same for the two-view loss (one block, X = Y = Z, gq = gk = gZ).  With g = rank b + i the row's own global row
// and lab its positive's row:
//   gZ[g]   += cs (beta_i sum_ks part + gdiag_i Z[lab])     query side
//   gZ[lab] += cs gdiag_i Z[g]                              label-column term of the key side
// The second line lands in another row, lab.  If lab belongs to this rank too, the wave that owns it adds the term
// (seen from there it reads gdiag_i' Z[lab'] with i' its positive, since the positive of the positive is the row
// itself); otherwise the wave of row i writes it.  Every row of gZ so has exactly one writer in this kernel.
// b: the real rows; bp: row pitch of the partial products.
__global__ __launch_bounds__(256) void k_query_finalize_ntxent(Blocks bl, int64_t b, int64_t bp, int64_t B, int64_t d, int rank, float cs, int splitk) {
  if (gated_off(bl)) return;
  const BlockPtrs& p = bl.z[0];
  const int lane = threadIdx.x & 63;
  const int64_t i = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (i >= b) return;
  const int64_t g = (int64_t)rank * b + i, lab = label_row(g, B, LOSS_NTXENT);
  const int64_t ip = lab - (int64_t)rank * b;                         // local index of the positive, if it is local
  const bool pos_local = ip >= 0 && ip < b;
  const float beta = p.beta[i], gd = p.gdiag[i], gd_pos = pos_local ? p.gdiag[ip] : 0.f;
  const uint16_t* Zfull = p.Y;
  float dot = 0.f;
  for (int64_t k = lane * 4; k < d; k += 256) {
    const f32x4 u = sum_slices(p.part, bp, i, d, k, 0, 1, splitk);
    const u32x2 zw = *reinterpret_cast<const u32x2*>(Zfull + g * d + k);        // Z[g]
    const u32x2 pw = *reinterpret_cast<const u32x2*>(Zfull + lab * d + k);      // Z[lab]
    const float zv[4] = {bf16_lo(zw[0]), bf16_hi(zw[0]), bf16_lo(zw[1]), bf16_hi(zw[1])};
    const float pv[4] = {bf16_lo(pw[0]), bf16_hi(pw[0]), bf16_lo(pw[1]), bf16_hi(pw[1])};
    f32x4 own = *reinterpret_cast<f32x4*>(p.gq + g * d + k);
    f32x4 oth = {0.f, 0.f, 0.f, 0.f};
    if (!pos_local) oth = *reinterpret_cast<f32x4*>(p.gq + lab * d + k);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float ga = fmaf(beta, u[e], gd * pv[e]);
      own[e] = fmaf(cs * gd_pos, pv[e], fmaf(cs, ga, own[e]));        // + what the local positive owes this row
      oth[e] = fmaf(cs * gd, zv[e], oth[e]);
      dot = fmaf(ga, zv[e], dot);
    }
    *reinterpret_cast<f32x4*>(p.gq + g * d + k) = own;
    if (!pos_local) *reinterpret_cast<f32x4*>(p.gq + lab * d + k) = oth;
  }
  dot = wave_sum(dot);
  if (lane == 0) p.rowds[i] = dot;
}

// loss_r = c sum ce, gs_r = c sum rowds over the blocks of the loss; one workgroup, fixed order.
__global__ __launch_bounds__(1024) void k_scalars(Blocks bl, int64_t b, float c, int accumulate, float* loss, float* gs) {
  if (gated_off(bl)) return;
  __shared__ float ra[16], rg[16];
  float a = 0.f, g = 0.f;
  for (int z = 0; z < bl.nblk; ++z)
    for (int64_t i0 = threadIdx.x; i0 < b; i0 += 4096) {              // four loads of each array in flight
      float c[4], r[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int64_t i = i0 + u * 1024;
        c[u] = i < b ? bl.z[z].ce[i] : 0.f;
        r[u] = i < b ? bl.z[z].rowds[i] : 0.f;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) { a += c[u]; g += r[u]; }
    }
  a = wave_sum(a);
  g = wave_sum(g);
  if ((threadIdx.x & 63) == 0) { ra[threadIdx.x >> 6] = a; rg[threadIdx.x >> 6] = g; }
  __syncthreads();
  if (threadIdx.x == 0) {
    float sa = 0.f, sg = 0.f;
    for (int w = 0; w < 16; ++w) { sa += ra[w]; sg += rg[w]; }
    *loss = (accumulate ? *loss : 0.f) + c * sa;
    *gs = (accumulate ? *gs : 0.f) + c * sg;
  }
}

// ------------------------------------------------------------------------------------------------
// Symmetric full loss (N = 1; Eq. 1 / Fig. 1: one B x B similarity matrix serves both directions, text -> image is
// its transpose).  z2_ij = s2 <I_i, T_j> is computed once and kept as ONE matrix of numerators against ONE reference r,
//   E_ij = exp2(z2_ij - r),      r = max(max_i z2_ii, s2 max|I_i| max|T_j| - headroom),
// whose row sums normalise image -> text (beta^A_i) and whose column sums normalise text -> image (beta^C_j).  A
// second pass turns it in place into the combined gradient matrix G_ij = E_ij (beta^A_i + beta^C_j) = P^A_ij + P^C_ji
// (bf16, label entries kept apart in fp32 as before), so that each feature gradient is one contraction:
//   gT = cs G^T I,   gI = cs G T     ->   2 + 4 = 6 B^2 d flop instead of 12.
// One reference for all rows and columns needs every row's and column's largest logit within about 60 (base 2)
// of r + 0; where a total falls under the floor, k_row_merge raises the flag at `gate`, the remaining kernels of
// this path return at once and the two-block path, launched behind them and gated the other way, does the call.

// r of the comment above, and the hand-over flag cleared.  One workgroup.
__global__ __launch_bounds__(1024) void k_sym_ref(const float* zd2, int64_t B, const float* wgmax, float s2, float* rglobal, int* gate) {
  __shared__ float red[16], nrm[2][16];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float m = -INFINITY;
  for (int64_t i = threadIdx.x; i < B; i += 1024) m = fmaxf(m, zd2[i]);
  float n0 = wgmax[threadIdx.x % NORM_BLOCKS], n1 = wgmax[NORM_BLOCKS + threadIdx.x % NORM_BLOCKS];
  for (int o = 32; o > 0; o >>= 1) {
    m = fmaxf(m, __shfl_xor(m, o));
    n0 = fmaxf(n0, __shfl_xor(n0, o));
    n1 = fmaxf(n1, __shfl_xor(n1, o));
  }
  if (lane == 0) { red[wave] = m; nrm[0][wave] = n0; nrm[1][wave] = n1; }
  __syncthreads();
  if (threadIdx.x == 0) {
    float a = red[0], x = nrm[0][0], y = nrm[1][0];
    for (int w = 1; w < 16; ++w) { a = fmaxf(a, red[w]); x = fmaxf(x, nrm[0][w]); y = fmaxf(y, nrm[1][w]); }
    *rglobal = row_reference(a, sqrtf(x), sqrtf(y), s2);
    *gate = 0;
  }
}

// Logit tiles of the symmetric path: k_logit_tiles for one block (X = I on the tile's N side, Y = T on its M side)
// with the one reference; the row sums come from the accumulators as there, the column sums (over the tile's
// query rows) from a copy of the bf16 tile that the epilogue leaves in LDS: a thread adds up its 8 columns over its
// 16 rows, lanes l and l + 32 join, the eight waves leave their sums in ring unit 4 and, after a barrier, 256
// threads add the eight.  (So the text -> image normalisation is that of the stored, rounded numerators.)
// bl.z[0]: E, row partial sums, label numerators; bl.z[1].lpart: column partial sums, one per query tile, cpart[it][j].
// B: the batch rounded up to whole tiles.  RAGGED: the batch is not whole tiles (X and Y are zero-padded copies): the
// last key tiles leave their padding columns out (so every row sum is right) and the column sums leave the padding
// rows out; what the padding rows hold in E meets zero feature rows in both contractions.
template <bool RAGGED>
__global__ __launch_bounds__(NTHREADS) void k_sym_logit(Blocks bl, int64_t B, int64_t d, float s2, const float* rglobal, int sbi, int sbj) {
  if (gated_off(bl)) return;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const BlockPtrs& p = bl.z[0];
  const int nI = (int)(B / BN), nJ = (int)(B / BM);
  const int total = nI * nJ;
  const int chunk = (total + 7) >> 3, padded = chunk << 3;
  const float ref = *rglobal;
  const float ref2[2] = {ref, ref};
  float* colpart = reinterpret_cast<float*>(smem + E_TILE_BYTES);       // [8 waves][256 keys]
  for (int u = blockIdx.x; u < padded; u += gridDim.x) {
    const int lin = (u & 7) * chunk + (u >> 3);
    if ((u >> 3) >= chunk || lin >= total) continue;
    int it, jt;
    superblock_tile(lin, nI, nJ, sbi, sbj, it, jt);
    const int64_t i0 = (int64_t)it * BN, j0 = (int64_t)jt * BM;
    f32x16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    mainloop<FMT_K, FMT_K, true>(p.Y + j0 * d, d, p.X + i0 * d, d, (int)(d / BK), smem, acc);
    // the label of query row i is key row i: only the tiles on the diagonal contain label columns
    // (ordinary stores: the matrix is read again by the combining pass and the two contractions)
    if (it == jt || (RAGGED && j0 + BM > bl.keys))
      logit_epilogue<true, true, RAGGED ? MASK_EDGE : MASK_DIAG, false, true, false>(p, acc, smem, B, s2, i0, j0, 0, LOSS_CLIP, bl.keys, ref2, j0, B);
    else logit_epilogue<true, true, MASK_NONE, false, true, false>(p, acc, smem, B, s2, i0, j0, 0, LOSS_CLIP, bl.keys, ref2, j0, B);
    lds_barrier();
    const int t = threadIdx.x;
    const int chunk16 = t & 31, r0 = t >> 5;
    float cs[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll 8
    for (int r = 0; r < 16; ++r) {
      const int row = r * 16 + r0;
      const u32x4 raw = *reinterpret_cast<const u32x4*>(smem + row * E_ROW_BYTES + ((chunk16 ^ ((row & 31) >> 1)) << 4));
      const u32x4 val = (row & 1) ? u32x4{raw[2], raw[3], raw[0], raw[1]} : raw;
      if (RAGGED && i0 + row >= bl.rows) continue;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        cs[2 * w] += bf16_lo(val[w]);
        cs[2 * w + 1] += bf16_hi(val[w]);
      }
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) cs[k] += __shfl_xor(cs[k], 32);
    if ((t & 63) < 32) {
      float* cp = colpart + (t >> 6) * 256 + chunk16 * 8;
      *reinterpret_cast<f32x4*>(cp) = f32x4{cs[0], cs[1], cs[2], cs[3]};
      *reinterpret_cast<f32x4*>(cp + 4) = f32x4{cs[4], cs[5], cs[6], cs[7]};
    }
    lds_barrier();
    if (t < BM) {
      float c = 0.f;
#pragma unroll
      for (int w = 0; w < 8; ++w) c += colpart[w * 256 + t];
      bl.z[1].lpart[(int64_t)it * B + j0 + t] = c;
    }
  }
}

// G_ij = E_ij (beta^A_i + beta^C_j) in place, bf16 (nearest even); the label entries stay 0.  A workgroup takes
// 64 x 64 blocks of the matrix (8 KiB contiguous, see e_index) one after the other; a thread 2 atoms of a block.
__global__ __launch_bounds__(256) void k_sym_combine(Blocks bl, int64_t B) {
  if (gated_off(bl)) return;
  const float* betaA = bl.z[0].beta;
  const float* betaC = bl.z[1].beta;
  uint16_t* E = bl.z[0].E;
  const int64_t nb = B >> 6, nblocks = nb * nb;
  const int t = threadIdx.x;
  for (int64_t blk = blockIdx.x; blk < nblocks; blk += gridDim.x) {
    const int64_t ib = blk / nb, jb = blk % nb;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int c = h * 256 + t;                          // atom of the block: key piece c >> 6, row c & 63
      const int row = c & 63, col = (c >> 6) * 8;
      u32x4* ptr = reinterpret_cast<u32x4*>(E + blk * 4096 + c * 8);
      const u32x4 raw = *ptr;
      const float ba = betaA[ib * 64 + row];
      const bool padding = ib * 64 + row >= bl.rows;      // a padding row of a ragged batch: exact zeros, whatever it holds
      const f32x4 bc0 = *reinterpret_cast<const f32x4*>(betaC + jb * 64 + col);
      const f32x4 bc1 = *reinterpret_cast<const f32x4*>(betaC + jb * 64 + col + 4);
      const float bc[8] = {bc0[0], bc0[1], bc0[2], bc0[3], bc1[0], bc1[1], bc1[2], bc1[3]};
      u32x4 out;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const __bf16 lo = (__bf16)(bf16_lo(raw[w]) * (ba + bc[2 * w]));
        const __bf16 hi = (__bf16)(bf16_hi(raw[w]) * (ba + bc[2 * w + 1]));
        out[w] = padding ? 0u : (uint32_t)__builtin_bit_cast(uint16_t, lo) | ((uint32_t)__builtin_bit_cast(uint16_t, hi) << 16);
      }
      *ptr = out;
    }
  }
}

// Row i of both gradients, for the symmetric path (every row is an own row): with u = sum_ks part[ks][i] = (G T)_i
// without the label entry and gd = (P^A_ii - 1) + (P^C_ii - 1),
//   gI[i] (+)= cs (u + gd T[i])      gT[i] += cs gd I[i]   (the key-side contraction has written or added its part)
// and the row's share of d/ds, <u + gd T[i], I[i]> (sum_ij G_ij S_ij = <G T, I> with the label entries included).
// B: the rows that exist; Bp: row pitch of the partial products.
__global__ __launch_bounds__(256) void k_sym_finalize(Blocks bl, int64_t B, int64_t Bp, int64_t d, float cs, int splitk, int accumulate) {
  if (gated_off(bl)) return;
  const BlockPtrs& p = bl.z[0];
  const int lane = threadIdx.x & 63;
  const int64_t i = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (i >= B) return;
  const float gd = p.gdiag[i] + bl.z[1].gdiag[i];
  float dot = 0.f;
  for (int64_t k = lane * 4; k < d; k += 256) {
    const f32x4 u = sum_slices(p.part, Bp, i, d, k, 0, 1, splitk);
    const u32x2 iw = *reinterpret_cast<const u32x2*>(p.X + i * d + k);
    const u32x2 tw = *reinterpret_cast<const u32x2*>(p.Y + i * d + k);
    const float iv[4] = {bf16_lo(iw[0]), bf16_hi(iw[0]), bf16_lo(iw[1]), bf16_hi(iw[1])};
    const float tv[4] = {bf16_lo(tw[0]), bf16_hi(tw[0]), bf16_lo(tw[1]), bf16_hi(tw[1])};
    f32x4 gi = {0.f, 0.f, 0.f, 0.f};
    if (accumulate) gi = *reinterpret_cast<const f32x4*>(p.gq + i * d + k);
    f32x4 gt = *reinterpret_cast<const f32x4*>(p.gk + i * d + k);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float ga = fmaf(gd, tv[e], u[e]);
      gi[e] = fmaf(cs, ga, gi[e]);
      gt[e] = fmaf(cs * gd, iv[e], gt[e]);
      dot = fmaf(ga, iv[e], dot);
    }
    *reinterpret_cast<f32x4*>(p.gq + i * d + k) = gi;
    *reinterpret_cast<f32x4*>(p.gk + i * d + k) = gt;
  }
  dot = wave_sum(dot);
  if (lane == 0) { p.rowds[i] = dot; bl.z[1].rowds[i] = 0.f; }
}

constexpr int NROWARRAYS = 7;

struct Plan {
  int64_t b, B, d;       // b and B rounded up to whole 256-row tiles: what the tile kernels and the layout below see
  int64_t b_real, B_real;
  bool ragged;           // b or B was rounded up: the kernels read zero-padded copies of the operands (off_pad)
  int64_t W;             // key panel width (B for the materialized path)
  int npanels;
  int nparts;            // B / 128
  int nMq, nN, splitk, ktps;
  size_t off_E, off_lpart, off_rows, off_Xs, off_part, off_ymax, off_flags, off_ref, off_pad, total;
  size_t rows_stride;    // bytes of one b-float row array (aligned)
};

// Key panels of the fused path: at most 16384 keys wide (so that one panel of both blocks' numerators
// stays within the 256 MiB last-level cache at the paper's rank shares) and at least two of them.
int fused_panels(int64_t B) {
  for (int n = 2; n <= 4096; ++n)
    if (B % ((int64_t)n * BM) == 0 && B / n <= 16384) return n;
  return 1;
}

Plan make_plan(int64_t B, int64_t d, int32_t N, bool fused, int nblk = 2) {
  Plan pl;
  pl.B_real = B; pl.b_real = B / N; pl.d = d;
  pl.b = (pl.b_real + BN - 1) / BN * BN;
  pl.B = (B + BM - 1) / BM * BM;
  pl.ragged = pl.b != pl.b_real || pl.B != pl.B_real;
  B = pl.B;
  const int64_t b = pl.b;
  pl.npanels = fused ? fused_panels(B) : 1;
  pl.W = B / pl.npanels;
  pl.nparts = (int)(B / 128);
  pl.nMq = (int)(b / BM);
  pl.nN = (int)((d + BN - 1) / BN);
  const int tiles = pl.nMq * pl.nN;
  const int kt_total = (int)(pl.W / BK);
  // Split of the query-side reduction: the 2 * tiles * sk workgroups run in rounds of one per compute unit (256 on
  // this chip), each taking kt_total / sk K-steps of about 1.1 us, and the sk partial tiles are written once and
  // read once at about 4 TB/s.  Take the sk with the least estimated time.
  int sk = 1;
  double best = 1e300;
  for (int c = 1; c <= 32 && c <= kt_total; ++c) {
    const int ktps = (kt_total + c - 1) / c;
    const int eff = (kt_total + ktps - 1) / ktps;                    // splits that are not empty
    const int rounds = (nblk * tiles * eff + 255) / 256;
    const double cost = rounds * ktps * 1.1 + eff * (2.0 * b * d * 4.0 * 2.0) / 4e6;
    if (cost < best) { best = cost; sk = c; }
  }
  pl.ktps = (kt_total + sk - 1) / sk;
  pl.splitk = (kt_total + pl.ktps - 1) / pl.ktps;
  size_t o = 0;
  pl.off_E = o;      o += 2 * align_up((size_t)b * pl.W * 2);
  pl.off_lpart = o;  o += 2 * align_up((size_t)pl.nparts * b * 4);
  pl.rows_stride = align_up((size_t)b * 4);
  pl.off_rows = o;   o += 2 * NROWARRAYS * pl.rows_stride;   // ediag, zd2, xnorm, beta, gdiag, ce, rowds
  pl.off_Xs = o;     o += 2 * align_up((size_t)d * b * 2);
  pl.off_part = o;   o += 2 * align_up((size_t)pl.splitk * b * d * 4);
  pl.off_ymax = o;   o += align_up((size_t)2 * NORM_BLOCKS * 4);         // partial maxima of the row norms
  pl.off_flags = o;  o += 2 * align_up((size_t)(b / BN) * 4);            // repair flags, one per query tile
  pl.off_ref = o;    o += 2 * pl.rows_stride;                            // exponent references of the rows
  pl.off_pad = o;                                                        // padded I, T, I_r, T_r of a ragged share
  if (pl.ragged) o += 2 * align_up((size_t)B * d * 2) + 2 * align_up((size_t)b * d * 2);
  pl.total = o;
  return pl;
}

// Query tiles per super-block of the logit tile walk (superblock_tile): the largest power of two <= 8 that divides
// the query tiles where that is at least 4 (or all of them), else up to 8 with a partial last super-block.
int superblock_width(int nI) {
  int sbi = 8;
  while (nI % sbi) sbi >>= 1;
  if (sbi < 4 && sbi < nI) sbi = nI < 8 ? nI : 8;
  return sbi;
}

// Compute units of the current device rounded down to a multiple of 8 (one persistent workgroup each).
int compute_units() {
  int dev = 0, n = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 8) n = 256;
  return n / 8 * 8;
}

template <class K>
bool allow_lds(K kernel, int bytes) {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, bytes) == hipSuccess;
}

// gate / gate_value: see Blocks.  marks: record the benchmark's stage events.
int mfma_run(const Problem& pr, bool fused, const int* gate = nullptr, int gate_value = 0, bool marks = true) {
  // the tile kernels use more LDS than the default limit; raised once per process (one device per process here)
  static const bool lds_ok = allow_lds(k_logit_tiles<true, true>, LOGIT_SMEM_BYTES) && allow_lds(k_logit_tiles<true, false>, LOGIT_SMEM_BYTES) &&
                             allow_lds(k_logit_tiles<false, true>, LOGIT_SMEM_BYTES) && allow_lds(k_logit_tiles<true, true, true>, LOGIT_SMEM_BYTES) &&
                             allow_lds(k_logit_tiles<true, false, true>, LOGIT_SMEM_BYTES) && allow_lds(k_logit_tiles<false, true, true>, LOGIT_SMEM_BYTES) &&
                             allow_lds(k_logit_repair<false>, LOGIT_SMEM_BYTES) &&
                             allow_lds(k_logit_repair<true>, LOGIT_SMEM_BYTES) && allow_lds(k_key_grad<false>, GEMM_SMEM_BYTES) &&
                             allow_lds(k_key_grad<true>, GEMM_SMEM_BYTES) && allow_lds(k_query_partial<false>, GEMM_SMEM_BYTES) &&
                             allow_lds(k_query_partial<true>, GEMM_SMEM_BYTES);
  if (!lds_ok) return DISCO_ERR_HIP;
  const int nblk = loss_blocks(pr.variant);
  const Plan pl = make_plan(pr.B, pr.d, pr.N, fused, nblk);
  const int persistent_wgs = compute_units();
  const int64_t b = pl.b, B = pl.B, d = pl.d, W = pl.W;     // whole tiles; the real sizes are pl.b_real, pl.B_real
  char* ws = static_cast<char*>(pr.ws);
  const uint16_t* I = static_cast<const uint16_t*>(pr.I);
  const uint16_t* T = static_cast<const uint16_t*>(pr.T);
  float* wgmax = reinterpret_cast<float*>(ws + pl.off_ymax);   // NORM_BLOCKS partial maxima of |I_j|^2, then of |T_j|^2

  uint16_t* Ipad = reinterpret_cast<uint16_t*>(ws + pl.off_pad);
  uint16_t* Tpad = reinterpret_cast<uint16_t*>(ws + pl.off_pad + align_up((size_t)B * d * 2));
  uint16_t* XIpad = reinterpret_cast<uint16_t*>(ws + pl.off_pad + 2 * align_up((size_t)B * d * 2));
  uint16_t* XTpad = reinterpret_cast<uint16_t*>(ws + pl.off_pad + 2 * align_up((size_t)B * d * 2) + align_up((size_t)b * d * 2));

  Blocks bl;
  bl.variant = pr.variant;
  bl.nblk = nblk;
  bl.rows = pl.b_real;
  bl.keys = pl.B_real;
  bl.gate = gate;
  bl.gate_value = gate_value;
  for (int z = 0; z < 2; ++z) {
    BlockPtrs& p = bl.z[z];
    const uint16_t* Xfull = z == 0 ? I : T;
    p.X = pl.ragged ? (z == 0 ? XIpad : XTpad) : Xfull + (size_t)pr.rank * b * d;
    p.Y = pl.ragged ? (z == 0 ? Tpad : Ipad) : (z == 0 ? T : I);
    p.E = reinterpret_cast<uint16_t*>(ws + pl.off_E + z * align_up((size_t)b * W * 2));
    p.lpart = reinterpret_cast<float*>(ws + pl.off_lpart + z * align_up((size_t)pl.nparts * b * 4));
    char* rows = ws + pl.off_rows + (size_t)z * NROWARRAYS * pl.rows_stride;
    p.ediag = reinterpret_cast<float*>(rows + 0 * pl.rows_stride);
    p.zd2 = reinterpret_cast<float*>(rows + 1 * pl.rows_stride);
    p.xnorm = reinterpret_cast<float*>(rows + 2 * pl.rows_stride);
    p.beta = reinterpret_cast<float*>(rows + 3 * pl.rows_stride);
    p.gdiag = reinterpret_cast<float*>(rows + 4 * pl.rows_stride);
    p.ce = reinterpret_cast<float*>(rows + 5 * pl.rows_stride);
    p.rowds = reinterpret_cast<float*>(rows + 6 * pl.rows_stride);
    p.ref2 = reinterpret_cast<float*>(ws + pl.off_ref + (size_t)z * pl.rows_stride);
    p.tileflag = reinterpret_cast<int*>(ws + pl.off_flags + z * align_up((size_t)(b / BN) * 4));
    p.ymax_parts = wgmax + (z == 0 ? NORM_BLOCKS : 0);     // block A's keys are T, block C's are I
    p.Xs = reinterpret_cast<uint16_t*>(ws + pl.off_Xs + z * align_up((size_t)d * b * 2));
    p.part = reinterpret_cast<float*>(ws + pl.off_part + z * align_up((size_t)pl.splitk * b * d * 4));
    p.gq = z == 0 ? pr.gI : pr.gT;
    p.gk = z == 0 ? pr.gT : pr.gI;
  }

  const float s2 = pr.s * LOG2E;
  const float c = loss_norm(pl.B_real, pr.variant);
  const float cs = c * pr.s;
  hipStream_t st = pr.stream;
  const int nI = (int)(b / BN);
  // super-block shape of the logit tile walk: sbi query tiles, then as many key tiles as keep it within 32 tiles
  const int sbi = superblock_width(nI);
  auto logit_grid = [&](int64_t keys, int& sbj) {
    const int nJ = (int)(keys / BM);
    sbj = 32 / sbi < nJ ? 32 / sbi : nJ;
    const int tiles2 = nblk * ((nI * nJ + 7) / 8 * 8);  // every block, each padded to a multiple of 8
    return dim3((unsigned)(tiles2 < persistent_wgs ? tiles2 : persistent_wgs));
  };
  const int nMk = (int)(W / BM);
  const dim3 key_grid((unsigned)(((nMk * pl.nN + 7) / 8) * 8), (unsigned)nblk);
  // k_query_partial's grid: see its slice -> XCD mapping
  const int qT = pl.nMq * pl.nN, qS = nblk * pl.splitk;
  const int q_wgs = qS % 8 == 0 ? 8 * qT * (qS / 8) : 8 % qS == 0 ? 8 * ((qT + 8 / qS - 1) / (8 / qS)) : (qS * qT + 7) / 8 * 8;
  const dim3 q_grid((unsigned)q_wgs);
  const int64_t g0 = (int64_t)pr.rank * pl.b_real;       // global row of the rank's first row
  int stage = 0;

  if (marks) stage_mark(st, stage++);
  if (pl.ragged)
    k_pad_operands<<<dim3((unsigned)(8 * persistent_wgs)), 256, 0, st>>>(I, T, pl.B_real, B, pl.b_real, b, d, pr.rank, Ipad, Tpad, XIpad, XTpad);
  k_prep<<<dim3((unsigned)(2 * NORM_BLOCKS + nblk * ((b + 3) / 4))), 256, 0, st>>>(bl, I, T, pl.B_real, pl.b_real, b, d, pr.rank, s2, wgmax);
  if (marks) stage_mark(st, stage++);

  int sbj;
  if (fused) {
    const dim3 g = logit_grid(B, sbj);
    if (pl.ragged) k_logit_tiles<true, false, true><<<g, NTHREADS, LOGIT_SMEM_BYTES, st>>>(bl, b, pl.B_real, d, g0, s2, 0, B, sbi, sbj, nblk);
    else k_logit_tiles<true, false><<<g, NTHREADS, LOGIT_SMEM_BYTES, st>>>(bl, b, pl.B_real, d, g0, s2, 0, B, sbi, sbj, nblk);
  } else {
    const dim3 g = logit_grid(B, sbj);
    if (pl.ragged) k_logit_tiles<true, true, true><<<g, NTHREADS, LOGIT_SMEM_BYTES, st>>>(bl, b, pl.B_real, d, g0, s2, 0, B, sbi, sbj, nblk);
    else k_logit_tiles<true, true><<<g, NTHREADS, LOGIT_SMEM_BYTES, st>>>(bl, b, pl.B_real, d, g0, s2, 0, B, sbi, sbj, nblk);
  }
  if (marks) stage_mark(st, stage++);
  k_row_merge<<<dim3((unsigned)(b / 64), (unsigned)nblk), 1024, 0, st>>>(bl, b, pl.nparts, pl.nparts, s2, nullptr, nullptr, d);
  if (fused) k_logit_repair<false><<<dim3((unsigned)(nblk * nI)), NTHREADS, LOGIT_SMEM_BYTES, st>>>(bl, b, B, d, pr.rank, s2);
  else k_logit_repair<true><<<dim3((unsigned)(nblk * nI)), NTHREADS, LOGIT_SMEM_BYTES, st>>>(bl, b, B, d, pr.rank, s2);
  if (marks) stage_mark(st, stage++);

  for (int pnl = 0; pnl < pl.npanels; ++pnl) {
    const int64_t jp0 = (int64_t)pnl * W;
    if (fused) {
      const dim3 g = logit_grid(W, sbj);
      if (pl.ragged) k_logit_tiles<false, true, true><<<g, NTHREADS, LOGIT_SMEM_BYTES, st>>>(bl, b, pl.B_real, d, g0, s2, jp0, W, sbi, sbj, nblk);
      else k_logit_tiles<false, true><<<g, NTHREADS, LOGIT_SMEM_BYTES, st>>>(bl, b, pl.B_real, d, g0, s2, jp0, W, sbi, sbj, nblk);
    }
    if (pr.accumulate)
      k_key_grad<true><<<key_grid, NTHREADS, GEMM_SMEM_BYTES, st>>>(bl, b, d, cs, jp0, W, nMk, pl.nN);
    else
      k_key_grad<false><<<key_grid, NTHREADS, GEMM_SMEM_BYTES, st>>>(bl, b, d, cs, jp0, W, nMk, pl.nN);
    if (!fused) if (marks) stage_mark(st, stage++);
    if (pnl > 0)
      k_query_partial<true><<<q_grid, NTHREADS, GEMM_SMEM_BYTES, st>>>(bl, b, d, jp0, W, pl.nMq, pl.nN, pl.splitk, pl.ktps);
    else
      k_query_partial<false><<<q_grid, NTHREADS, GEMM_SMEM_BYTES, st>>>(bl, b, d, jp0, W, pl.nMq, pl.nN, pl.splitk, pl.ktps);
  }
  if (marks) stage_mark(st, stage++);
  if (pr.variant == LOSS_NTXENT) k_query_finalize_ntxent<<<dim3((unsigned)((pl.b_real + 3) / 4)), 256, 0, st>>>(bl, pl.b_real, b, pl.B_real, d, pr.rank, cs, pl.splitk);
  else if (pl.b_real <= FINALIZE_ROWWG_MAX) k_query_finalize<true><<<dim3((unsigned)pl.b_real), 256, 0, st>>>(bl, pl.b_real, b, d, pr.rank, cs, pl.splitk);
  else k_query_finalize<false><<<dim3((unsigned)((pl.b_real + 3) / 4)), 256, 0, st>>>(bl, pl.b_real, b, d, pr.rank, cs, pl.splitk);
  k_scalars<<<1, 1024, 0, st>>>(bl, pl.b_real, c, pr.accumulate, pr.loss, pr.gs);
  if (marks) stage_mark(st, stage++);
  return hipGetLastError() == hipSuccess ? DISCO_OK : DISCO_ERR_HIP;
}

// The symmetric full loss (see the kernels above): one matrix of numerators, both directions' statistics, one
// combined gradient matrix, two contractions; then, behind the flag, the two-block path for inputs it cannot take.
size_t sym_tail(int64_t B, int64_t d) {
  const size_t a = make_plan(B, d, 1, false, 1).total, c = make_plan(B, d, 1, false, 2).total;
  return a > c ? a : c;
}

int mfma_sym_run_impl(const Problem& pr) {
  static const bool lds_ok = allow_lds(k_sym_logit<false>, LOGIT_SMEM_BYTES) && allow_lds(k_sym_logit<true>, LOGIT_SMEM_BYTES);
  if (!lds_ok) return DISCO_ERR_HIP;
  const Plan pl = make_plan(pr.B, pr.d, 1, false, 1);
  const int persistent_wgs = compute_units();
  const int64_t B = pl.B, d = pl.d, Br = pl.B_real;        // whole tiles / the rows that exist
  char* ws = static_cast<char*>(pr.ws);
  const size_t tail = sym_tail(Br, d);
  int* gate = reinterpret_cast<int*>(ws + tail);
  float* rglobal = reinterpret_cast<float*>(ws + tail + 128);
  const uint16_t* I = static_cast<const uint16_t*>(pr.I);
  const uint16_t* T = static_cast<const uint16_t*>(pr.T);
  float* wgmax = reinterpret_cast<float*>(ws + pl.off_ymax);

  // a batch that is not whole tiles: zero-padded copies of I and T (the copies of "the rank's rows" are not used)
  uint16_t* Ipad = reinterpret_cast<uint16_t*>(ws + pl.off_pad);
  uint16_t* Tpad = reinterpret_cast<uint16_t*>(ws + pl.off_pad + align_up((size_t)B * d * 2));

  Blocks bl;
  bl.variant = LOSS_CLIP;
  bl.nblk = 1;
  bl.rows = Br;
  bl.keys = Br;
  bl.gate = nullptr;
  bl.gate_value = 0;
  BlockPtrs& p = bl.z[0];
  char* rows0 = ws + pl.off_rows;
  char* rows1 = rows0 + (size_t)NROWARRAYS * pl.rows_stride;
  p.X = pl.ragged ? Ipad : I;
  p.Y = pl.ragged ? Tpad : T;
  p.E = reinterpret_cast<uint16_t*>(ws + pl.off_E);
  p.lpart = reinterpret_cast<float*>(ws + pl.off_lpart);
  p.ediag = reinterpret_cast<float*>(rows0 + 0 * pl.rows_stride);
  p.zd2 = reinterpret_cast<float*>(rows0 + 1 * pl.rows_stride);
  p.xnorm = reinterpret_cast<float*>(rows0 + 2 * pl.rows_stride);
  p.beta = reinterpret_cast<float*>(rows0 + 3 * pl.rows_stride);
  p.gdiag = reinterpret_cast<float*>(rows0 + 4 * pl.rows_stride);
  p.ce = reinterpret_cast<float*>(rows0 + 5 * pl.rows_stride);
  p.rowds = reinterpret_cast<float*>(rows0 + 6 * pl.rows_stride);
  p.ref2 = reinterpret_cast<float*>(ws + pl.off_ref);
  p.tileflag = reinterpret_cast<int*>(ws + pl.off_flags);
  p.ymax_parts = wgmax + NORM_BLOCKS;
  p.Xs = reinterpret_cast<uint16_t*>(ws + pl.off_Xs);
  p.part = reinterpret_cast<float*>(ws + pl.off_part);
  p.gq = pr.gI;
  p.gk = pr.gT;
  // "block 1" holds the column side: partial column sums and the text -> image statistics; label numerators,
  // positive-pair logits and the reference are the row side's
  BlockPtrs& q = bl.z[1];
  q = p;
  q.lpart = reinterpret_cast<float*>(ws + pl.off_lpart + align_up((size_t)pl.nparts * B * 4));
  q.beta = reinterpret_cast<float*>(rows1 + 3 * pl.rows_stride);
  q.gdiag = reinterpret_cast<float*>(rows1 + 4 * pl.rows_stride);
  q.ce = reinterpret_cast<float*>(rows1 + 5 * pl.rows_stride);
  q.rowds = reinterpret_cast<float*>(rows1 + 6 * pl.rows_stride);
  q.ref2 = reinterpret_cast<float*>(ws + pl.off_ref + pl.rows_stride);
  q.tileflag = reinterpret_cast<int*>(ws + pl.off_flags + align_up((size_t)(B / BN) * 4));

  const float s2 = pr.s * LOG2E;
  const float c = loss_norm(Br, LOSS_CLIP);
  const float cs = c * pr.s;
  hipStream_t st = pr.stream;
  const int nT = (int)(B / BN);
  const int sbi = superblock_width(nT);
  const int sbj = 32 / sbi < nT ? 32 / sbi : nT;
  const int tiles = (nT * nT + 7) / 8 * 8;
  const dim3 logit_grid((unsigned)(tiles < persistent_wgs ? tiles : persistent_wgs));
  const dim3 key_grid((unsigned)(((nT * pl.nN + 7) / 8) * 8), 1);
  const int qT = pl.nMq * pl.nN, qS = pl.splitk;
  const int q_wgs = qS % 8 == 0 ? 8 * qT * (qS / 8) : 8 % qS == 0 ? 8 * ((qT + 8 / qS - 1) / (8 / qS)) : (qS * qT + 7) / 8 * 8;
  int stage = 0;

  stage_mark(st, stage++);
  if (pl.ragged) k_pad_operands<<<dim3((unsigned)(8 * persistent_wgs)), 256, 0, st>>>(I, T, Br, B, 0, 0, d, 0, Ipad, Tpad, Ipad, Tpad);
  k_prep<<<dim3((unsigned)(2 * NORM_BLOCKS + (B + 3) / 4)), 256, 0, st>>>(bl, I, T, Br, Br, B, d, 0, s2, wgmax);
  k_sym_ref<<<1, 1024, 0, st>>>(p.zd2, Br, wgmax, s2, rglobal, gate);
  stage_mark(st, stage++);
  if (pl.ragged) k_sym_logit<true><<<logit_grid, NTHREADS, LOGIT_SMEM_BYTES, st>>>(bl, B, d, s2, rglobal, sbi, sbj);
  else k_sym_logit<false><<<logit_grid, NTHREADS, LOGIT_SMEM_BYTES, st>>>(bl, B, d, s2, rglobal, sbi, sbj);
  stage_mark(st, stage++);
  Blocks both = bl;
  both.nblk = 2;
  k_row_merge<<<dim3((unsigned)((B + 63) / 64), 2), 1024, 0, st>>>(both, B, pl.nparts, nT, s2, rglobal, gate, 0);
  Blocks go = bl;                                   // from here on only while no total was lost
  go.gate = gate;
  go.gate_value = 0;
  k_transpose<<<dim3((unsigned)(B / 64)), 1024, 0, st>>>(go, B, d);
  stage_mark(st, stage++);
  k_sym_combine<<<dim3((unsigned)(8 * persistent_wgs)), 256, 0, st>>>(go, B);
  stage_mark(st, stage++);
  if (pr.accumulate) k_key_grad<true><<<key_grid, NTHREADS, GEMM_SMEM_BYTES, st>>>(go, B, d, cs, 0, B, nT, pl.nN);
  else k_key_grad<false><<<key_grid, NTHREADS, GEMM_SMEM_BYTES, st>>>(go, B, d, cs, 0, B, nT, pl.nN);
  stage_mark(st, stage++);
  k_query_partial<false><<<dim3((unsigned)q_wgs), NTHREADS, GEMM_SMEM_BYTES, st>>>(go, B, d, 0, B, pl.nMq, pl.nN, pl.splitk, pl.ktps);
  stage_mark(st, stage++);
  k_sym_finalize<<<dim3((unsigned)((Br + 3) / 4)), 256, 0, st>>>(go, Br, B, d, cs, pl.splitk, pr.accumulate);
  Blocks go2 = go;
  go2.nblk = 2;
  k_scalars<<<1, 1024, 0, st>>>(go2, Br, c, pr.accumulate, pr.loss, pr.gs);
  stage_mark(st, stage++);
  if (hipGetLastError() != hipSuccess) return DISCO_ERR_HIP;
  return mfma_run(pr, false, gate, 1, false);
}

}  // namespace

bool mfma_supported(int64_t B, int64_t d, int32_t N, int dtype, int variant) {
  if (dtype != DISCO_BF16) return false;
  if (N <= 0 || B % N != 0) return false;
  const int64_t b = B / N;
  if (variant == LOSS_NTXENT && B % 2 != 0) return false;                   // two views
  // per-lane load offsets are 32-bit byte offsets inside one operand tile: 256 rows of pitch b (Xs) or four block
  // rows of pitch 64 W (row groups of the stored numerators) must stay below 4 GiB
  if (B > ((int64_t)1 << 23) || b > ((int64_t)1 << 22)) return false;      // (rounding up to whole tiles stays within them)
  return d % 64 == 0;
}

bool mfma_whole_tiles(int64_t B, int32_t N) { return N > 0 && B % N == 0 && (B / N) % 256 == 0; }

size_t mfma_stored_workspace_bytes(int64_t B, int64_t d, int32_t N, int variant) { return make_plan(B, d, N, false, loss_blocks(variant)).total; }
size_t mfma_fused_workspace_bytes(int64_t B, int64_t d, int32_t N, int variant) { return make_plan(B, d, N, true, loss_blocks(variant)).total; }
int mfma_stored_run(const Problem& pr) { return mfma_run(pr, false); }
int mfma_fused_run(const Problem& pr) { return mfma_run(pr, true); }
size_t mfma_sym_workspace_bytes(int64_t B, int64_t d) { return sym_tail(B, d) + 256; }
int mfma_sym_run(const Problem& pr) { return mfma_sym_run_impl(pr); }

}  // namespace disco
