// Device-side building blocks of the bf16 MFMA path: the 256x256x32 NT tile main loop (8 waves = two
// per SIMD, each 128x64 = 4x2 MFMA 32x32x16 blocks, four LDS stages, swizzled 16-byte chunks), the
// operand tile loaders and the LDS-staged tile store.  Included by mfma_kernels.hip only.
//
// Why two waves per SIMD: a wave issues its instructions strictly one after the other, and an LDS write
// or a global load keeps it busy for tens of cycles, so a lone wave cannot hide them behind its own
// MFMAs (measured: their costs simply add up).  With a second wave on the SIMD the matrix pipe takes
// MFMAs from one wave while the other issues memory instructions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace disco {
namespace tile {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr int NTHREADS = 512;                     // 8 waves: 2 (M) x 4 (N), wave tile 128 x 64
constexpr int BM = 256, BN = 256, BK = 32;
constexpr int NSTAGE = 4;
constexpr int A_BYTES = BM * BK * 2;              // 16 KiB
constexpr int STAGE_BYTES = (BM + BN) * BK * 2;   // 32 KiB
constexpr int SMEM_BYTES = NSTAGE * STAGE_BYTES;  // 128 KiB of the CU's 160 KiB

// Byte offset of 16-byte chunk `chunk` (0..3) of tile row `row` (64-byte rows: 32 bf16 of the reduction
// index).  The LDS has 64 banks of 4 bytes, so four consecutive rows span all banks once.  Two
// permutations keep every access pattern below conflict-free:
//   * the chunk is XOR-ed with bits 2..3 of the row, so the 16 consecutive rows that a quarter-wave reads
//     for an MFMA operand (same chunk) hit 16 different 16-byte bank groups;
//   * the two low row bits are XOR-ed with bits 2..3 as well, so rows that are 4 apart (what neighbouring
//     lanes of the transposing loader write) fall into different quarters of the banks.
__device__ __forceinline__ uint32_t lds_off(int row, int chunk) {
  const int g = (row >> 2) & 3;
  return (uint32_t)(row ^ g) * 64u + (uint32_t)((chunk ^ g) << 4);
}

// Copies a 256 x 32 bf16 operand tile from global memory to LDS through registers (512 threads).
//   MODE 0: element (r, k) is at base[r * ld + k]   (reduction index contiguous): two 16-byte loads,
//           thread t owns chunk t % 4 of rows t/4 and t/4 + 128;
//   MODE 1: element (r, k) is at base[k * ld + r]   (row index contiguous): thread t loads a 4 (k) x 4 (r)
//           block with four 8-byte loads, transposes it in registers and writes four 8-byte row pieces.
template <int MODE>
struct TileLoader {
  u32x2 r[4];      // MODE 0: two 16-byte chunks as (r[0], r[1]) and (r[2], r[3]); MODE 1: four 8-byte rows
  uint32_t voff;   // this thread's byte offset inside the tile; everything else in an address is wave-uniform
  __device__ __forceinline__ void init(int64_t ld, int t) {
    if (MODE == 0) voff = (uint32_t)(((t >> 2) * ld + (t & 3) * 8) * 2);
    else voff = (uint32_t)(((t & 7) * 4 * ld + (t >> 3) * 4) * 2);
  }
  // base: wave-uniform pointer to element (row 0, k 0) of the tile's current K-step
  __device__ __forceinline__ void load(const uint16_t* base, int64_t ld) {
    if (MODE == 0) {
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const u32x4 v = *reinterpret_cast<const u32x4*>(reinterpret_cast<const char*>(base + (int64_t)(128 * i) * ld) + voff);
        r[2 * i][0] = v[0]; r[2 * i][1] = v[1]; r[2 * i + 1][0] = v[2]; r[2 * i + 1][1] = v[3];
      }
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        r[e] = *reinterpret_cast<const u32x2*>(reinterpret_cast<const char*>(base + (int64_t)e * ld) + voff);
    }
  }
  __device__ __forceinline__ void store(char* lds, int t) const {
    if (MODE == 0) {
      const int kb = t & 3, rb = t >> 2;
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        u32x4 v;
        v[0] = r[2 * i][0]; v[1] = r[2 * i][1]; v[2] = r[2 * i + 1][0]; v[3] = r[2 * i + 1][1];
        *reinterpret_cast<u32x4*>(lds + lds_off(rb + 128 * i, kb)) = v;
      }
    } else {
      // r[e] = (rows 0,1 | rows 2,3) of reduction index 4 kq + e.  Output row u needs reduction indices
      // (0,1) in its first dword and (2,3) in its second: low halves for even u, high halves for odd u.
      const int kq = t & 7, rq = t >> 3;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const uint32_t sel = (u & 1) ? 0x07060302u : 0x05040100u;
        u32x2 o;
        o[0] = __builtin_amdgcn_perm(r[1][u >> 1], r[0][u >> 1], sel);
        o[1] = __builtin_amdgcn_perm(r[3][u >> 1], r[2][u >> 1], sel);
        *reinterpret_cast<u32x2*>(lds + lds_off(rq * 4 + u, kq >> 1) + (kq & 1) * 8) = o;
      }
    }
  }
};

// acc[bm][bn] += A_tile(256 x K) * B_tile(256 x K)^T for this wave's 128 x 64 piece.
// A, Bp point at element (row 0, k 0) of the tile; ktiles = K / 32, which must be even and positive.
//
// Software pipeline.  Four LDS stages of one 32-wide K-step each and two register sets:
//   step kt, sub-step 0: MFMAs on the first 16 of the reduction index; fetch the fragments of sub-step 1;
//                        issue the global loads of K-step kt+3 into the register set that is free;
//   barrier (LDS traffic only, never the global loads);
//   step kt, sub-step 1: MFMAs; fetch the first fragments of step kt+1 from its stage; write the other
//                        register set (K-step kt+2, loaded during step kt-1) into stage (kt+2) % 4.
// A global load has one and a half steps to land; an LDS stage is complete a full step before it is read
// and is not overwritten until two barriers after its last reader.  Loads past the end are clamped to
// the last K-step (redundant, never out of range).
#define DISCO_SGB(mask, n) __builtin_amdgcn_sched_group_barrier(mask, n, 0)
constexpr int SG_MFMA = 0x008, SG_VMEM_RD = 0x020, SG_DS_RD = 0x100, SG_DS_WR = 0x200;

__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

template <int MA, int MB>
__device__ __forceinline__ void mainloop(const uint16_t* __restrict__ A, int64_t lda, const uint16_t* __restrict__ Bp,
                                         int64_t ldb, int ktiles, char* smem, f32x16 (&acc)[4][2]) {
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int64_t stepA = MA == 0 ? BK : (int64_t)BK * lda;
  const int64_t stepB = MB == 0 ? BK : (int64_t)BK * ldb;
  const int last = ktiles - 1;
  const int arow = (wave >> 2) * 128 + (lane & 31), brow = (wave & 3) * 64 + (lane & 31), kc = lane >> 5;
  constexpr int NLD = (MA == 0 ? 2 : 4) + (MB == 0 ? 2 : 4);   // global loads / LDS writes per thread and K-step
  TileLoader<MA> la0, la1;
  TileLoader<MB> lb0, lb1;
  la0.init(lda, t); la1.init(lda, t); lb0.init(ldb, t); lb1.init(ldb, t);
  bf16x8 af0[4], bf0[2], af1[4], bf1[2];

  // prologue: K-steps 0 and 1 into stages 0 and 1, K-step 2 into register set 1
  la0.load(A, lda);
  lb0.load(Bp, ldb);
  {
    const int k1 = last < 1 ? last : 1;
    la1.load(A + k1 * stepA, lda);
    lb1.load(Bp + k1 * stepB, ldb);
  }
  la0.store(smem, t);
  lb0.store(smem + A_BYTES, t);
  la1.store(smem + STAGE_BYTES, t);
  lb1.store(smem + STAGE_BYTES + A_BYTES, t);
  {
    const int k2 = last < 2 ? last : 2;
    la1.load(A + k2 * stepA, lda);
    lb1.load(Bp + k2 * stepB, ldb);
  }
  lds_barrier();
#pragma unroll
  for (int i = 0; i < 4; ++i) af0[i] = *reinterpret_cast<const bf16x8*>(smem + lds_off(arow + 32 * i, kc));
#pragma unroll
  for (int i = 0; i < 2; ++i) bf0[i] = *reinterpret_cast<const bf16x8*>(smem + A_BYTES + lds_off(brow + 32 * i, kc));

  // one K-step: loads go into (la_new, lb_new), LDS writes come from (la_old, lb_old)
  auto step = [&](int kt, TileLoader<MA>& la_new, TileLoader<MB>& lb_new, const TileLoader<MA>& la_old,
                  const TileLoader<MB>& lb_old) __attribute__((always_inline)) {
    const char* cur = smem + (kt & 3) * STAGE_BYTES;
    const char* nxt = smem + ((kt + 1) & 3) * STAGE_BYTES;
    char* wr = smem + ((kt + 2) & 3) * STAGE_BYTES;
    const int kload = kt + 3 < ktiles ? kt + 3 : last;
    // sub-step 0
#pragma unroll
    for (int i = 0; i < 4; ++i) af1[i] = *reinterpret_cast<const bf16x8*>(cur + lds_off(arow + 32 * i, 2 + kc));
#pragma unroll
    for (int i = 0; i < 2; ++i) bf1[i] = *reinterpret_cast<const bf16x8*>(cur + A_BYTES + lds_off(brow + 32 * i, 2 + kc));
    la_new.load(A + kload * stepA, lda);
    lb_new.load(Bp + kload * stepB, ldb);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af0[i], bf0[j], acc[i][j], 0, 0, 0);
#pragma unroll
    for (int g = 0; g < 3; ++g) { DISCO_SGB(SG_DS_RD, 2); DISCO_SGB(SG_MFMA, 1); }
    DISCO_SGB(SG_VMEM_RD, NLD / 2); DISCO_SGB(SG_MFMA, 2);
    DISCO_SGB(SG_VMEM_RD, NLD - NLD / 2); DISCO_SGB(SG_MFMA, 3);
    __builtin_amdgcn_sched_barrier(0);   // nothing moves between sub-steps
    // sub-step 1
    lds_barrier();
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < 4; ++i) af0[i] = *reinterpret_cast<const bf16x8*>(nxt + lds_off(arow + 32 * i, kc));
#pragma unroll
    for (int i = 0; i < 2; ++i) bf0[i] = *reinterpret_cast<const bf16x8*>(nxt + A_BYTES + lds_off(brow + 32 * i, kc));
    la_old.store(wr, t);
    lb_old.store(wr + A_BYTES, t);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af1[i], bf1[j], acc[i][j], 0, 0, 0);
#pragma unroll
    for (int g = 0; g < 3; ++g) { DISCO_SGB(SG_DS_RD, 2); DISCO_SGB(SG_MFMA, 1); }
    DISCO_SGB(SG_DS_WR, NLD / 2); DISCO_SGB(SG_MFMA, 2);
    DISCO_SGB(SG_DS_WR, NLD - NLD / 2); DISCO_SGB(SG_MFMA, 3);
    __builtin_amdgcn_sched_barrier(0);
  };

  // ktiles is even (callers guarantee K % 64 == 0): the two register sets alternate without a branch
  for (int kt = 0; kt < ktiles; kt += 2) {
    step(kt, la0, lb0, la1, lb1);
    step(kt + 1, la1, lb1, la0, lb0);
  }
}

// Writes a workgroup's 256 x 256 fp32 accumulator tile to row-major global memory through LDS, so that
// every global store is a full 1 KiB row segment (the accumulator layout would give 4-byte elements per
// lane).  Two passes of 128 rows; LDS rows padded to 1056 bytes so that the two half-waves of a 4-byte
// write land on different banks.  out points at the tile's first element; value = scale * acc (+ old).
constexpr int OUT_ROW_BYTES = BN * 4 + 32;
constexpr int OUT_SMEM_BYTES = 128 * OUT_ROW_BYTES;       // 132 KiB
typedef __attribute__((ext_vector_type(4))) float f32x4;

template <bool ACCUMULATE>
__device__ __forceinline__ void store_tile_f32(f32x16 (&acc)[4][2], char* smem, float* out, int64_t ld, float scale) {
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = wave >> 2, wn = wave & 3, half = lane >> 5;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    lds_barrier();
    if (wm == h) {
#pragma unroll
      for (int bn = 0; bn < 2; ++bn)
#pragma unroll
        for (int bm = 0; bm < 4; ++bm)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int row = bm * 32 + (e >> 2) * 8 + half * 4 + (e & 3);
            const int col = wn * 64 + bn * 32 + (lane & 31);
            *reinterpret_cast<float*>(smem + row * OUT_ROW_BYTES + col * 4) = scale * acc[bm][bn][e];
          }
    }
    lds_barrier();
    const int chunk = t & 63, r0 = t >> 6;
#pragma unroll 4
    for (int r = 0; r < 16; ++r) {
      const int row = r * 8 + r0;
      f32x4 v = *reinterpret_cast<const f32x4*>(smem + row * OUT_ROW_BYTES + chunk * 16);
      float* g = out + (int64_t)(h * 128 + row) * ld + chunk * 4;
      if (ACCUMULATE) v += *reinterpret_cast<const f32x4*>(g);
      *reinterpret_cast<f32x4*>(g) = v;
    }
  }
}

}  // namespace tile
}  // namespace disco
