// Device-side building blocks of the bf16 MFMA path: the 256x256x64 NT tile main loop
// (4 waves, each 128x128 = 4x4 MFMA 32x32x16 blocks, LDS double buffered, XOR-swizzled 16-byte
// chunks) and the operand tile loaders.  Included by mfma_kernels.hip only.
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

constexpr int BM = 256, BN = 256, BK = 32;
constexpr int NSTAGE = 4;
constexpr int A_BYTES = BM * BK * 2;              // 16 KiB
constexpr int STAGE_BYTES = (BM + BN) * BK * 2;   // 32 KiB
constexpr int SMEM_BYTES = NSTAGE * STAGE_BYTES;  // 128 KiB of the CU's 160 KiB

// Byte offset of 16-byte chunk `chunk` (0..3) of tile row `row` (64-byte rows: 32 bf16 of the reduction
// index).  The LDS has 64 banks of 4 bytes, so four consecutive rows span all banks once; XOR-ing the
// chunk with bits 2..3 of the row makes the 16 rows that a quarter-wave reads for an MFMA operand (same
// chunk, consecutive rows) hit 16 different 16-byte bank groups.
__device__ __forceinline__ uint32_t lds_off(int row, int chunk) {
  return (uint32_t)row * 64u + (uint32_t)((chunk ^ ((row >> 2) & 3)) << 4);
}

// Copies a 256 x 32 bf16 operand tile from global memory to LDS through registers.
//   MODE 0: element (r, k) is at base[r * ld + k]   (reduction index contiguous): 16-byte loads, thread t
//           owns chunk t % 4 of rows t/4 + 64 i;
//   MODE 1: element (r, k) is at base[k * ld + r]   (row index contiguous): thread t loads an 8 (k) x 4 (r)
//           block with 8-byte loads, transposes it in registers and writes 4 rows of 16 bytes.
template <int MODE>
struct TileLoader {
  u32x4 r[4];
  uint32_t voff;   // this thread's byte offset inside the tile; everything else in an address is wave-uniform
  __device__ __forceinline__ void init(int64_t ld, int t) {
    const int kb = t & 3, rb = t >> 2;
    voff = MODE == 0 ? (uint32_t)((rb * ld + kb * 8) * 2) : (uint32_t)((kb * 8 * ld + rb * 4) * 2);
  }
  // base: wave-uniform pointer to element (row 0, k 0) of the tile's current K-step
  __device__ __forceinline__ void load(const uint16_t* base, int64_t ld) {
    if (MODE == 0) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
        r[i] = *reinterpret_cast<const u32x4*>(reinterpret_cast<const char*>(base + (int64_t)(64 * i) * ld) + voff);
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const u32x2 v = *reinterpret_cast<const u32x2*>(reinterpret_cast<const char*>(base + (int64_t)e * ld) + voff);
        r[e >> 1][(e & 1) * 2] = v[0];
        r[e >> 1][(e & 1) * 2 + 1] = v[1];
      }
    }
  }
  __device__ __forceinline__ void store(char* lds, int t) const {
    const int kb = t & 3, rb = t >> 2;
    if (MODE == 0) {
#pragma unroll
      for (int i = 0; i < 4; ++i) *reinterpret_cast<u32x4*>(lds + lds_off(rb + 64 * i, kb)) = r[i];
    } else {
      // reduction index e lives in r[e/2][(e%2)*2 + p], p = row pair (rows 2p, 2p+1 in the low/high half).
      // Row u of the output needs, in dword q, reduction indices (2q, 2q+1) of row u.
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        u32x4 o;
#pragma unroll
        for (int q = 0; q < 4; ++q)
          o[q] = __builtin_amdgcn_perm(r[q][2 + (u >> 1)], r[q][u >> 1], (u & 1) ? 0x07060302u : 0x05040100u);
        *reinterpret_cast<u32x4*>(lds + lds_off(rb * 4 + u, kb)) = o;
      }
    }
  }
};

// acc[bm][bn] += A_tile(256 x K) * B_tile(256 x K)^T for this wave's 128x128 quarter.
// A, Bp point at element (row 0, k 0) of the tile; ktiles = K / 32, which must be even and positive.
//
// Software pipeline.  Four LDS stages of one 32-wide K-step each and two register sets:
//   step kt, sub-step 0: MFMAs on the first 16 of the reduction index; fetch the fragments of sub-step 1;
//                        issue the global loads of K-step kt+3 into the register set that is free;
//   barrier (LDS traffic only, never the global loads);
//   step kt, sub-step 1: MFMAs; fetch the first fragments of step kt+1 from its stage; write the other
//                        register set (K-step kt+2, loaded during step kt-1) into stage (kt+2) % 4.
// Every sub-step therefore carries 16 MFMAs, 8 LDS reads and 8 loads or LDS writes: no bursts.  A global
// load has one and a half steps to land; an LDS stage is complete a full step before it is read and is
// not overwritten until two barriers after its last reader.  Loads past the end are clamped to the last
// K-step (redundant, never out of range).
#define DISCO_SGB(mask, n) __builtin_amdgcn_sched_group_barrier(mask, n, 0)
constexpr int SG_MFMA = 0x008, SG_VMEM_RD = 0x020, SG_DS_RD = 0x100, SG_DS_WR = 0x200;

__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

template <int MA, int MB>
__device__ __forceinline__ void mainloop(const uint16_t* __restrict__ A, int64_t lda, const uint16_t* __restrict__ Bp,
                                         int64_t ldb, int ktiles, char* smem, f32x16 (&acc)[4][4]) {
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int64_t stepA = MA == 0 ? BK : (int64_t)BK * lda;
  const int64_t stepB = MB == 0 ? BK : (int64_t)BK * ldb;
  const int last = ktiles - 1;
  const int arow = (wave >> 1) * 128 + (lane & 31), brow = (wave & 1) * 128 + (lane & 31), kc = lane >> 5;
  TileLoader<MA> la0, la1;
  TileLoader<MB> lb0, lb1;
  la0.init(lda, t); la1.init(lda, t); lb0.init(ldb, t); lb1.init(ldb, t);
  bf16x8 af0[4], bf0[4], af1[4], bf1[4];

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
  for (int i = 0; i < 4; ++i) {
    af0[i] = *reinterpret_cast<const bf16x8*>(smem + lds_off(arow + 32 * i, kc));
    bf0[i] = *reinterpret_cast<const bf16x8*>(smem + A_BYTES + lds_off(brow + 32 * i, kc));
  }

  // one K-step: loads go into (la_new, lb_new), LDS writes come from (la_old, lb_old)
  auto step = [&](int kt, TileLoader<MA>& la_new, TileLoader<MB>& lb_new, const TileLoader<MA>& la_old,
                  const TileLoader<MB>& lb_old) __attribute__((always_inline)) {
    const char* cur = smem + (kt & 3) * STAGE_BYTES;
    const char* nxt = smem + ((kt + 1) & 3) * STAGE_BYTES;
    char* wr = smem + ((kt + 2) & 3) * STAGE_BYTES;
    const int kload = kt + 3 < ktiles ? kt + 3 : last;
    // sub-step 0
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      af1[i] = *reinterpret_cast<const bf16x8*>(cur + lds_off(arow + 32 * i, 2 + kc));
      bf1[i] = *reinterpret_cast<const bf16x8*>(cur + A_BYTES + lds_off(brow + 32 * i, 2 + kc));
    }
    la_new.load(A + kload * stepA, lda);
    lb_new.load(Bp + kload * stepB, ldb);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af0[i], bf0[j], acc[i][j], 0, 0, 0);
#pragma unroll
    for (int g = 0; g < 4; ++g) { DISCO_SGB(SG_DS_RD, 2); DISCO_SGB(SG_MFMA, 2); }
#pragma unroll
    for (int g = 0; g < 4; ++g) { DISCO_SGB(SG_VMEM_RD, (MA == 0 ? 1 : 2) + (MB == 0 ? 1 : 2)); DISCO_SGB(SG_MFMA, 2); }
    __builtin_amdgcn_sched_barrier(0);   // nothing moves between sub-steps
    // sub-step 1
    lds_barrier();
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      af0[i] = *reinterpret_cast<const bf16x8*>(nxt + lds_off(arow + 32 * i, kc));
      bf0[i] = *reinterpret_cast<const bf16x8*>(nxt + A_BYTES + lds_off(brow + 32 * i, kc));
    }
    la_old.store(wr, t);
    lb_old.store(wr + A_BYTES, t);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af1[i], bf1[j], acc[i][j], 0, 0, 0);
#pragma unroll
    for (int g = 0; g < 4; ++g) { DISCO_SGB(SG_DS_RD, 2); DISCO_SGB(SG_MFMA, 2); }
#pragma unroll
    for (int g = 0; g < 4; ++g) { DISCO_SGB(SG_DS_WR, 2); DISCO_SGB(SG_MFMA, 2); }
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
__device__ __forceinline__ void store_tile_f32(f32x16 (&acc)[4][4], char* smem, float* out, int64_t ld, float scale) {
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = wave >> 1, wn = wave & 1, half = lane >> 5;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    lds_barrier();
    if (wm == h) {
#pragma unroll
      for (int bn = 0; bn < 4; ++bn)
#pragma unroll
        for (int bm = 0; bm < 4; ++bm)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int row = bm * 32 + (e >> 2) * 8 + half * 4 + (e & 3);
            const int col = wn * 128 + bn * 32 + (lane & 31);
            *reinterpret_cast<float*>(smem + row * OUT_ROW_BYTES + col * 4) = scale * acc[bm][bn][e];
          }
    }
    lds_barrier();
    const int chunk = t & 63, r0 = t >> 6;
#pragma unroll 4
    for (int r = 0; r < 32; ++r) {
      const int row = r * 4 + r0;
      f32x4 v = *reinterpret_cast<const f32x4*>(smem + row * OUT_ROW_BYTES + chunk * 16);
      float* g = out + (int64_t)(h * 128 + row) * ld + chunk * 4;
      if (ACCUMULATE) v += *reinterpret_cast<const f32x4*>(g);
      *reinterpret_cast<f32x4*>(g) = v;
    }
  }
}

}  // namespace tile
}  // namespace disco
