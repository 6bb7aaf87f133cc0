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

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int A_BYTES = BM * BK * 2;              // 32 KiB
constexpr int STAGE_BYTES = (BM + BN) * BK * 2;   // 64 KiB
constexpr int SMEM_BYTES = 2 * STAGE_BYTES;       // 128 KiB of the CU's 160 KiB
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;
constexpr float REF_HEADROOM = 100.f;             // largest exponent (base 2) a stored numerator may reach

// byte offset of 16-byte chunk `chunk` (0..7) of tile row `row` (128-byte rows, XOR swizzle)
__device__ __forceinline__ uint32_t lds_off(int row, int chunk) {
  return (uint32_t)row * 128u + (uint32_t)((chunk ^ (row & 7)) << 4);
}

// Copies a 256 x 64 bf16 operand tile from global memory to LDS through registers.
//   MODE 0: element (r, k) is at base[r * ld + k]   (reduction index contiguous)
//   MODE 1: element (r, k) is at base[k * ld + r]   (row index contiguous; 8x8 transposed in registers)
// Thread t owns chunk column kb = t % 8; in mode 0 rows (t/8) + 32 i, in mode 1 rows 8 (t/8) .. + 7.
template <int MODE>
struct TileLoader {
  u32x4 r[8];
  __device__ __forceinline__ void load(const uint16_t* base, int64_t ld, int t) {
    const int kb = t & 7, rb = t >> 3;
    if (MODE == 0) {
#pragma unroll
      for (int i = 0; i < 8; ++i) r[i] = *reinterpret_cast<const u32x4*>(base + (int64_t)(rb + 32 * i) * ld + kb * 8);
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) r[e] = *reinterpret_cast<const u32x4*>(base + (int64_t)(kb * 8 + e) * ld + rb * 8);
    }
  }
  __device__ __forceinline__ void store(char* lds, int t) const {
    const int kb = t & 7, rb = t >> 3;
    if (MODE == 0) {
#pragma unroll
      for (int i = 0; i < 8; ++i) *reinterpret_cast<u32x4*>(lds + lds_off(rb + 32 * i, kb)) = r[i];
    } else {
      // r[e][p] holds rows (2p, 2p+1) of reduction index e.  Row u of the output needs, in dword q,
      // reduction indices (2q, 2q+1): the low halves (u even) or high halves (u odd) of r[2q][u/2], r[2q+1][u/2].
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        u32x4 o;
#pragma unroll
        for (int q = 0; q < 4; ++q)
          o[q] = __builtin_amdgcn_perm(r[2 * q + 1][u >> 1], r[2 * q][u >> 1], (u & 1) ? 0x07060302u : 0x05040100u);
        *reinterpret_cast<u32x4*>(lds + lds_off(rb * 8 + u, kb)) = o;
      }
    }
  }
};

// acc[bm][bn] += A_tile(256 x K) * B_tile(256 x K)^T for this wave's 128x128 quarter.
// A, Bp point at element (row 0, k 0) of the tile; ktiles = K / 64.
//
// Software pipeline (one basic block per K-step so the interleaving below can be pinned).  Registers
// hold the global data of K-step kt+1 when step kt starts; LDS is double buffered.  Step kt:
//   sub-step 0,1: MFMAs, fetching the next sub-step's operand fragments from the current buffer;
//   sub-step 2  : fetch the last fragments, then write the registers to the other buffer, MFMAs;
//   barrier (waits on LDS traffic only, never on global loads);
//   sub-step 3  : fetch the first fragments of step kt+1 from the other buffer, issue the global loads
//                 of step kt+2 (clamped to the last step: redundant, never out of range), MFMAs.
// LDS reads never have to move across LDS writes, so the pinned order is also the program order.
#define DISCO_SGB(mask, n) __builtin_amdgcn_sched_group_barrier(mask, n, 0)
constexpr int SG_MFMA = 0x008, SG_VMEM_RD = 0x020, SG_DS_RD = 0x100, SG_DS_WR = 0x200;

__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

template <int MA, int MB>
__device__ __forceinline__ void mainloop(const uint16_t* __restrict__ A, int64_t lda, const uint16_t* __restrict__ Bp,
                                         int64_t ldb, int ktiles, char* smem, f32x16 (&acc)[4][4]) {
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int64_t stepA = MA == 0 ? BK : (int64_t)BK * lda;
  const int64_t stepB = MB == 0 ? BK : (int64_t)BK * ldb;
  TileLoader<MA> la;
  TileLoader<MB> lb;
  la.load(A, lda, t);
  lb.load(Bp, ldb, t);
  la.store(smem, t);
  lb.store(smem + A_BYTES, t);
  {
    const int k1 = ktiles > 1 ? 1 : 0;
    la.load(A + k1 * stepA, lda, t);
    lb.load(Bp + k1 * stepB, ldb, t);
  }
  lds_barrier();
  const int arow = wm * 128 + (lane & 31), brow = wn * 128 + (lane & 31), kc = lane >> 5;
  bf16x8 af[2][4], bfr[2][4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    af[0][i] = *reinterpret_cast<const bf16x8*>(smem + lds_off(arow + 32 * i, kc));
    bfr[0][i] = *reinterpret_cast<const bf16x8*>(smem + A_BYTES + lds_off(brow + 32 * i, kc));
  }
  for (int kt = 0; kt < ktiles; ++kt) {
    char* cur = smem + (kt & 1) * STAGE_BYTES;
    char* nxt = smem + ((kt + 1) & 1) * STAGE_BYTES;
    const int kload = kt + 2 < ktiles ? kt + 2 : ktiles - 1;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const int c = ks & 1, n = c ^ 1;
      if (ks == 3) lds_barrier();
      char* src = ks < 3 ? cur : nxt;
      const int kchunk = (ks < 3 ? (ks + 1) * 2 : 0) + kc;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        af[n][i] = *reinterpret_cast<const bf16x8*>(src + lds_off(arow + 32 * i, kchunk));
        bfr[n][i] = *reinterpret_cast<const bf16x8*>(src + A_BYTES + lds_off(brow + 32 * i, kchunk));
      }
      if (ks == 2) {
        la.store(nxt, t);
        lb.store(nxt + A_BYTES, t);
      }
      if (ks == 3) {
        la.load(A + kload * stepA, lda, t);
        lb.load(Bp + kload * stepB, ldb, t);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[c][i], bfr[c][j], acc[i][j], 0, 0, 0);
      // pin the interleaving of this sub-step
      if (ks < 2) {
#pragma unroll
        for (int g = 0; g < 8; ++g) { DISCO_SGB(SG_DS_RD, 1); DISCO_SGB(SG_MFMA, 2); }
      } else if (ks == 2) {
#pragma unroll
        for (int g = 0; g < 4; ++g) { DISCO_SGB(SG_DS_RD, 2); DISCO_SGB(SG_MFMA, 1); }
#pragma unroll
        for (int g = 0; g < 4; ++g) { DISCO_SGB(SG_DS_WR, 4); DISCO_SGB(SG_MFMA, 3); }
      } else {
#pragma unroll
        for (int g = 0; g < 8; ++g) { DISCO_SGB(SG_DS_RD, 1); DISCO_SGB(SG_VMEM_RD, 2); DISCO_SGB(SG_MFMA, 2); }
      }
    }
  }
}

}  // namespace tile
}  // namespace disco
