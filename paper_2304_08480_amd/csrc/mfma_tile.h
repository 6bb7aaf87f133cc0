// Device-side building blocks of the bf16 MFMA path: the 256x256x64 NT tile main loop, the operand
// tile formats and the tile store of the fp32 outputs (through LDS).  Included by mfma_kernels.hip only.
//
// Shape of the loop.  A workgroup of 8 waves (two per SIMD) owns a 256x256 output tile; each wave owns
// 128x64 of it as 4x2 MFMA 32x32x16 bf16 blocks with fp32 accumulators.  The reduction runs in K-steps of
// 64.  Operand tiles travel global memory -> LDS directly (global_load_lds_dwordx4): no staging
// registers, no LDS write instructions, and the data in flight lives in LDS.  K-steps are 64 wide so that
// a load instruction of a reduction-contiguous operand covers 8 rows x 128 bytes, i.e. whole cache lines
// (with 32-wide steps each line is fetched in two halves and such loads cost twice as much).
//
// A direct-to-LDS load holds its wave's instruction issue for tens of cycles (more when the memory
// pipeline is backed up), during which that wave issues no MFMA.  The loop therefore splits the loading
// between the two waves of each SIMD and staggers it by half a K-step: waves 0-3 load the A operand in the
// second quarter of a K-step, waves 4-7 the B operand in the fourth, so that one wave of every SIMD is
// always free to feed the matrix pipe.  To give those loads room, the LDS (all 160 KiB) is a ring of five
// 32 KiB units, each holding one operand of one K-step: A(kt), B(kt), A(kt+1), B(kt+1) resident or landing,
// plus one unit being refilled (see kloop).
//
// Operand tile formats in one unit:
//   format K - the operand's reduction index is contiguous in memory (element (r,k) at base[r*ld + k]):
//              256 rows of 128 bytes, 16-byte chunks XOR-swizzled with bits 1..3 of the row so that the
//              16 consecutive rows a quarter-wave reads (same chunk) hit 16 different bank groups of the
//              64-bank LDS; fragments are read with ds_read_b128.
//   format R - the operand's row index is contiguous in memory (element (r,k) at base[k*ld + r]): 64
//              reduction rows of 512 bytes; the 32-byte group index is XOR-ed with twice the low two bits
//              of the reduction row, so the 4 reduction rows x 2 row groups that a half-wave reads at once
//              cover a 256-byte bank window exactly; fragments are read with the transposing
//              ds_read_b64_tr_b16 (two per fragment).
// A direct-to-LDS load puts lane l's 16 bytes at (wave-uniform LDS base) + 16*l, so a swizzle is applied by
// choosing which global chunk each lane fetches.
//
// FMT_KA / FMT_RA read an operand kept in memory in "atoms": 16-byte pieces holding 8 consecutive columns of one
// row, laid out by groups of 64 rows, inside a group column piece by column piece, inside a column piece row by
// row: element (r, c) at ((r / 64) * (ncols / 8) + c / 8) * 512 + (r % 64) * 8 + c % 8; `ld` = elements between
// row groups (64 * ncols).  A column piece of a row group is 1 KiB of memory, a 64 x 64 block 8 KiB, and a producer
// whose lanes hold 8 consecutive columns of 32 or 64 consecutive rows stores whole 512-byte or 1 KiB runs straight
// from registers.
//   FMT_KA reduces along the columns (a K-step is 8 column pieces of each of the tile's four row groups: four
//          contiguous 8 KiB runs, and a load instruction fetches one column piece of one row group, 1 KiB).  Its LDS
//          tile keeps that order too: column piece c of the K-step at 4096 c, inside it tile row r at 16 r; the 16
//          consecutive rows a quarter-wave reads with ds_read_b128 are 256 contiguous bytes, so no swizzle.
//   FMT_RA reduces down the rows (a K-step is one row group; the tile's 256 rows are 32 column pieces of it: one
//          contiguous 32 KiB run, and a load instruction fetches one column piece, 1 KiB).  Its LDS tile keeps that
//          order: column piece c at 1024 c, inside it reduction row kap at 16 (kap ^ 4 (c % 4)), so that the
//          4 reduction rows x 4 column pieces x 2 halves which a half-wave reads at once with ds_read_b64_tr_b16
//          cover a 256-byte bank window exactly.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace disco {
namespace tile {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr int NTHREADS = 512;                     // 8 waves: 2 (M) x 4 (N), wave tile 128 x 64
constexpr int BM = 256, BN = 256, BK = 64;
constexpr int UNIT_BYTES = BM * BK * 2;           // 32 KiB: one operand, one K-step
constexpr int NUNITS = 5;
constexpr int SMEM_BYTES = NUNITS * UNIT_BYTES;   // all 160 KiB of the CU's LDS
constexpr int NLD = 8;                            // load instructions per loading wave and unit

enum { FMT_K = 0, FMT_R = 1, FMT_KA = 2, FMT_RA = 3 };
// bytes between the LDS destinations of a wave's consecutive load instructions (FMT_KA: the wave loads the 8 column
// pieces of its row group, which lie 4 KiB apart; else its instructions fill 8 KiB contiguously)
constexpr int lds_step(int f) { return f == FMT_KA ? 4096 : 1024; }

__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

template <int N>
__device__ __forceinline__ void wait_vmcnt() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }

// ---- LDS reads as opaque instructions: the compiler cannot tell which direct-to-LDS load a read depends
// on and would wait for all of them; the waits are placed by hand instead (wait_frags).
template <int OFF>
__device__ __forceinline__ u32x4 ds_read128(uint32_t addr) {
  u32x4 v;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
  return v;
}
template <int OFF>
__device__ __forceinline__ u32x2 ds_read64_tr(uint32_t addr) {
  u32x2 v;
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
  return v;
}

// Operand fragments of one 16-wide sub-step: 4 for the A side (rows 32 i), 2 for the B side.
struct Frags {
  u32x4 a[4], b[2];
};
// All LDS reads issued so far have returned; ties the registers to the wait so no MFMA moves above it.
__device__ __forceinline__ void wait_frags(Frags& f) {
  asm volatile("s_waitcnt lgkmcnt(0)"
               : "+v"(f.a[0]), "+v"(f.a[1]), "+v"(f.a[2]), "+v"(f.a[3]), "+v"(f.b[0]), "+v"(f.b[1])
               :
               : "memory");
}

// A pointer that is the same in every lane, handed to the compiler as scalar registers: the loads below then take
// the form scalar base + 32-bit lane offset, with no 64-bit vector address arithmetic and no vector registers for it.
__device__ __forceinline__ const char* uniform_ptr(const void* p) {
  const uint64_t v = reinterpret_cast<uint64_t>(p);
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return reinterpret_cast<const char*>(((uint64_t)hi << 32) | lo);
}

// ---- per-lane addressing of one operand
template <int FMT, int NFRAG>
struct Operand {
  uint32_t ld_off[NLD];     // byte offset of this lane's global chunk for the wave's load instructions
  uint32_t rd[4];           // FMT_K/KA: rd[ks] base for sub-step ks; FMT_R: rd[i] base for fragment i; FMT_RA: rd[h]
                            // base of the fragment's first (h = 0) and second (h = 1) transposing read
  uint32_t lds_q;           // LDS byte offset (inside the operand tile) of the wave's first load instruction

  // lw: index 0..3 of this wave among the four that load this operand; row0: first tile row of this
  // wave's fragments (multiple of 32); ld in elements; nvalid: tile rows that exist in memory (a multiple of
  // 8, at most 256): loads of the rows past them are redirected to the last existing rows, so that they
  // stay in bounds (the caller does not use the output rows or columns they feed)
  __device__ __forceinline__ void init(int64_t ld, int lw, int lane, int row0, int nvalid = BM) {
    const int wave = lw;
    lds_q = FMT == FMT_KA ? wave * 1024 : NLD * wave * 1024;
#pragma unroll
    for (int n = 0; n < NLD; ++n) {
      const int q = NLD * wave + n;               // which 1 KiB slice of the 32 KiB tile
      if (FMT == FMT_K) {
        const int rho = 8 * q + (lane >> 3), pc = lane & 7;
        const int ch = (pc ^ ((rho >> 1) & 7)) << 3;
        const int rsrc = rho < nvalid ? rho : nvalid - 1;
        ld_off[n] = (uint32_t)(((int64_t)rsrc * ld + ch) * 2);
      } else if (FMT == FMT_KA) {                   // row group `wave`, column piece n of the K-step, row `lane` of the group
        ld_off[n] = (uint32_t)(((int64_t)wave * ld + n * 512 + lane * 8) * 2);
      } else if (FMT == FMT_RA) {
        const int c = q;                            // this instruction's column piece; lane = position in it
        ld_off[n] = (uint32_t)((c * 512 + (lane ^ ((c & 3) << 2)) * 8) * 2);
      } else {
        const int kap = 2 * q + (lane >> 5), pcw = lane & 31;
        const int c0 = (((pcw >> 1) ^ ((kap & 3) << 1)) << 1) | (pcw & 1);
        const int c = (c0 << 3) < nvalid ? c0 : (nvalid >> 3) - 1;
        ld_off[n] = (uint32_t)(((int64_t)kap * ld + (c << 3)) * 2);
      }
    }
    if (FMT == FMT_K) {
      const int row = row0 + (lane & 31), g = (row >> 1) & 7, kc = lane >> 5;
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) rd[ks] = (uint32_t)(row * 128 + (((ks * 2 + kc) ^ g) << 4));
    } else if (FMT == FMT_KA) {
      const int row = row0 + (lane & 31), kc = lane >> 5;
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) rd[ks] = (uint32_t)((ks * 2 + kc) * 4096 + row * 16);
    } else if (FMT == FMT_RA) {
      const int grp = lane >> 4, L = lane & 15, piece = L & 3;     // piece: 8-byte quarter of a 16-row (32-byte) group
      const int c = ((row0 + (grp & 1) * 16) >> 3) + (piece >> 1);   // + 4 per fragment: c % 4 unchanged
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int kap = (grp >> 1) * 8 + (L >> 2) + 4 * h;           // + 16 ks: bits 2..3 unchanged
        rd[h] = (uint32_t)(c * 1024 + ((kap ^ ((c & 3) << 2)) << 4) + (piece & 1) * 8);
      }
    } else {
      const int grp = lane >> 4, L = lane & 15;
      const int kap = (grp >> 1) * 8 + (L >> 2);  // + 16 ks + 4 h, multiples of 4: (kap & 3) unchanged
#pragma unroll
      for (int i = 0; i < NFRAG; ++i) {
        const int G = (row0 + 32 * i + (grp & 1) * 16) >> 4;
        rd[i] = (uint32_t)(kap * 512 + ((G ^ ((kap & 3) << 1)) << 5) + 8 * (L & 3));
      }
    }
  }
  // issue this wave's loads of the K-step whose tile starts at `base` into the unit at `lds`
  __device__ __forceinline__ void load(const uint16_t* base, char* lds) const {
    char* l0 = lds + __builtin_amdgcn_readfirstlane(lds_q);
    const char* ub = uniform_ptr(base);
#pragma unroll
    for (int n = 0; n < NLD; ++n) {
      const char* gp = ub + ld_off[n];
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gp,
                                       (__attribute__((address_space(3))) void*)(l0 + n * lds_step(FMT)), 16, 0, 0);
    }
  }
};

__device__ __forceinline__ u32x4 join(u32x2 lo, u32x2 hi) { return u32x4{lo[0], lo[1], hi[0], hi[1]}; }

// fragment i of sub-step KS from the operand tile at LDS byte address `tile`
template <int FMT, int NFRAG, int KS, int I>
__device__ __forceinline__ u32x4 read_frag(const Operand<FMT, NFRAG>& op, uint32_t tile) {
  if (FMT == FMT_K) return ds_read128<I * 4096>(tile + op.rd[KS]);
  if (FMT == FMT_KA) return ds_read128<I * 512>(tile + op.rd[KS]);
  if (FMT == FMT_RA) return join(ds_read64_tr<KS * 256 + I * 4096>(tile + op.rd[0]), ds_read64_tr<KS * 256 + I * 4096>(tile + op.rd[1]));
  return join(ds_read64_tr<KS * 8192>(tile + op.rd[I]), ds_read64_tr<KS * 8192 + 2048>(tile + op.rd[I]));
}
template <int FA, int FB, int KS>
__device__ __forceinline__ void read_frags(Frags& f, const Operand<FA, 4>& a, const Operand<FB, 2>& b, uint32_t ta, uint32_t tb) {
  f.a[0] = read_frag<FA, 4, KS, 0>(a, ta);
  f.b[0] = read_frag<FB, 2, KS, 0>(b, tb);
  f.a[1] = read_frag<FA, 4, KS, 1>(a, ta);
  f.b[1] = read_frag<FB, 2, KS, 1>(b, tb);
  f.a[2] = read_frag<FA, 4, KS, 2>(a, ta);
  f.a[3] = read_frag<FA, 4, KS, 3>(a, ta);
}
__device__ __forceinline__ void mfma1(f32x16& c, const u32x4& a, const u32x4& b) {
  c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}
// acc = a * b (the matrix instruction takes a literal zero for its addend: no registers are cleared)
__device__ __forceinline__ void mfma_block_first(const Frags& f, f32x16 (&acc)[4][2]) {
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f.a[i]), __builtin_bit_cast(bf16x8, f.b[j]), zero, 0, 0, 0);
}
__device__ __forceinline__ void mfma_block(const Frags& f, f32x16 (&acc)[4][2]) {
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) mfma1(acc[i][j], f.a[i], f.b[j]);
}
// the 8 MFMAs of a sub-step with this wave's 8 load instructions of one unit interleaved (two after each of the
// first four: how they are spread over the sub-step makes no measurable difference).  The wave runs this
// sub-step at raised priority: it then wins the SIMD's issue slots from the other wave group's wave, its loads
// leave early in the K-step and have the longest time to land (query-side GEMM 6 % faster, logit kernel 1 %;
// raising the priority of every MFMA block instead is 1-4 % slower everywhere)
template <int FMT, int NFRAG>
__device__ __forceinline__ void mfma_block_loads(const Frags& f, f32x16 (&acc)[4][2], const Operand<FMT, NFRAG>& op,
                                                 const uint16_t* base, char* lds) {
  char* l0 = lds + __builtin_amdgcn_readfirstlane(op.lds_q);
  const char* ub = uniform_ptr(base);
#define DISCO_LD(n)                                                                                                         \
  __builtin_amdgcn_global_load_lds(                                                                                         \
      (const __attribute__((address_space(1))) void*)(ub + op.ld_off[n]),                                                   \
      (__attribute__((address_space(3))) void*)(l0 + n * lds_step(FMT)), 16, 0, 0)
  __builtin_amdgcn_s_setprio(1);
  mfma1(acc[0][0], f.a[0], f.b[0]); DISCO_LD(0); DISCO_LD(1);
  mfma1(acc[0][1], f.a[0], f.b[1]); DISCO_LD(2); DISCO_LD(3);
  mfma1(acc[1][0], f.a[1], f.b[0]); DISCO_LD(4); DISCO_LD(5);
  mfma1(acc[1][1], f.a[1], f.b[1]); DISCO_LD(6); DISCO_LD(7);
  mfma1(acc[2][0], f.a[2], f.b[0]);
  mfma1(acc[2][1], f.a[2], f.b[1]);
  mfma1(acc[3][0], f.a[3], f.b[0]);
  mfma1(acc[3][1], f.a[3], f.b[1]);
  __builtin_amdgcn_s_setprio(0);
#undef DISCO_LD
}

__device__ __forceinline__ int ring_next(int u, int step) { u += step; return u >= NUNITS ? u - NUNITS : u; }

// The K loop of one wave group.  GROUP 0 (waves 0-3) loads the A units, GROUP 1 (waves 4-7) the B units.
//
// Ring of five units; the operand tiles are laid into it in the order A0 B0 A1 B1 A2 B2 ..., item n in
// unit n mod 5.  K-step kt computes from A(kt), B(kt) in four 16-wide sub-steps, each fetching the next
// sub-step's fragments while its MFMAs run:
//   sub-step 0;
//   sub-step 1: group 0 issues the loads of A(kt+2) into the unit that held B(kt-1);
//   sub-step 2, then: wait for this wave's loads of K-step kt+1 (group 0 may leave the 8 loads of A(kt+2)
//       in flight, group 1 has nothing younger), wait for its own LDS reads, barrier: K-step kt+1 is complete
//       in LDS and nobody reads the units of K-step kt any more (the last fragments are in registers);
//   sub-step 3: group 1 issues the loads of B(kt+2) into the unit that held A(kt); the first fragments of
//       K-step kt+1 are fetched.
// So an A load has six sub-steps to land and a B load four.  Loads past the end are clamped to the last
// K-step (redundant, never out of range, into a unit nobody reads again).
// READS_FIRST: issue a sub-step's LDS reads ahead of its MFMAs (otherwise the compiler places them).
template <int FMT>
__device__ __forceinline__ int64_t kstep_elems(int64_t ld) {
  return FMT == FMT_K ? BK : FMT == FMT_KA ? 4096 : FMT == FMT_R ? (int64_t)BK * ld : ld;
}

// WRITE_FIRST: the first K-step is peeled off the loop and writes the accumulators (acc = product, acc need not be
// initialised); else every K-step adds to them (acc += product).  Peeling gains 2-5 % on the gradient GEMMs; in the
// logit kernel it costs the epilogue registers it does not have.
template <int FA, int FB, int GROUP, bool READS_FIRST, bool WRITE_FIRST>
__device__ __forceinline__ void kloop(const uint16_t* __restrict__ A, int64_t lda, const uint16_t* __restrict__ Bp, int64_t ldb,
                                      int ktiles, char* smem, f32x16 (&acc)[4][2], int nvalid_b) {
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int64_t stepA = kstep_elems<FA>(lda);
  const int64_t stepB = kstep_elems<FB>(ldb);
  const int last = ktiles - 1;
  Operand<FA, 4> oa;
  Operand<FB, 2> ob;
  oa.init(lda, wave & 3, lane, (wave >> 2) * 128);
  ob.init(ldb, wave & 3, lane, (wave & 3) * 64, nvalid_b);
  const uint32_t smem_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem;   // LDS byte address
  const int k1 = last < 1 ? last : 1;
  if (GROUP == 0) {
    oa.load(A, smem);
    oa.load(A + k1 * stepA, smem + 2 * UNIT_BYTES);
  } else {
    ob.load(Bp, smem + UNIT_BYTES);
    ob.load(Bp + k1 * stepB, smem + 3 * UNIT_BYTES);
  }
  wait_vmcnt<NLD>();
  lds_barrier();
  Frags f0, f1;
  read_frags<FA, FB, 0>(f0, oa, ob, smem_addr, smem_addr + UNIT_BYTES);
  wait_frags(f0);

  int rA = 0;                                       // unit of A(kt); B(kt) is the next unit of the ring
  // One K-step (FIRST_BLOCK: what sub-step 0 does with its fragments: mfma_block adds to the accumulators,
  // mfma_block_first writes them).
#define DISCO_KSTEP(FIRST_BLOCK)                                                                                             \
  {                                                                                                                        \
    const int rB = ring_next(rA, 1), nA = ring_next(rA, 2), nB = ring_next(rA, 3), lA = ring_next(rA, 4);                  \
    const uint32_t ta = smem_addr + (uint32_t)(rA * UNIT_BYTES), tb = smem_addr + (uint32_t)(rB * UNIT_BYTES);             \
    const int kload = kt + 2 < ktiles ? kt + 2 : last;                                                                     \
    /* sub-step 0 */                                                                                                       \
    read_frags<FA, FB, 1>(f1, oa, ob, ta, tb);                                                                             \
    if (READS_FIRST) __builtin_amdgcn_sched_barrier(0);                                                                    \
    FIRST_BLOCK(f0, acc);                                                                                                  \
    __builtin_amdgcn_sched_barrier(0);                                                                                     \
    wait_frags(f1);                                                                                                        \
    /* sub-step 1 */                                                                                                       \
    read_frags<FA, FB, 2>(f0, oa, ob, ta, tb);                                                                             \
    if (READS_FIRST) __builtin_amdgcn_sched_barrier(0);                                                                    \
    if (GROUP == 0) mfma_block_loads(f1, acc, oa, A + kload * stepA, smem + lA * UNIT_BYTES);                              \
    else mfma_block(f1, acc);                                                                                              \
    __builtin_amdgcn_sched_barrier(0);                                                                                     \
    wait_frags(f0);                                                                                                        \
    /* sub-step 2 */                                                                                                       \
    read_frags<FA, FB, 3>(f1, oa, ob, ta, tb);                                                                             \
    if (READS_FIRST) __builtin_amdgcn_sched_barrier(0);                                                                    \
    mfma_block(f0, acc);                                                                                                   \
    __builtin_amdgcn_sched_barrier(0);                                                                                     \
    if (GROUP == 0) wait_vmcnt<NLD>(); else wait_vmcnt<0>();                                                               \
    wait_frags(f1);                                                                                                        \
    asm volatile("s_barrier" ::: "memory");                                                                                \
    __builtin_amdgcn_sched_barrier(0);                                                                                     \
    /* sub-step 3 */                                                                                                       \
    read_frags<FA, FB, 0>(f0, oa, ob, smem_addr + (uint32_t)(nA * UNIT_BYTES), smem_addr + (uint32_t)(nB * UNIT_BYTES));   \
    if (READS_FIRST) __builtin_amdgcn_sched_barrier(0);                                                                    \
    if (GROUP == 1) mfma_block_loads(f1, acc, ob, Bp + kload * stepB, smem + rA * UNIT_BYTES);                             \
    else mfma_block(f1, acc);                                                                                              \
    __builtin_amdgcn_sched_barrier(0);                                                                                     \
    wait_frags(f0);                                                                                                        \
    __builtin_amdgcn_sched_barrier(0);                                                                                     \
    rA = nA;                                                                                                               \
  }
  if constexpr (WRITE_FIRST) {
    // (the K-step as a generic lambda instantiated twice: this form, not only the peeling, is what the compiler
    // schedules 2-5 % better in the gradient GEMMs)
    auto kstep = [&](int kt, auto first) {
      if constexpr (decltype(first)::value) DISCO_KSTEP(mfma_block_first)
      else DISCO_KSTEP(mfma_block)
    };
    kstep(0, std::true_type{});
    for (int kt = 1; kt < ktiles; ++kt) kstep(kt, std::false_type{});
  } else {
    for (int kt = 0; kt < ktiles; ++kt) DISCO_KSTEP(mfma_block)
  }
#undef DISCO_KSTEP
  wait_vmcnt<0>();
  lds_barrier();
}

// acc[bm][bn] (+)= A_tile(256 x K) * B_tile(256 x K)^T for this wave's 128 x 64 piece (WRITE_FIRST: =, see kloop).
//   FA / FB : tile format of the A / B operand (FMT_K: element (r,k) at base[r*ld + k]; FMT_R: at base[k*ld + r];
//             FMT_KA / FMT_RA: the same for storage in 16-byte atoms, see the top of this file).
//   A, Bp   : element (row 0, k 0) of the workgroup's operand tiles; ktiles = K / 64 >= 1.
//   smem    : SMEM_BYTES of LDS, 16-byte aligned; on return no load is in flight and every wave has passed
//             a barrier, so the caller may reuse it at once.
//   nvalid_b: rows of the B tile that exist in memory (multiple of 8, <= 256); the output columns from
//             nvalid_b on are then meaningless and must not be stored.
template <int FA, int FB, bool READS_FIRST, bool WRITE_FIRST = false>
__device__ __forceinline__ void mainloop(const uint16_t* __restrict__ A, int64_t lda, const uint16_t* __restrict__ Bp,
                                         int64_t ldb, int ktiles, char* smem, f32x16 (&acc)[4][2], int nvalid_b = BN) {
  if (threadIdx.x < NTHREADS / 2) kloop<FA, FB, 0, READS_FIRST, WRITE_FIRST>(A, lda, Bp, ldb, ktiles, smem, acc, nvalid_b);
  else kloop<FA, FB, 1, READS_FIRST, WRITE_FIRST>(A, lda, Bp, ldb, ktiles, smem, acc, nvalid_b);
}

// Writes a workgroup's 256 x 256 fp32 accumulator tile to row-major global memory through LDS, so that
// every global store is a full 1 KiB row segment (the accumulator layout would give 4-byte elements per
// lane).  Two passes of 128 rows; LDS rows padded to 1056 bytes so that the two half-waves of a 4-byte
// write land on different banks.  out points at the tile's first element; value = scale * acc (+ old);
// only the first ncols columns (a multiple of 4) of the first nrows rows are touched.
constexpr int OUT_ROW_BYTES = BN * 4 + 32;
constexpr int OUT_SMEM_BYTES = 128 * OUT_ROW_BYTES;       // 132 KiB

template <bool ACCUMULATE, bool ROWMASK>
__device__ __forceinline__ void store_tile_f32_rows(f32x16 (&acc)[4][2], char* smem, float* out, int64_t ld, float scale, int ncols, int nrows) {
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = wave >> 2, wn = wave & 3, half = lane >> 5;
  const int chunk = t & 63, r0 = t >> 6;
  const bool live = chunk * 4 < ncols;             // this thread's four columns exist (ncols is a multiple of 4)
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    // when accumulating, the old values are requested eight rows at a time, the first eight before the
    // staging so that their latency is paid under the LDS traffic
    f32x4 old[8];
    if (ACCUMULATE && live) {
#pragma unroll
      for (int r = 0; r < 8; ++r)
        if (!ROWMASK || h * 128 + r * 8 + r0 < nrows) old[r] = *reinterpret_cast<const f32x4*>(out + (int64_t)(h * 128 + r * 8 + r0) * ld + chunk * 4);
    }
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
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      f32x4 v[8];
#pragma unroll
      for (int r = 0; r < 8; ++r) v[r] = *reinterpret_cast<const f32x4*>(smem + ((q * 8 + r) * 8 + r0) * OUT_ROW_BYTES + chunk * 16);
      if (ACCUMULATE && q == 1 && live) {
#pragma unroll
        for (int r = 0; r < 8; ++r)
          if (!ROWMASK || h * 128 + (8 + r) * 8 + r0 < nrows) old[r] = *reinterpret_cast<const f32x4*>(out + (int64_t)(h * 128 + (8 + r) * 8 + r0) * ld + chunk * 4);
      }
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        const bool there = live && (!ROWMASK || h * 128 + (q * 8 + r) * 8 + r0 < nrows);
        float* g = out + (int64_t)(h * 128 + (q * 8 + r) * 8 + r0) * ld + chunk * 4;
        if (ACCUMULATE && there) v[r] += old[r];
        if (there) *reinterpret_cast<f32x4*>(g) = v[r];
      }
    }
  }
}

// (a tile whose rows all exist takes the instance without the per-row tests)
template <bool ACCUMULATE>
__device__ __forceinline__ void store_tile_f32(f32x16 (&acc)[4][2], char* smem, float* out, int64_t ld, float scale, int ncols = BN,
                                               int nrows = BM) {
  if (nrows >= BM) store_tile_f32_rows<ACCUMULATE, false>(acc, smem, out, ld, scale, ncols, nrows);
  else store_tile_f32_rows<ACCUMULATE, true>(acc, smem, out, ld, scale, ncols, nrows);
}

}  // namespace tile
}  // namespace disco
