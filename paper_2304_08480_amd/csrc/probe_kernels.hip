// Measurement only: a matrix-core issue loop with no memory traffic, to show what the chip sustains when every
// compute unit does nothing but bf16 MFMAs (the ceiling that the clock management leaves under the published
// peak), and the shader clock it runs at meanwhile.  Called by bench.py --op mfma-peak.
#include "common.h"

namespace disco {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

// 512 threads = two waves per SIMD, each with eight independent 32x32 accumulators (the shape of the tile loops);
// operands are pseudo-random bf16 patterns: with `varied` sign, exponent and mantissa differ from element to element,
// so that the multipliers toggle as they do on real data; without, only the mantissas do (values in [0.5, 1)), which
// draws less power and shows how much of the ceiling is the data's doing.
// clocks[0..1] of workgroup 0: elapsed shader-clock ticks and elapsed ticks of the fixed 100 MHz counter.
__global__ __launch_bounds__(512) void k_mfma_probe(int iters, int varied, float* sink, unsigned long long* clocks) {
  const unsigned long long t0 = __builtin_readcyclecounter(), r0 = __builtin_amdgcn_s_memrealtime();
  f32x16 acc[8];
#pragma unroll
  for (int a = 0; a < 8; ++a)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[a][e] = 0.f;
  uint32_t h = 0x9e3779b9u * (threadIdx.x + 1) + blockIdx.x;
  uint32_t w[16];
#pragma unroll
  for (int k = 0; k < 16; ++k) {
    h = h * 1664525u + 1013904223u;
    // two bf16 values: random sign and mantissa, magnitude 2^-7 .. 2^-3; or positive values in [0.5, 1)
    w[k] = varied ? ((h & 0x81ff81ffu) | 0x3c003c00u) : ((h & 0x007f007fu) | 0x3f003f00u);
  }
  typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
  const bf16x8 x0 = __builtin_bit_cast(bf16x8, u32x4{w[0], w[1], w[2], w[3]}), x1 = __builtin_bit_cast(bf16x8, u32x4{w[4], w[5], w[6], w[7]});
  const bf16x8 y0 = __builtin_bit_cast(bf16x8, u32x4{w[8], w[9], w[10], w[11]}), y1 = __builtin_bit_cast(bf16x8, u32x4{w[12], w[13], w[14], w[15]});
  for (int i = 0; i < iters; ++i) {
#pragma unroll
    for (int a = 0; a < 8; ++a)
      acc[a] = __builtin_amdgcn_mfma_f32_32x32x16_bf16((a & 1) ? x1 : x0, (a & 2) ? y1 : y0, acc[a], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int a = 0; a < 8; ++a) s += acc[a][a];
  if (s == 12345.678f) sink[0] = s;                    // keeps the loop alive, never true
  const unsigned long long t1 = __builtin_readcyclecounter(), r1 = __builtin_amdgcn_s_memrealtime();
  if (blockIdx.x == 0 && threadIdx.x == 0) { clocks[0] = t1 - t0; clocks[1] = r1 - r0; }
}

}  // namespace
}  // namespace disco

extern "C" int disco_mfma_probe(int workgroups, int iters, int varied, float* sink, unsigned long long* clocks, void* hip_stream) {
  if (!sink || !clocks) return DISCO_ERR_NULL;
  if (workgroups <= 0 || workgroups > (1 << 20) || iters <= 0) return DISCO_ERR_SHAPE;
  disco::k_mfma_probe<<<dim3((unsigned)workgroups), 512, 0, static_cast<hipStream_t>(hip_stream)>>>(iters, varied, sink, clocks);
  return hipGetLastError() == hipSuccess ? DISCO_OK : DISCO_ERR_HIP;
}
