// Feature preparation around the loss: row L2 normalisation (forward and backward) and the
// parametrisation of the logit multiplier.  HBM-bound row kernels, one wave per row.
//
//   forward :  u = x / max(|x|, eps),  inv = 1 / max(|x|, eps),  eps = 1e-12
//   backward:  dx = (g - <g, u> u) inv          (|x| > eps; Jacobian (I - u u^T) / |x|)
//              dx = g inv                        (the cap is active)
//   multiplier: s = min(exp(theta), s_max),  d/dtheta = gs exp(theta) where exp(theta) <= s_max, else 0
#include "common.h"

namespace disco {
namespace {

typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr float NORM_EPS = 1e-12f;

__device__ __forceinline__ float wave_sum(float v) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}
__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  __bf16 v = (__bf16)f;     // round to nearest even
  return *reinterpret_cast<uint16_t*>(&v);
}

template <bool BF16>
__device__ __forceinline__ float load1(const void* p, int64_t idx) {
  return BF16 ? bf16_to_f32(static_cast<const uint16_t*>(p)[idx]) : static_cast<const float*>(p)[idx];
}
// four consecutive elements starting at idx (idx and the row pitch are multiples of 4)
template <bool BF16>
__device__ __forceinline__ f32x4 load4(const void* p, int64_t idx) {
  if (BF16) {
    const u32x2 w = *reinterpret_cast<const u32x2*>(static_cast<const uint16_t*>(p) + idx);
    return f32x4{__uint_as_float(w[0] << 16), __uint_as_float(w[0] & 0xffff0000u), __uint_as_float(w[1] << 16),
                 __uint_as_float(w[1] & 0xffff0000u)};
  }
  return *reinterpret_cast<const f32x4*>(static_cast<const float*>(p) + idx);
}
template <bool BF16>
__device__ __forceinline__ void store4(void* p, int64_t idx, f32x4 v) {
  if (BF16) {
    u32x2 w;
    w[0] = (uint32_t)f32_to_bf16(v[0]) | ((uint32_t)f32_to_bf16(v[1]) << 16);
    w[1] = (uint32_t)f32_to_bf16(v[2]) | ((uint32_t)f32_to_bf16(v[3]) << 16);
    *reinterpret_cast<u32x2*>(static_cast<uint16_t*>(p) + idx) = w;
  } else {
    *reinterpret_cast<f32x4*>(static_cast<float*>(p) + idx) = v;
  }
}
template <bool BF16>
__device__ __forceinline__ void store1(void* p, int64_t idx, float v) {
  if (BF16) static_cast<uint16_t*>(p)[idx] = f32_to_bf16(v);
  else static_cast<float*>(p)[idx] = v;
}

// One wave per row, rows dealt round-robin to the waves of the grid.  The row is read twice (sum of squares,
// then scaling); the second read is served by the cache.  VEC: d is a multiple of 4.
template <bool IN_BF16, bool OUT_BF16, bool VEC>
__global__ __launch_bounds__(256) void k_normalize_fwd(const void* X, int64_t rows, int64_t d, void* U, float* inv_norm) {
  const int lane = threadIdx.x & 63;
  const int64_t wave0 = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6), nwaves = (int64_t)gridDim.x * 4;
  for (int64_t r = wave0; r < rows; r += nwaves) {
    const int64_t base = r * d;
    float ss = 0.f;
    if (VEC) {
      for (int64_t k = lane * 4; k < d; k += 256) {
        const f32x4 v = load4<IN_BF16>(X, base + k);
        ss = fmaf(v[0], v[0], ss); ss = fmaf(v[1], v[1], ss); ss = fmaf(v[2], v[2], ss); ss = fmaf(v[3], v[3], ss);
      }
    } else {
      for (int64_t k = lane; k < d; k += 64) { const float v = load1<IN_BF16>(X, base + k); ss = fmaf(v, v, ss); }
    }
    ss = wave_sum(ss);
    const float inv = 1.0f / fmaxf(sqrtf(ss), NORM_EPS);
    if (lane == 0) inv_norm[r] = inv;
    if (VEC) {
      for (int64_t k = lane * 4; k < d; k += 256) store4<OUT_BF16>(U, base + k, load4<IN_BF16>(X, base + k) * inv);
    } else {
      for (int64_t k = lane; k < d; k += 64) store1<OUT_BF16>(U, base + k, load1<IN_BF16>(X, base + k) * inv);
    }
  }
}

template <bool IN_BF16, bool VEC>
__global__ __launch_bounds__(256) void k_normalize_bwd(const float* G, const void* X, const float* inv_norm, int64_t rows, int64_t d,
                                                       float* DX) {
  const int lane = threadIdx.x & 63;
  const int64_t wave0 = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6), nwaves = (int64_t)gridDim.x * 4;
  for (int64_t r = wave0; r < rows; r += nwaves) {
    const int64_t base = r * d;
    const float inv = inv_norm[r];
    const bool capped = inv >= 0.5f / NORM_EPS;         // forward divided by eps, not by |x|
    float dot = 0.f;
    if (!capped) {
      if (VEC) {
        for (int64_t k = lane * 4; k < d; k += 256) {
          const f32x4 g = *reinterpret_cast<const f32x4*>(G + base + k), x = load4<IN_BF16>(X, base + k);
          dot = fmaf(g[0], x[0], dot); dot = fmaf(g[1], x[1], dot); dot = fmaf(g[2], x[2], dot); dot = fmaf(g[3], x[3], dot);
        }
      } else {
        for (int64_t k = lane; k < d; k += 64) dot = fmaf(G[base + k], load1<IN_BF16>(X, base + k), dot);
      }
      dot = wave_sum(dot);
    }
    const float w = capped ? 0.f : dot * inv * inv;     // <g, u> / |x| : dx = (g - w x) inv
    if (VEC) {
      for (int64_t k = lane * 4; k < d; k += 256) {
        const f32x4 g = *reinterpret_cast<const f32x4*>(G + base + k), x = load4<IN_BF16>(X, base + k);
        *reinterpret_cast<f32x4*>(DX + base + k) = (g - x * w) * inv;
      }
    } else {
      for (int64_t k = lane; k < d; k += 64) DX[base + k] = (G[base + k] - w * load1<IN_BF16>(X, base + k)) * inv;
    }
  }
}

__global__ void k_logit_scale_fwd(const float* theta, float s_max, float* s) {
  if (threadIdx.x == 0) *s = fminf(expf(*theta), s_max);
}
__global__ void k_logit_scale_bwd(const float* theta, float s_max, const float* gs, float* gtheta, int accumulate) {
  if (threadIdx.x == 0) {
    const float e = expf(*theta);
    const float g = e <= s_max ? *gs * e : 0.f;
    *gtheta = (accumulate ? *gtheta : 0.f) + g;
  }
}

unsigned row_grid(int64_t rows) {
  const int64_t blocks = (rows + 3) / 4;
  return (unsigned)(blocks < 8192 ? blocks : 8192);
}
bool dtype_ok(int t) { return t == DISCO_F32 || t == DISCO_BF16; }
bool rows_ok(int64_t rows, int64_t d) { return rows > 0 && d > 0 && rows <= ((int64_t)1 << 40) / d; }

}  // namespace
}  // namespace disco

using namespace disco;

extern "C" int disco_normalize_fwd(const void* X, int64_t rows, int64_t d, int x_dtype, void* U, int u_dtype, float* inv_norm,
                                   void* hip_stream) {
  if (!X || !U || !inv_norm) return DISCO_ERR_NULL;
  if (!rows_ok(rows, d)) return DISCO_ERR_SHAPE;
  if (!dtype_ok(x_dtype) || !dtype_ok(u_dtype)) return DISCO_ERR_UNSUPPORTED;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const dim3 g(row_grid(rows));
  const bool vec = d % 4 == 0;
#define DISCO_FWD(IB, OB)                                                                                  \
  do {                                                                                                     \
    if (vec) k_normalize_fwd<IB, OB, true><<<g, 256, 0, st>>>(X, rows, d, U, inv_norm);                     \
    else k_normalize_fwd<IB, OB, false><<<g, 256, 0, st>>>(X, rows, d, U, inv_norm);                        \
  } while (0)
  if (x_dtype == DISCO_BF16 && u_dtype == DISCO_BF16) DISCO_FWD(true, true);
  else if (x_dtype == DISCO_BF16) DISCO_FWD(true, false);
  else if (u_dtype == DISCO_BF16) DISCO_FWD(false, true);
  else DISCO_FWD(false, false);
#undef DISCO_FWD
  return hipGetLastError() == hipSuccess ? DISCO_OK : DISCO_ERR_HIP;
}

extern "C" int disco_normalize_bwd(const float* G, const void* X, int x_dtype, const float* inv_norm, int64_t rows, int64_t d,
                                   float* DX, void* hip_stream) {
  if (!G || !X || !inv_norm || !DX) return DISCO_ERR_NULL;
  if (!rows_ok(rows, d)) return DISCO_ERR_SHAPE;
  if (!dtype_ok(x_dtype)) return DISCO_ERR_UNSUPPORTED;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const dim3 g(row_grid(rows));
  const bool vec = d % 4 == 0;
  if (x_dtype == DISCO_BF16) {
    if (vec) k_normalize_bwd<true, true><<<g, 256, 0, st>>>(G, X, inv_norm, rows, d, DX);
    else k_normalize_bwd<true, false><<<g, 256, 0, st>>>(G, X, inv_norm, rows, d, DX);
  } else {
    if (vec) k_normalize_bwd<false, true><<<g, 256, 0, st>>>(G, X, inv_norm, rows, d, DX);
    else k_normalize_bwd<false, false><<<g, 256, 0, st>>>(G, X, inv_norm, rows, d, DX);
  }
  return hipGetLastError() == hipSuccess ? DISCO_OK : DISCO_ERR_HIP;
}

extern "C" int disco_logit_scale_fwd(const float* theta, float s_max, float* s, void* hip_stream) {
  if (!theta || !s) return DISCO_ERR_NULL;
  if (!(s_max > 0.f)) return DISCO_ERR_SHAPE;
  k_logit_scale_fwd<<<1, 64, 0, static_cast<hipStream_t>(hip_stream)>>>(theta, s_max, s);
  return hipGetLastError() == hipSuccess ? DISCO_OK : DISCO_ERR_HIP;
}

extern "C" int disco_logit_scale_bwd(const float* theta, float s_max, const float* gs, float* gtheta, int accumulate,
                                     void* hip_stream) {
  if (!theta || !gs || !gtheta) return DISCO_ERR_NULL;
  if (!(s_max > 0.f)) return DISCO_ERR_SHAPE;
  k_logit_scale_bwd<<<1, 64, 0, static_cast<hipStream_t>(hip_stream)>>>(theta, s_max, gs, gtheta, accumulate);
  return hipGetLastError() == hipSuccess ? DISCO_OK : DISCO_ERR_HIP;
}
