// The quantization operators of the generic quantization flow (paper Section 4.2):
//   simQ(x, beta, sigma, rho) = clip(round(x / rho * 2^(beta - sigma))) * rho / 2^(beta - sigma)
//   Q(x, rho, beta, sigma)    = cast(clip(round(x / rho * 2^(beta - sigma)), qtype))
// Elementwise and bandwidth-bound: 16-byte loads, one pass.  The code is decided in fp32, in the
// order written (an IEEE division, an exact scaling by a power of two, the rounding rule), so a
// host implementation in float32 reaches the same integers.  Clip is symmetric: +-(2^(beta-1) - 1).
#include "rounding.hpp"

namespace relay {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ float quantize_code(float x, float rho, float pow2, float qlo, float qhi, int mode,
                                               WordStream& rng, unsigned long long index) {
  const float t = (x / rho) * pow2;
  float q;
  if (mode == ROUND_NEAREST) q = floorf(t + 0.5f);  // ties toward +infinity
  else if (mode == ROUND_FLOOR) q = floorf(t);
  else if (mode == ROUND_CEIL) q = ceilf(t);
  else q = floorf(t + (float)(rng.word(index) >> 8) * 0x1p-24f);
  if (qlo == 0.f) return q > 0.f ? fminf(q, qhi) : 0.f;  // unsigned: whatever is not positive is the code +0
  return fminf(fmaxf(q, qlo), qhi);
}

// 8 elements per thread
template <bool SRC_F16, bool SIM>
__global__ __launch_bounds__(256) void quantize_kernel(long n, const void* xv, float rho, float pow2, float qlo,
                                                       float qhi, int mode, unsigned seed_lo, unsigned seed_hi,
                                                       void* yv) {
  const long i0 = ((long)blockIdx.x * 256 + threadIdx.x) * 8;
  if (i0 >= n) return;
  float x[8];
  const bool full = i0 + 8 <= n;
  if constexpr (SRC_F16) {
    const _Float16* xp = static_cast<const _Float16*>(xv) + i0;
    if (full) {
      const half8 v = *reinterpret_cast<const half8*>(xp);
#pragma unroll
      for (int e = 0; e < 8; ++e) x[e] = (float)v[e];
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) x[e] = i0 + e < n ? (float)xp[e] : 0.f;
    }
  } else {
    const float* xp = static_cast<const float*>(xv) + i0;
    if (full) {
      const float4 a = *reinterpret_cast<const float4*>(xp), b = *reinterpret_cast<const float4*>(xp + 4);
      x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w; x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) x[e] = i0 + e < n ? xp[e] : 0.f;
    }
  }
  WordStream rng{seed_lo, seed_hi};
  float q[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) q[e] = quantize_code(x[e], rho, pow2, qlo, qhi, mode, rng, (unsigned long long)(i0 + e));
  if constexpr (SIM) {
    float* yp = static_cast<float*>(yv) + i0;
#pragma unroll
    for (int e = 0; e < 8; ++e) q[e] = (q[e] * rho) / pow2;
    if (full) {
      *reinterpret_cast<float4*>(yp) = make_float4(q[0], q[1], q[2], q[3]);
      *reinterpret_cast<float4*>(yp + 4) = make_float4(q[4], q[5], q[6], q[7]);
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e)
        if (i0 + e < n) yp[e] = q[e];
    }
  } else {
    int8_t* yp = static_cast<int8_t*>(yv) + i0;
    if (full) {
      unsigned lo = 0, hi = 0;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        lo |= (unsigned)((int)q[e] & 0xff) << (8 * e);
        hi |= (unsigned)((int)q[4 + e] & 0xff) << (8 * e);
      }
      *reinterpret_cast<uint2*>(yp) = make_uint2(lo, hi);
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e)
        if (i0 + e < n) yp[e] = (int8_t)(int)q[e];
    }
  }
}

}  // namespace

hipError_t launch_quantize(bool src_f16, long n, const void* x, float rho, int beta, int sigma, int mode,
                           unsigned seed_lo, unsigned seed_hi, int8_t* y, hipStream_t st) {
  const float pow2 = __builtin_ldexpf(1.f, beta - sigma);
  // a signed type (sigma >= 1) clips symmetrically, an unsigned one (sigma == 0) to [0, 2^beta - 1]
  const float qhi = sigma == 0 ? (float)((1 << beta) - 1) : (float)((1 << (beta - 1)) - 1), qlo = sigma == 0 ? 0.f : -qhi;
  const unsigned grid = (unsigned)((n + 2047) / 2048);
  if (src_f16)
    hipLaunchKernelGGL((quantize_kernel<true, false>), dim3(grid), dim3(256), 0, st, n, x, rho, pow2, qlo, qhi, mode, seed_lo,
                       seed_hi, (void*)y);
  else
    hipLaunchKernelGGL((quantize_kernel<false, false>), dim3(grid), dim3(256), 0, st, n, x, rho, pow2, qlo, qhi, mode, seed_lo,
                       seed_hi, (void*)y);
  return hipGetLastError();
}

hipError_t launch_sim_quantize(long n, const float* x, float rho, int beta, int sigma, int mode, unsigned seed_lo,
                               unsigned seed_hi, float* y, hipStream_t st) {
  const float pow2 = __builtin_ldexpf(1.f, beta - sigma);
  // a signed type (sigma >= 1) clips symmetrically, an unsigned one (sigma == 0) to [0, 2^beta - 1]
  const float qhi = sigma == 0 ? (float)((1 << beta) - 1) : (float)((1 << (beta - 1)) - 1), qlo = sigma == 0 ? 0.f : -qhi;
  const unsigned grid = (unsigned)((n + 2047) / 2048);
  hipLaunchKernelGGL((quantize_kernel<false, true>), dim3(grid), dim3(256), 0, st, n, (const void*)x, rho, pow2, qlo, qhi, mode,
                     seed_lo, seed_hi, (void*)y);
  return hipGetLastError();
}

}  // namespace relay
