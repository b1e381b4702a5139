// dense + bias + activation:  y[m,j] = sum_i x[m,i] * w[j,i] + b[j]   (one fused
// primitive function, paper Section 4.1).  At inference batch sizes this op only streams
// the weight matrix once (weight-bandwidth bound), so a wave owns one output unit j,
// its lanes stride along the reduction axis with 16-byte loads, and the same weight
// vector feeds MB rows of x before a cross-lane sum.
#include "kernels.hpp"

namespace relay {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));

template <bool IS_F16, int MB>
__global__ __launch_bounds__(256) void dense_kernel(int M, int N, int K, const void* xv, const void* wv,
                                                    const float* bias, int act, void* yv) {
  constexpr int VE = IS_F16 ? 8 : 4;
  const int lane = threadIdx.x & 63;
  const int j = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (j >= N) return;  // whole wave leaves together
  for (int m0 = 0; m0 < M; m0 += MB) {
    float acc[MB];
#pragma unroll
    for (int i = 0; i < MB; ++i) acc[i] = 0.f;
    for (int k0 = lane * VE; k0 < K; k0 += 64 * VE) {
      float wf[VE];
      if constexpr (IS_F16) {
        const half8 t = *reinterpret_cast<const half8*>(static_cast<const _Float16*>(wv) + (long)j * K + k0);
#pragma unroll
        for (int e = 0; e < VE; ++e) wf[e] = (float)t[e];
      } else {
        const float4 t = *reinterpret_cast<const float4*>(static_cast<const float*>(wv) + (long)j * K + k0);
        wf[0] = t.x; wf[1] = t.y; wf[2] = t.z; wf[3] = t.w;
      }
#pragma unroll
      for (int i = 0; i < MB; ++i) {
        const int m = m0 + i;
        if (m >= M) break;
        if constexpr (IS_F16) {
          const half8 t = *reinterpret_cast<const half8*>(static_cast<const _Float16*>(xv) + (long)m * K + k0);
#pragma unroll
          for (int e = 0; e < VE; ++e) acc[i] = fmaf((float)t[e], wf[e], acc[i]);
        } else {
          const float4 t = *reinterpret_cast<const float4*>(static_cast<const float*>(xv) + (long)m * K + k0);
          acc[i] = fmaf(t.x, wf[0], acc[i]);
          acc[i] = fmaf(t.y, wf[1], acc[i]);
          acc[i] = fmaf(t.z, wf[2], acc[i]);
          acc[i] = fmaf(t.w, wf[3], acc[i]);
        }
      }
    }
#pragma unroll
    for (int i = 0; i < MB; ++i) {
      float v = acc[i];
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
      const int m = m0 + i;
      if (lane == 0 && m < M) {
        if (bias) v += bias[j];
        if (act == 1) v = v > 0.f ? v : 0.f;
        if constexpr (IS_F16)
          static_cast<_Float16*>(yv)[(long)m * N + j] = (_Float16)v;
        else
          static_cast<float*>(yv)[(long)m * N + j] = v;
      }
    }
  }
}

}  // namespace

hipError_t launch_dense(int m, int n, int k, bool is_f16, const void* x, const void* w, const float* bias, int act,
                        void* y, hipStream_t st) {
  // a wave keeps MB rows of x against one weight row: 32 when the batch has that many, so the
  // weights are read once and one round of loads covers the whole reduction of a typical layer
  dim3 block(256), grid((unsigned)((n + 3) / 4));
  if (is_f16) {
    if (m > 8)
      hipLaunchKernelGGL((dense_kernel<true, 32>), grid, block, 0, st, m, n, k, x, w, bias, act, y);
    else
      hipLaunchKernelGGL((dense_kernel<true, 8>), grid, block, 0, st, m, n, k, x, w, bias, act, y);
  } else {
    hipLaunchKernelGGL((dense_kernel<false, 8>), grid, block, 0, st, m, n, k, x, w, bias, act, y);
  }
  return hipGetLastError();
}

}  // namespace relay
