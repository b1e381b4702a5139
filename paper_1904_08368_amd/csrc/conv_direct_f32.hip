// Direct fp32 conv2d, NCHW / OIHW, with the fused float epilogue (paper Section 4.1).
// One thread per output element; a wave covers 64 consecutive q, so input reads are
// coalesced rows and filter reads are wave-uniform.  Meant for small fp32 layers, which
// are launch-latency bound; the contraction is a plain FMA chain in (c, r, s) order.
#include "kernels.hpp"

namespace relay {
namespace {

__global__ __launch_bounds__(256) void conv_direct_f32_kernel(const ConvArgs a) {
  const long total = (long)a.N * a.K * a.Ho * a.Wo;
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int q = (int)(idx % a.Wo);
  long t = idx / a.Wo;
  const int p = (int)(t % a.Ho);
  t /= a.Ho;
  const int k = (int)(t % a.K);
  const int n = (int)(t / a.K);
  const float* x = static_cast<const float*>(a.x) + (long)n * a.C * a.H * a.W;
  const float* w = static_cast<const float*>(a.w) + (long)k * a.C * a.R * a.S;
  const int ih0 = p * a.sh - a.ph, iw0 = q * a.sw - a.pw;
  float acc = 0.f;
  for (int c = 0; c < a.C; ++c)
    for (int r = 0; r < a.R; ++r) {
      const int ih = ih0 + r;
      if ((unsigned)ih >= (unsigned)a.H) continue;
      for (int s = 0; s < a.S; ++s) {
        const int iw = iw0 + s;
        if ((unsigned)iw >= (unsigned)a.W) continue;
        acc = fmaf(x[((long)c * a.H + ih) * a.W + iw], w[(c * a.R + r) * a.S + s], acc);
      }
    }
  if (a.flags & F_BIAS) acc += a.bias[k];
  if (a.flags & F_BN) acc = acc * a.scale[k] + a.shift[k];
  if (a.flags & F_RES) acc += static_cast<const float*>(a.res)[idx];
  if (a.flags & F_RELU) acc = acc > 0.f ? acc : 0.f;
  static_cast<float*>(a.y)[idx] = acc;
}

}  // namespace

hipError_t launch_conv_direct_f32(const ConvArgs& a, hipStream_t st) {
  const long total = (long)a.N * a.K * a.Ho * a.Wo;
  dim3 grid((unsigned)((total + 255) / 256)), block(256);
  hipLaunchKernelGGL(conv_direct_f32_kernel, grid, block, 0, st, a);
  return hipGetLastError();
}

}  // namespace relay
