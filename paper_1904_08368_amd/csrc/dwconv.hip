// Depthwise 3x3 conv2d, NHWC fp16, fp32 accumulation, fused scale/shift/relu epilogue
// (paper Section 4.1: the elementwise operators behind a contraction run in its kernel).
//
// Bandwidth-bound (4.5 FLOP/B at stride 1), so no MFMA: channels lie across lanes as
// 16-byte vectors of 8, every global access is a coalesced run along C, and each thread
// keeps a TH x TW patch of outputs in registers so that an input vector fetched once
// feeds every tap that needs it (the 3x3 windows of neighbouring outputs overlap).
#include "kernels.hpp"

namespace relay {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));

template <int STRIDE, int TH, int TW>
__global__ __launch_bounds__(256) void dwconv3x3_f16_kernel(const ConvArgs a) {
  constexpr int IH = (TH - 1) * STRIDE + 3, IW = (TW - 1) * STRIDE + 3;
  const int cvecs = a.C >> 3;
  const int tiles_w = (a.Wo + TW - 1) / TW, tiles_h = (a.Ho + TH - 1) / TH;
  const long total = (long)a.N * tiles_h * tiles_w * cvecs;
  long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int cv = (int)(idx % cvecs);
  idx /= cvecs;
  const int tw = (int)(idx % tiles_w);
  idx /= tiles_w;
  const int th = (int)(idx % tiles_h);
  const int n = (int)(idx / tiles_h);
  const int c0 = cv * 8;
  const int p0 = th * TH, q0 = tw * TW;
  const int ih0 = p0 * STRIDE - a.ph, iw0 = q0 * STRIDE - a.pw;

  const _Float16* x = static_cast<const _Float16*>(a.x) + (long)n * a.H * a.W * a.C + c0;
  const _Float16* w = static_cast<const _Float16*>(a.w) + c0;  // [r][s][c]
  half8 wv[9];
#pragma unroll
  for (int t = 0; t < 9; ++t) wv[t] = *reinterpret_cast<const half8*>(w + (long)t * a.C);

  float acc[TH][TW][8];
#pragma unroll
  for (int i = 0; i < TH; ++i)
#pragma unroll
    for (int j = 0; j < TW; ++j)
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[i][j][e] = 0.f;

#pragma unroll
  for (int r = 0; r < IH; ++r) {
    const int ih = ih0 + r;
    const bool rok = (unsigned)ih < (unsigned)a.H;
    half8 row[IW];
#pragma unroll
    for (int s = 0; s < IW; ++s) {
      const int iw = iw0 + s;
      const bool ok = rok && (unsigned)iw < (unsigned)a.W;
      half8 z;
#pragma unroll
      for (int e = 0; e < 8; ++e) z[e] = 0;
      row[s] = ok ? *reinterpret_cast<const half8*>(x + ((long)ih * a.W + iw) * a.C) : z;
    }
#pragma unroll
    for (int i = 0; i < TH; ++i) {
      const int fr = r - i * STRIDE;  // filter row this input row meets for output row i
      if (fr < 0 || fr > 2) continue;
#pragma unroll
      for (int j = 0; j < TW; ++j)
#pragma unroll
        for (int fs = 0; fs < 3; ++fs) {
          const half8 xv = row[j * STRIDE + fs];
          const half8 ww = wv[fr * 3 + fs];
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[i][j][e] = fmaf((float)xv[e], (float)ww[e], acc[i][j][e]);
        }
    }
  }

  float bi[8], sc[8], sf[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    bi[e] = (a.flags & F_BIAS) ? a.bias[c0 + e] : 0.f;
    sc[e] = (a.flags & F_BN) ? a.scale[c0 + e] : 1.f;
    sf[e] = (a.flags & F_BN) ? a.shift[c0 + e] : 0.f;
  }
  _Float16* y = static_cast<_Float16*>(a.y) + (long)n * a.Ho * a.Wo * a.C + c0;
#pragma unroll
  for (int i = 0; i < TH; ++i) {
    const int p = p0 + i;
    if (p >= a.Ho) continue;
#pragma unroll
    for (int j = 0; j < TW; ++j) {
      const int q = q0 + j;
      if (q >= a.Wo) continue;
      half8 o;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        float v = acc[i][j][e];
        if (a.flags & F_BIAS) v += bi[e];
        if (a.flags & F_BN) v = v * sc[e] + sf[e];
        if (a.flags & F_RELU) v = v > 0.f ? v : 0.f;
        o[e] = (_Float16)v;
      }
      *reinterpret_cast<half8*>(y + ((long)p * a.Wo + q) * a.C) = o;
    }
  }
}

template <int STRIDE, int TH, int TW>
hipError_t launch_dw(const ConvArgs& a, hipStream_t st) {
  const long total = (long)a.N * ((a.Ho + TH - 1) / TH) * ((a.Wo + TW - 1) / TW) * (a.C / 8);
  dim3 grid((unsigned)((total + 255) / 256)), block(256);
  hipLaunchKernelGGL((dwconv3x3_f16_kernel<STRIDE, TH, TW>), grid, block, 0, st, a);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_dwconv_f16(const ConvArgs& a, hipStream_t st) {
  if (a.sh == 1) return launch_dw<1, 2, 4>(a, st);
  return launch_dw<2, 2, 2>(a, st);
}

}  // namespace relay
