// Small kernels around the fused primitive functions: filter packing and the NCHW->NHWC
// conversion (compile-time layout alteration in the paper's terms, Section 5.3), and the
// two pools that chain ResNet / MobileNet layer shapes.
#include "kernels.hpp"

namespace relay {
namespace {

// OIHW [K][Csrc][R][S] -> [K][Kp] with reduction index (r, s, c), c < C, zero elsewhere.
template <typename T>
__global__ __launch_bounds__(256) void pack_filters_kernel(const T* w, T* out, int K, int Csrc, int C, int R, int S,
                                                           int Kp) {
  const long total = (long)K * Kp;
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int kk = (int)(idx % Kp);
  const int k = (int)(idx / Kp);
  T v = 0;
  if (kk < R * S * C) {
    const int tap = kk / C, c = kk - tap * C;
    const int r = tap / S, s = tap - r * S;
    if (c < Csrc) v = w[(((long)k * Csrc + c) * R + r) * S + s];
  }
  out[idx] = v;
}

// depthwise filters [C][RS] -> [RS][C]
__global__ __launch_bounds__(256) void pack_dw_kernel(const uint16_t* w, uint16_t* out, int C, int RS) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= C * RS) return;
  const int c = idx % C, t = idx / C;
  out[idx] = w[c * RS + t];
}

template <typename T>
__global__ __launch_bounds__(256) void nchw_to_nhwc_kernel(const T* x, T* y, int N, int C, int H, int W, int Cpad) {
  const long total = (long)N * H * W * Cpad;
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int c = (int)(idx % Cpad);
  long t = idx / Cpad;
  const int w_ = (int)(t % W);
  t /= W;
  const int h = (int)(t % H);
  const int n = (int)(t / H);
  y[idx] = c < C ? x[(((long)n * C + c) * H + h) * W + w_] : (T)0;
}

// [N][C<=4][H][W] -> [N][H+2ph][Wp][4], zeros in the border, in the slack columns and in the
// channels past C: one thread per output pixel, reads coalesced along w in each plane.
template <typename T, typename V4>
__global__ __launch_bounds__(256) void pack_input_nhwc4_kernel(const T* x, V4* y, int N, int C, int H, int W, int ph,
                                                               int pw, int Hp, int Wp) {
  // (32-bit index arithmetic: the padded tensor has fewer than 2^31 pixels, checked by the entry point)
  const unsigned total = (unsigned)N * Hp * Wp;
  const unsigned idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int wq = (int)(idx % (unsigned)Wp);
  const unsigned t = idx / (unsigned)Wp;
  const int hq = (int)(t % (unsigned)Hp);
  const int n = (int)(t / (unsigned)Hp);
  const int h = hq - ph, w_ = wq - pw;
  T v[4] = {0, 0, 0, 0};
  if ((unsigned)h < (unsigned)H && (unsigned)w_ < (unsigned)W) {
    for (int c = 0; c < C; ++c) v[c] = x[(((long)n * C + c) * H + h) * W + w_];
  }
  V4 o;
  o.x = v[0];
  o.y = v[1];
  o.z = v[2];
  o.w = v[3];
  y[idx] = o;
}

// OIHW [K][Csrc][R][S] -> [K][Kp], reduction index r*ck + s*4 + c (one filter row per chunk)
template <typename T>
__global__ __launch_bounds__(256) void pack_filters_rows_kernel(const T* w, T* out, int K, int Csrc, int R, int S,
                                                                int ck, int Kp) {
  const long total = (long)K * Kp;
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int kk = (int)(idx % Kp);
  const int k = (int)(idx / Kp);
  T v = 0;
  const int r = kk / ck, in_row = kk - r * ck;
  const int s = in_row >> 2, c = in_row & 3;
  if (r < R && s < S && c < Csrc) v = w[(((long)k * Csrc + c) * R + r) * S + s];
  out[idx] = v;
}

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef signed char char16 __attribute__((ext_vector_type(16)));

// max pool, NHWC, one 16-byte channel vector per thread; padding taps are skipped.
template <typename V, int VE>
__global__ __launch_bounds__(256) void maxpool_kernel(const V* x, V* y, int N, int CV, int H, int W, int R, int stride,
                                                      int pad, int Ho, int Wo) {
  const long total = (long)N * Ho * Wo * CV;
  long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int cv = (int)(idx % CV);
  long t = idx / CV;
  const int q = (int)(t % Wo);
  t /= Wo;
  const int p = (int)(t % Ho);
  const int n = (int)(t / Ho);
  V best;
  bool have = false;
  for (int r = 0; r < R; ++r) {
    const int ih = p * stride - pad + r;
    if ((unsigned)ih >= (unsigned)H) continue;
    for (int s = 0; s < R; ++s) {
      const int iw = q * stride - pad + s;
      if ((unsigned)iw >= (unsigned)W) continue;
      const V v = x[(((long)n * H + ih) * W + iw) * CV + cv];
      if (!have) {
        best = v;
        have = true;
      } else {
#pragma unroll
        for (int e = 0; e < VE; ++e) best[e] = v[e] > best[e] ? v[e] : best[e];
      }
    }
  }
  if (!have) {
#pragma unroll
    for (int e = 0; e < VE; ++e) best[e] = 0;
  }
  y[idx] = best;
}

// The same for a compile-time window R x R: every tap is loaded, with its coordinates clamped
// into the image.  A clamped tap repeats an element that the window already holds (the window
// of a valid output overlaps the image in both directions), so the maximum is unchanged, and
// with no branches all R*R loads are in flight at once.  Workgroups are renumbered so that an
// XCD works through a contiguous range of output rows: rows that two windows share are then
// fetched into one L2.
template <typename V, int VE, int R>
__global__ __launch_bounds__(256) void maxpool_fixed_kernel(const V* x, V* y, int N, int CV, int H, int W, int stride,
                                                            int pad, int Ho, int Wo) {
  const long total = (long)N * Ho * Wo * CV;
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int per = gridDim.x >> 3, rem = gridDim.x & 7;
  const long bid = xcd < rem ? (long)xcd * (per + 1) + slot : (long)rem * (per + 1) + (long)(xcd - rem) * per + slot;
  const long idx = bid * 256 + threadIdx.x;
  if (idx >= total) return;
  const int cv = (int)(idx % CV);
  long t = idx / CV;
  const int q = (int)(t % Wo);
  t /= Wo;
  const int p = (int)(t % Ho);
  const int n = (int)(t / Ho);
  V v[R][R];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int ih = min(max(p * stride - pad + r, 0), H - 1);
#pragma unroll
    for (int s = 0; s < R; ++s) {
      const int iw = min(max(q * stride - pad + s, 0), W - 1);
      v[r][s] = x[(((long)n * H + ih) * W + iw) * CV + cv];
    }
  }
  V best = v[0][0];
#pragma unroll
  for (int r = 0; r < R; ++r)
#pragma unroll
    for (int s = 0; s < R; ++s)
#pragma unroll
      for (int e = 0; e < VE; ++e) best[e] = v[r][s][e] > best[e] ? v[r][s][e] : best[e];
  y[idx] = best;
}

// global average pool, NHWC fp16 -> [N][C] fp16, fp32 sum.  One workgroup per (image, group
// of up to 256 channel vectors); the HW positions are split over 256/CVB thread groups whose
// partial sums meet in LDS.
__global__ __launch_bounds__(256) void avgpool_f16_kernel(const half8* x, half8* y, int N, int CV, int HW, int CVB) {
  __shared__ float part[256 * 8];
  const int groups = (CV + CVB - 1) / CVB;
  const int n = blockIdx.x / groups, g = blockIdx.x % groups;
  const int parts = 256 / CVB;
  const int cvl = threadIdx.x % CVB, pi = threadIdx.x / CVB;
  const int cv = g * CVB + cvl;
  float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  if (cv < CV && pi < parts)
    for (int i = pi; i < HW; i += parts) {
      const half8 v = x[((long)n * HW + i) * CV + cv];
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] += (float)v[e];
    }
#pragma unroll
  for (int e = 0; e < 8; ++e) part[threadIdx.x * 8 + e] = acc[e];
  __syncthreads();
  if (pi == 0 && cv < CV) {
    for (int p = 1; p < parts; ++p)
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] += part[(p * CVB + cvl) * 8 + e];
    half8 o;
    const float inv = 1.0f / (float)HW;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = (_Float16)(acc[e] * inv);
    y[(long)n * CV + cv] = o;
  }
}

inline unsigned blocks_for(long total) { return (unsigned)((total + 255) / 256); }

}  // namespace

hipError_t launch_pack_filters(const void* w, void* out, int K, int Csrc, int C, int R, int S, int Kp, int esize,
                               hipStream_t st) {
  const long total = (long)K * Kp;
  dim3 grid(blocks_for(total)), block(256);
  if (esize == 1)
    hipLaunchKernelGGL((pack_filters_kernel<int8_t>), grid, block, 0, st, (const int8_t*)w, (int8_t*)out, K, Csrc, C,
                       R, S, Kp);
  else if (esize == 2)
    hipLaunchKernelGGL((pack_filters_kernel<uint16_t>), grid, block, 0, st, (const uint16_t*)w, (uint16_t*)out, K,
                       Csrc, C, R, S, Kp);
  else
    hipLaunchKernelGGL((pack_filters_kernel<uint32_t>), grid, block, 0, st, (const uint32_t*)w, (uint32_t*)out, K,
                       Csrc, C, R, S, Kp);
  return hipGetLastError();
}

hipError_t launch_pack_dw_filters(const void* w, void* out, int C, int RS, hipStream_t st) {
  hipLaunchKernelGGL(pack_dw_kernel, dim3(blocks_for((long)C * RS)), dim3(256), 0, st, (const uint16_t*)w,
                     (uint16_t*)out, C, RS);
  return hipGetLastError();
}

namespace {
typedef _Float16 half8v __attribute__((ext_vector_type(8)));

// One unfused elementwise operator over an fp16 NHWC tensor: what a framework without operator
// fusion launches behind a convolution (paper Section 5.2 measures fusion against exactly this).
// Every operator reads its input tensor and writes a new one, rounded to fp16.
//   OP 0 bias add: x + p0[c];  1 scale/shift: x*p0[c] + p1[c];  2 add: x + other;  3 relu
template <int OP>
__global__ __launch_bounds__(256) void elementwise_f16_kernel(long nvec, int cvecs, const half8v* x, const float* p0,
                                                              const float* p1, const half8v* other, half8v* y) {
  const long i = (long)blockIdx.x * 256 + threadIdx.x;
  if (i >= nvec) return;
  const int c = (int)(i % cvecs) * 8;
  const half8v v = x[i];
  half8v o;
  if constexpr (OP == 2) {
    const half8v r = other[i];
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = (_Float16)((float)v[e] + (float)r[e]);
  } else {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float t = (float)v[e];
      float u;
      if constexpr (OP == 0) u = t + p0[c + e];
      else if constexpr (OP == 1) u = t * p0[c + e] + p1[c + e];
      else u = t > 0.f ? t : 0.f;
      o[e] = (_Float16)u;
    }
  }
  y[i] = o;
}
}  // namespace

hipError_t launch_elementwise_f16(int op, long npix, int c, const void* x, const float* p0, const float* p1,
                                  const void* other, void* y, hipStream_t st) {
  const long nvec = npix * (c / 8);
  const dim3 grid((unsigned)((nvec + 255) / 256)), block(256);
  const half8v* xv = static_cast<const half8v*>(x);
  const half8v* ov = static_cast<const half8v*>(other);
  half8v* yv = static_cast<half8v*>(y);
  switch (op) {
    case 0: hipLaunchKernelGGL((elementwise_f16_kernel<0>), grid, block, 0, st, nvec, c / 8, xv, p0, p1, ov, yv); break;
    case 1: hipLaunchKernelGGL((elementwise_f16_kernel<1>), grid, block, 0, st, nvec, c / 8, xv, p0, p1, ov, yv); break;
    case 2: hipLaunchKernelGGL((elementwise_f16_kernel<2>), grid, block, 0, st, nvec, c / 8, xv, p0, p1, ov, yv); break;
    default: hipLaunchKernelGGL((elementwise_f16_kernel<3>), grid, block, 0, st, nvec, c / 8, xv, p0, p1, ov, yv); break;
  }
  return hipGetLastError();
}

namespace {
// Axis scale folding (paper Section 4.4): the per-channel factor next to a convolution is
// multiplied into the OIHW filters once, ahead of time.  The product of a filter value and an
// fp32 factor is exact in fp64, so the result is rounded exactly once, to the filter type.
template <typename T>
__global__ __launch_bounds__(256) void fold_scale_axis_kernel(long n, int C, int RS, bool axis_in, const T* w,
                                                              const float* scale, T* out) {
  const long i = (long)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const long kc = i / RS;  // k*C + c
  const int ch = axis_in ? (int)(kc % C) : (int)(kc / C);
  out[i] = (T)((double)w[i] * (double)scale[ch]);
}

__global__ __launch_bounds__(256) void fold_bias_kernel(int K, const float* bias, const float* scale,
                                                        const float* shift, float* out) {
  const int k = blockIdx.x * 256 + threadIdx.x;
  if (k >= K) return;
  const double b = bias ? (double)bias[k] : 0.0;
  out[k] = (float)__dadd_rn(__dmul_rn(b, (double)scale[k]), (double)shift[k]);  // product rounded, then the sum: no fma
}
}  // namespace

hipError_t launch_fold_scale_axis(bool is_f16, int K, int C, int RS, bool axis_in, const void* w, const float* scale,
                                  void* w_out, hipStream_t st) {
  const long n = (long)K * C * RS;
  if (is_f16)
    hipLaunchKernelGGL((fold_scale_axis_kernel<_Float16>), dim3(blocks_for(n)), dim3(256), 0, st, n, C, RS, axis_in,
                       (const _Float16*)w, scale, (_Float16*)w_out);
  else
    hipLaunchKernelGGL((fold_scale_axis_kernel<float>), dim3(blocks_for(n)), dim3(256), 0, st, n, C, RS, axis_in,
                       (const float*)w, scale, (float*)w_out);
  return hipGetLastError();
}

hipError_t launch_fold_bias(int K, const float* bias, const float* scale, const float* shift, float* out,
                            hipStream_t st) {
  hipLaunchKernelGGL(fold_bias_kernel, dim3(blocks_for(K)), dim3(256), 0, st, K, bias, scale, shift, out);
  return hipGetLastError();
}

hipError_t launch_maxpool(bool is_i8, int N, int C, int H, int W, int R, int stride, int pad, int Ho, int Wo,
                          const void* x, void* y, hipStream_t st) {
  if (R == 3 && !is_i8) {
    const int cv = C / 8;
    hipLaunchKernelGGL((maxpool_fixed_kernel<half8, 8, 3>), dim3(blocks_for((long)N * Ho * Wo * cv)), dim3(256), 0, st,
                       (const half8*)x, (half8*)y, N, cv, H, W, stride, pad, Ho, Wo);
  } else if (R == 3) {
    const int cv = C / 16;
    hipLaunchKernelGGL((maxpool_fixed_kernel<char16, 16, 3>), dim3(blocks_for((long)N * Ho * Wo * cv)), dim3(256), 0, st,
                       (const char16*)x, (char16*)y, N, cv, H, W, stride, pad, Ho, Wo);
  } else if (is_i8) {
    const int cv = C / 16;
    hipLaunchKernelGGL((maxpool_kernel<char16, 16>), dim3(blocks_for((long)N * Ho * Wo * cv)), dim3(256), 0, st,
                       (const char16*)x, (char16*)y, N, cv, H, W, R, stride, pad, Ho, Wo);
  } else {
    const int cv = C / 8;
    hipLaunchKernelGGL((maxpool_kernel<half8, 8>), dim3(blocks_for((long)N * Ho * Wo * cv)), dim3(256), 0, st,
                       (const half8*)x, (half8*)y, N, cv, H, W, R, stride, pad, Ho, Wo);
  }
  return hipGetLastError();
}

hipError_t launch_avgpool_f16(int N, int C, int HW, const void* x, void* y, hipStream_t st) {
  const int cv = C / 8;
  int cvb = 256;  // channel vectors per workgroup: the largest power of two that leaves >= 4 position groups
  while (cvb > 1 && (cvb > cv || 256 / cvb < 4)) cvb >>= 1;
  const int groups = (cv + cvb - 1) / cvb;
  hipLaunchKernelGGL(avgpool_f16_kernel, dim3((unsigned)(N * groups)), dim3(256), 0, st, (const half8*)x, (half8*)y,
                     N, cv, HW, cvb);
  return hipGetLastError();
}

hipError_t launch_pack_input_nhwc4(int esize, int N, int C, int H, int W, int ph, int pw, int Wp, const void* x,
                                   void* y, hipStream_t st) {
  const int Hp = H + 2 * ph;
  dim3 grid(blocks_for((long)N * Hp * Wp)), block(256);
  if (esize == 1)
    hipLaunchKernelGGL((pack_input_nhwc4_kernel<int8_t, char4>), grid, block, 0, st, (const int8_t*)x, (char4*)y, N,
                       C, H, W, ph, pw, Hp, Wp);
  else
    hipLaunchKernelGGL((pack_input_nhwc4_kernel<uint16_t, ushort4>), grid, block, 0, st, (const uint16_t*)x,
                       (ushort4*)y, N, C, H, W, ph, pw, Hp, Wp);
  return hipGetLastError();
}

hipError_t launch_pack_filters_rows(const void* w, void* out, int K, int Csrc, int R, int S, int ck, int Kp,
                                    int esize, hipStream_t st) {
  dim3 grid(blocks_for((long)K * Kp)), block(256);
  if (esize == 1)
    hipLaunchKernelGGL((pack_filters_rows_kernel<int8_t>), grid, block, 0, st, (const int8_t*)w, (int8_t*)out, K, Csrc,
                       R, S, ck, Kp);
  else
    hipLaunchKernelGGL((pack_filters_rows_kernel<uint16_t>), grid, block, 0, st, (const uint16_t*)w, (uint16_t*)out,
                       K, Csrc, R, S, ck, Kp);
  return hipGetLastError();
}

hipError_t launch_nchw_to_nhwc(int esize, int N, int C, int H, int W, int Cpad, const void* x, void* y,
                               hipStream_t st) {
  const long total = (long)N * H * W * Cpad;
  dim3 grid(blocks_for(total)), block(256);
  if (esize == 1)
    hipLaunchKernelGGL((nchw_to_nhwc_kernel<int8_t>), grid, block, 0, st, (const int8_t*)x, (int8_t*)y, N, C, H, W,
                       Cpad);
  else if (esize == 2)
    hipLaunchKernelGGL((nchw_to_nhwc_kernel<uint16_t>), grid, block, 0, st, (const uint16_t*)x, (uint16_t*)y, N, C, H,
                       W, Cpad);
  else
    hipLaunchKernelGGL((nchw_to_nhwc_kernel<uint32_t>), grid, block, 0, st, (const uint32_t*)x, (uint32_t*)y, N, C, H,
                       W, Cpad);
  return hipGetLastError();
}

}  // namespace relay
