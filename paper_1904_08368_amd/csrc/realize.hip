// Compile-time half of the quantization flow on the device (paper Section 4.2, "Calibrate" and
// "Realize"; the axis scale folding of Section 4.4 first): power-of-two ranges by the "no overflow"
// rule, and for one convolution the int8 filters, the int32 bias and the two shifts of the fused
// requantization.  Everything stays on the device and on the caller's stream; the few scalars a
// caller needs back (range of the filters, the shifts, a status word) are left in device memory.
//
// Scheme: beta = 8 bits, sigma = 1 (signed), every range rho a power of two; a tensor with range
// rho holds code * rho / 2^7, so one count of a conv's int32 accumulator is worth
// unit = rho_x * rho_w / 2^14.
#include "kernels.hpp"

namespace relay {
namespace {

// Smallest power of two that |v| <= holds for every v seen (2^-20 for a tensor of zeros): the bit
// patterns of non-negative floats order like unsigned integers, so the maximum is one atomic.
__device__ __forceinline__ float pow2_at_least(float max_abs) {
  if (!(max_abs > 0.f)) return 0x1p-20f;
  int e;
  const float m = frexpf(max_abs, &e);  // max_abs = m * 2^e, 0.5 <= m < 1
  return ldexpf(1.f, m == 0.5f ? e - 1 : e);
}

// log2 of a positive double if it is an integer, else `bad`
__device__ __forceinline__ int exact_log2(double v, int bad) {
  if (!(v > 0.0) || v > 1.0e300) return bad;
  int e;
  const double m = frexp(v, &e);
  return m == 0.5 ? e - 1 : bad;
}

__global__ void clear_word_kernel(unsigned* cell) { *cell = 0u; }

template <typename T>
__global__ __launch_bounds__(256) void abs_max_kernel(long n, const T* x, unsigned* cell) {
  const long i0 = (long)blockIdx.x * 256 + threadIdx.x;
  unsigned best = 0u;
  for (long i = i0; i < n; i += (long)gridDim.x * 256) {
    const float v = fabsf((float)x[i]);
    const unsigned b = __builtin_bit_cast(unsigned, v);
    if (v == v && b > best) best = b;   // (NaN never raises the range)
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const unsigned o = (unsigned)__shfl_xor((int)best, off);
    best = o > best ? o : best;
  }
  if ((threadIdx.x & 63) == 0 && best) atomicMax(cell, best);
}

__global__ void range_from_max_kernel(const unsigned* cell, float* rho) {
  *rho = pow2_at_least(__builtin_bit_cast(float, *cell));
}

// w'[k][c][i] = w[k][c][i] * scale[k] (exact product in fp64, one rounding to fp32) and its range
__global__ __launch_bounds__(256) void fold_and_max_kernel(long n, int per_k, const float* w, const float* scale,
                                                           float* folded, unsigned* cell) {
  const long i0 = (long)blockIdx.x * 256 + threadIdx.x;
  unsigned best = 0u;
  for (long i = i0; i < n; i += (long)gridDim.x * 256) {
    const float v = scale ? (float)((double)w[i] * (double)scale[i / per_k]) : w[i];
    folded[i] = v;
    const unsigned b = __builtin_bit_cast(unsigned, fabsf(v));
    if (v == v && b > best) best = b;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const unsigned o = (unsigned)__shfl_xor((int)best, off);
    best = o > best ? o : best;
  }
  if ((threadIdx.x & 63) == 0 && best) atomicMax(cell, best);
}

// one thread: the range of the folded filters, then the two shifts
//   s = log2(2^7 rho_y / (rho_x rho_w)),  l = log2(2^7 rho_r / (rho_x rho_w))
__global__ void realize_scalars_kernel(const unsigned* cell, float rho_x, float rho_y, float rho_r, RealizedConv* out) {
  const float rho_w = pow2_at_least(__builtin_bit_cast(float, *cell));
  const double unit = (double)rho_x * (double)rho_w / 16384.0;
  int status = 0;
  const int s = exact_log2((double)rho_y / 128.0 / unit, -1);
  if (s < 0 || s > 31) status |= REALIZE_BAD_OUT_SHIFT;
  int l = 0;
  if (rho_r > 0.f) {
    l = exact_log2((double)rho_r / 128.0 / unit, -1);
    if (l < 0 || l > 23) status |= REALIZE_BAD_RES_SHIFT;
  }
  out->rho_w = rho_w;
  out->out_rshift = s;
  out->residual_lshift = l;
  out->status = status;   // (the bias kernel, which runs after this one, may still add its bit)
}

// Q(w', rho_w, 8, 1) with rounding to nearest: the code is decided in fp32 in the order division,
// scaling by 2^7, floor(t + 1/2), clip to +-127 -- the order of the library's quantize operator
__global__ __launch_bounds__(256) void realize_filters_kernel(long n, const float* folded, const RealizedConv* out, int8_t* wq) {
  const long i = (long)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const float rho = out->rho_w;
  const float t = (folded[i] / rho) * 128.f;
  const float q = fminf(fmaxf(floorf(t + 0.5f), -127.f), 127.f);
  wq[i] = (int8_t)(int)q;
}

// bias_q[k] = floor((bias[k] * scale[k] + shift[k]) / unit + 1/2): the additive term of the float
// tail, (acc + bias) * scale + shift = acc * scale + (bias * scale + shift), in accumulator counts.
// fp64; product and sum are rounded one after the other (no fused multiply-add), the division by
// the power of two is exact.
__global__ __launch_bounds__(256) void realize_bias_kernel(int K, const float* bias, const float* scale, const float* shift,
                                                           float rho_x, RealizedConv* out, int32_t* bias_q) {
  const int k = blockIdx.x * 256 + threadIdx.x;
  if (k >= K) return;
  double add = bias ? (double)bias[k] : 0.0;
  if (scale) add = __dadd_rn(__dmul_rn(add, (double)scale[k]), (double)shift[k]);
  const double unit = (double)rho_x * (double)out->rho_w / 16384.0;
  const double b = floor(__dadd_rn(add / unit, 0.5));
  if (!(fabs(b) < 2147483648.0)) {
    atomicOr(&out->status, REALIZE_BIAS_OVERFLOW);
    bias_q[k] = 0;
  } else {
    bias_q[k] = (int32_t)b;
  }
}

unsigned grid_for(long n) {
  const long b = (n + 255) / 256;
  return (unsigned)(b < 1 ? 1 : (b > 4096 ? 4096 : b));
}

}  // namespace

hipError_t launch_pow2_range(int esize, long n, const void* x, float* rho, unsigned* cell, hipStream_t st) {
  hipLaunchKernelGGL(clear_word_kernel, dim3(1), dim3(1), 0, st, cell);
  if (esize == 2)
    hipLaunchKernelGGL((abs_max_kernel<_Float16>), dim3(grid_for(n)), dim3(256), 0, st, n, (const _Float16*)x, cell);
  else
    hipLaunchKernelGGL((abs_max_kernel<float>), dim3(grid_for(n)), dim3(256), 0, st, n, (const float*)x, cell);
  hipLaunchKernelGGL(range_from_max_kernel, dim3(1), dim3(1), 0, st, (const unsigned*)cell, rho);
  return hipGetLastError();
}

hipError_t launch_realize_conv(int K, long per_k, const float* w, const float* bias, const float* scale,
                               const float* shift, float rho_x, float rho_y, float rho_r, int8_t* wq, int32_t* bias_q,
                               RealizedConv* out, float* folded, unsigned* cell, hipStream_t st) {
  const long n = (long)K * per_k;
  hipLaunchKernelGGL(clear_word_kernel, dim3(1), dim3(1), 0, st, cell);
  hipLaunchKernelGGL(fold_and_max_kernel, dim3(grid_for(n)), dim3(256), 0, st, n, (int)per_k, w, scale, folded, cell);
  hipLaunchKernelGGL(realize_scalars_kernel, dim3(1), dim3(1), 0, st, (const unsigned*)cell, rho_x, rho_y, rho_r, out);
  hipLaunchKernelGGL(realize_filters_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, n, (const float*)folded,
                     (const RealizedConv*)out, wq);
  if (bias_q)
    hipLaunchKernelGGL(realize_bias_kernel, dim3((unsigned)((K + 255) / 256)), dim3(256), 0, st, K, bias, scale, shift, rho_x,
                       out, bias_q);
  return hipGetLastError();
}

}  // namespace relay
