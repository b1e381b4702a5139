// Further quantization schemes of the generic flow (paper Section 4.2: a scheme chooses signed or
// unsigned integer types; Section 5.4 lists a 16/32 scheme beside 8/32 and 8/16):
//   * unsigned 8-bit activations on the signed matrix cores: x_u = x_s + 128, so
//     conv(x_u, w) = conv(x_s, w) + 128 * sum(w[k]) provided the padding, which is the unsigned code 0,
//     becomes the signed code -128 -- the activations are re-coded into a physically padded signed
//     tensor (one pass) and the constant term is folded into the bias at compile time;
//   * 16/32: int16 activations and filters with int32 accumulation.  The matrix cores have no 16-bit
//     integer form, so this scheme runs on the vector ALUs: a direct convolution, one output pixel
//     x four channels per thread, 16-byte loads along the channel axis.
#include "rounding.hpp"

namespace relay {
namespace {

typedef short short8 __attribute__((ext_vector_type(8)));
typedef short short4v __attribute__((ext_vector_type(4)));

// [N][H][W][C] uint8 -> [N][H + 2ph][W + 2pw][C] int8, x - 128 inside, -128 (the unsigned zero) in the border
__global__ __launch_bounds__(256) void recode_u8_padded_kernel(const uint4* x, uint4* y, int N, int H, int W, int cv, int ph, int pw) {
  const int Hp = H + 2 * ph, Wp = W + 2 * pw;
  const long total = (long)N * Hp * Wp * cv;
  const long i = (long)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int v = (int)(i % cv);
  long t = i / cv;
  const int q = (int)(t % Wp);
  t /= Wp;
  const int p = (int)(t % Hp);
  const int n = (int)(t / Hp);
  const int ih = p - ph, iw = q - pw;
  uint4 o = make_uint4(0x80808080u, 0x80808080u, 0x80808080u, 0x80808080u);   // -128 in every byte
  if ((unsigned)ih < (unsigned)H && (unsigned)iw < (unsigned)W) {
    const uint4 u = x[((long)(n * H + ih) * W + iw) * cv + v];
    o = make_uint4(u.x ^ 0x80808080u, u.y ^ 0x80808080u, u.z ^ 0x80808080u, u.w ^ 0x80808080u);   // u - 128 = u xor 0x80 as int8
  }
  y[i] = o;
}

// out[k] = bias[k] + zero_point * sum_i w[k][i] (exact in 64 bits, must fit int32)
__global__ __launch_bounds__(256) void fold_zero_point_kernel(int K, long per_k, const int8_t* w, const int32_t* bias, int zp, int32_t* out) {
  const int k = blockIdx.x;
  long long s = 0;
  for (long i = threadIdx.x; i < per_k; i += 256) s += w[(long)k * per_k + i];
  __shared__ long long part[256];
  part[threadIdx.x] = s;
  __syncthreads();
  for (int off = 128; off > 0; off >>= 1) {
    if ((int)threadIdx.x < off) part[threadIdx.x] += part[threadIdx.x + off];
    __syncthreads();
  }
  if (threadIdx.x == 0) out[k] = (int32_t)((bias ? (long long)bias[k] : 0ll) + (long long)zp * part[0]);
}

// int16 x int16 -> int32 (wrapping), NHWC, packed filters [K][Kp]; thread = one pixel x 4 channels
__global__ __launch_bounds__(256) void qconv16_direct_kernel(const ConvArgs a) {
  const int kq = a.K >> 2;
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (long)a.M * kq) return;
  const int k0 = (int)(idx % kq) * 4;
  const int m = (int)(idx / kq);
  const int q = m % a.Wo, p = (m / a.Wo) % a.Ho, n = m / (a.Wo * a.Ho);
  const short* x = static_cast<const short*>(a.x);
  const short* w = static_cast<const short*>(a.w);
  unsigned acc[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) acc[j] = (a.flags & F_BIAS) ? (unsigned)a.qbias[k0 + j] : 0u;
  for (int r = 0; r < a.R; ++r) {
    const int ih = p * a.sh - a.ph + r;
    if ((unsigned)ih >= (unsigned)a.H) continue;
    for (int s = 0; s < a.S; ++s) {
      const int iw = q * a.sw - a.pw + s;
      if ((unsigned)iw >= (unsigned)a.W) continue;
      const short* xp = x + ((long)(n * a.H + ih) * a.W + iw) * a.C;
      const short* wp = w + (long)k0 * a.Kp + (r * a.S + s) * a.C;
      for (int c = 0; c < a.C; c += 8) {
        const short8 xv = *reinterpret_cast<const short8*>(xp + c);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const short8 wv = *reinterpret_cast<const short8*>(wp + (long)j * a.Kp + c);
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[j] += (unsigned)((int)xv[e] * (int)wv[e]);   // (unsigned: the sum wraps like int32 hardware)
        }
      }
    }
  }
  short4v out;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    int t = shift_round((int)acc[j], (unsigned)a.round_add, a.rshift);
    t = t < -32767 ? -32767 : (t > 32767 ? 32767 : t);
    if (a.flags & F_RELU) t = t > 0 ? t : 0;
    out[j] = (short)t;
  }
  *reinterpret_cast<short4v*>(static_cast<short*>(a.y) + (long)m * a.K + k0) = out;
}

}  // namespace

hipError_t launch_recode_u8_padded(const void* x, void* y, int N, int H, int W, int C, int ph, int pw, hipStream_t st) {
  const long total = (long)N * (H + 2 * ph) * (W + 2 * pw) * (C / 16);
  hipLaunchKernelGGL(recode_u8_padded_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, static_cast<const uint4*>(x),
                     static_cast<uint4*>(y), N, H, W, C / 16, ph, pw);
  return hipGetLastError();
}

hipError_t launch_fold_zero_point(int K, long per_k, const int8_t* w, const int32_t* bias, int zero_point, int32_t* out, hipStream_t st) {
  hipLaunchKernelGGL(fold_zero_point_kernel, dim3(K), dim3(256), 0, st, K, per_k, w, bias, zero_point, out);
  return hipGetLastError();
}

hipError_t launch_qconv16_direct(const ConvArgs& a, hipStream_t st) {
  const long total = (long)a.M * (a.K / 4);
  hipLaunchKernelGGL(qconv16_direct_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, a);
  return hipGetLastError();
}

}  // namespace relay
