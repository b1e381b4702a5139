// The first layer of an image network for gfx950: conv2d 3x3 / stride 2 / pad 1 on 3 input channels + bias +
// folded batch norm + relu as one fused primitive function (paper Section 4.1), read from the image as it
// arrives (NCHW fp16) and written as NHWC fp16 for the layers behind it.
//
// Why not the matrix cores: with 27 products per output the layer is bound by its tensors, not by arithmetic
// (MobileNet-v1 at batch 32: 9.6 MB in, 25.7 MB out against 0.7 GFLOP).  The implicit-GEMM route needs the
// image repacked as padded NHWC4 first -- a launch of its own that reads the image and writes 1.4 times its
// size -- and then moves every input element through the texture path four and a half times.  Here a thread
// owns two neighbouring output pixels of one row: per input channel and filter row it reads the four input
// columns under them as one 8-byte load (plus the one column to their left), coalesced along the row of the
// NCHW plane.  (Four pixels per thread halve the number of waves and leave the SIMDs unevenly loaded: 17.4
// against 16.5 us at batch 32; finished values staged through LDS for 1 KB stores changed nothing.)
//
// Arithmetic: v_dot2_f32_f16, two fp16 products added to an fp32 accumulator per lane and instruction.  The
// filter columns 1 and 2 of a (channel, row) are one such pair against the input columns (2q, 2q + 1), which
// is how they sit in the loaded words; the nine column-0 taps are paired among themselves (the last with a
// zero).  The fourteen filter pairs of every output channel are the same for all lanes: they are packed
// ahead of time as [channel / 4][pair][channel % 4] and come in through the scalar unit, 56 registers per
// group of four output channels, as the scalar operand of the dot products (as LDS broadcasts they cost the
// LDS port 16 clocks per 16-byte read and bound the kernel: 19.6 us for MobileNet-v1's layer at batch 32).
// Output channels go in passes of sixteen to bound the registers.
#include "dw_math.hpp"
#include "fastdiv.hpp"
#include "kernels.hpp"

namespace relay {
namespace {

typedef _Float16 half2v __attribute__((ext_vector_type(2)));
constexpr int kPairs = 14;   // 9 (column 1, column 2) pairs + ceil(9 / 2) pairs of column-0 taps
constexpr int kPix = 2;      // output pixels per thread
constexpr int kPass = 16;    // output channels per pass

__device__ __forceinline__ float dot2(unsigned x, unsigned w, float acc) {
  return __builtin_amdgcn_fdot2(__builtin_bit_cast(half2v, x), __builtin_bit_cast(half2v, w), acc, false);
}

__global__ __launch_bounds__(128) void conv_first_kernel(const ConvArgs a) {
  extern __shared__ uint4 lds[];
  float* cmul = reinterpret_cast<float*>(lds);                              // [K]
  float* cadd = cmul + a.K;                                                 // [K]
  // the packed filters, read through the scalar cache: the table is written before the launch and never by it
  typedef const unsigned __attribute__((address_space(4)))* const_words;
  const const_words wt = (const_words)(unsigned long)a.w;
  const int tid = threadIdx.x;
  // ---- this thread's kPix pixels: (n, p, q0 .. q0 + kPix - 1)
  const int wq = a.Wo / kPix;                                // threads per output row
  const unsigned t_raw = blockIdx.x * blockDim.x + tid, t_end = (unsigned)(a.N * a.Ho * wq);
  const bool live = t_raw < t_end;                           // (threads past the end load the last pixels again and store nothing)
  const unsigned t = live ? t_raw : t_end - 1;
  const unsigned row = fast_div(t, a.fd_howo);               // n * Ho + p  (the launch sets this divisor to wq,
  const int q0 = (int)(t - row * (unsigned)wq) * kPix;
  const int n = (int)fast_div(row, a.fd_wo);                 //  and this one to Ho)
  const int p = (int)row - n * a.Ho;

  // xb[cr][i]: input columns (2 (q0 + i), 2 (q0 + i) + 1) of (channel, row) cr; xl[cr]: columns (2 q0 - 2, 2 q0 - 1)
  unsigned xb[9][kPix], xl[9];
  const _Float16* x = static_cast<const _Float16*>(a.x);
#pragma unroll
  for (int c = 0; c < 3; ++c)
#pragma unroll
    for (int r = 0; r < 3; ++r) {
      const int ih = 2 * p - 1 + r;
      const bool ok = ih >= 0 && ih < a.H;
      const _Float16* src = x + (((long)n * 3 + c) * a.H + (ok ? ih : 0)) * a.W + 2 * q0;
      unsigned v[4] = {0u, 0u, 0u, 0u};
      unsigned l = 0u;
      if (ok) {
        if constexpr (kPix == 4) {
          const uint4 t4 = *reinterpret_cast<const uint4*>(src);
          v[0] = t4.x; v[1] = t4.y; v[2] = t4.z; v[3] = t4.w;
        } else {
          const uint2 t2 = *reinterpret_cast<const uint2*>(src);
          v[0] = t2.x; v[1] = t2.y;
        }
        if (q0 > 0) l = *reinterpret_cast<const unsigned*>(src - 2);
      }
#pragma unroll
      for (int i = 0; i < kPix; ++i) xb[c * 3 + r][i] = v[i];
      xl[c * 3 + r] = l;
    }
  // ---- the constants of the tail into LDS (behind the image loads above, so that both memory latencies pass together)
  for (int k = tid; k < a.K; k += blockDim.x) {
    const float sc = a.scale ? a.scale[k] : 1.f, sf = a.shift ? a.shift[k] : 0.f, bb = a.bias ? a.bias[k] : 0.f;
    cmul[k] = sc;
    cadd[k] = bb * sc + sf;   // (acc + b) * sc + sf
  }
  __syncthreads();

  // the column-0 tap of pixel i is input column 2 (q0 + i) - 1: the high half of the pair to its left
  unsigned xs[5][kPix];
#pragma unroll
  for (int i = 0; i < kPix; ++i)
#pragma unroll
    for (int j = 0; j < 5; ++j) {
      const unsigned lo = i ? xb[2 * j][i - 1] : xl[2 * j];
      const unsigned hi = 2 * j + 1 < 9 ? (i ? xb[2 * j + 1][i - 1] : xl[2 * j + 1]) : 0u;
      xs[j][i] = __builtin_amdgcn_perm(hi, lo, 0x07060302u);   // (lo >> 16) | (hi & 0xffff0000)
    }

  const float lo_bound = (a.flags & F_RELU) ? 0.f : -__builtin_inff();
  if (!live) return;
  _Float16* y = static_cast<_Float16*>(a.y) + (size_t)t * kPix * a.K;   // (thread t owns pixels t * kPix ... of the NHWC output)
  for (int kb = 0; kb < a.K; kb += kPass) {
    float acc[kPix][kPass];
#pragma unroll
    for (int i = 0; i < kPix; ++i)
#pragma unroll
      for (int k = 0; k < kPass; ++k) acc[i][k] = 0.f;
#pragma unroll
    for (int k4 = 0; k4 < kPass / 4; ++k4) {
      unsigned wk[kPairs][4];   // (uniform: scalar registers)
#pragma unroll
      for (int pair = 0; pair < kPairs; ++pair)
#pragma unroll
        for (int e = 0; e < 4; ++e) wk[pair][e] = wt[((kb >> 2) + k4) * (kPairs * 4) + pair * 4 + e];
#pragma unroll
      for (int pair = 0; pair < kPairs; ++pair)
#pragma unroll
        for (int i = 0; i < kPix; ++i) {
          const unsigned xv = pair < 9 ? xb[pair][i] : xs[pair - 9][i];
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[i][4 * k4 + e] = dot2(xv, wk[pair][e], acc[i][4 * k4 + e]);
        }
    }
    float mul[kPass], add[kPass];
#pragma unroll
    for (int k4 = 0; k4 < kPass / 4; ++k4) {
      const float4 m4 = *reinterpret_cast<const float4*>(cmul + kb + 4 * k4);
      const float4 a4 = *reinterpret_cast<const float4*>(cadd + kb + 4 * k4);
      mul[4 * k4] = m4.x; mul[4 * k4 + 1] = m4.y; mul[4 * k4 + 2] = m4.z; mul[4 * k4 + 3] = m4.w;
      add[4 * k4] = a4.x; add[4 * k4 + 1] = a4.y; add[4 * k4 + 2] = a4.z; add[4 * k4 + 3] = a4.w;
    }
#pragma unroll
    for (int i = 0; i < kPix; ++i)
#pragma unroll
      for (int h = 0; h < kPass / 8; ++h) {
        float a8[8], m8[8], s8[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          a8[e] = acc[i][8 * h + e];
          m8[e] = mul[8 * h + e];
          s8[e] = add[8 * h + e];
        }
        *reinterpret_cast<uint4*>(y + (size_t)i * a.K + kb + 8 * h) = scale_shift_narrow8(a8, m8, s8, lo_bound);
      }
  }
}

// [k][c][r][s] halves -> [k / 4][pair][k % 4] pairs of halves
__global__ void pack_first_filters_kernel(const unsigned short* w, unsigned* out, int K) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= K * kPairs) return;
  const int k = i / kPairs, pair = i - k * kPairs;
  unsigned lo, hi;
  if (pair < 9) {   // (c, r) = (pair / 3, pair % 3): columns 1 and 2
    lo = w[k * 27 + pair * 3 + 1];
    hi = w[k * 27 + pair * 3 + 2];
  } else {          // column 0 of (c, r) number 2 (pair - 9) and of the next one
    const int j = 2 * (pair - 9);
    lo = w[k * 27 + j * 3];
    hi = j + 1 < 9 ? w[k * 27 + (j + 1) * 3] : 0u;
  }
  out[(k >> 2) * (kPairs * 4) + pair * 4 + (k & 3)] = lo | (hi << 16);
}

}  // namespace

size_t conv_first_packed_bytes(int K) { return (size_t)K * kPairs * 4; }

hipError_t launch_pack_first_filters(const void* w_oihw, void* out, int K, hipStream_t st) {
  hipLaunchKernelGGL(pack_first_filters_kernel, dim3((unsigned)((K * kPairs + 255) / 256)), dim3(256), 0, st,
                     static_cast<const unsigned short*>(w_oihw), static_cast<unsigned*>(out), K);
  return hipGetLastError();
}

// 3 input channels, 3x3 / stride 2 / pad 1, NCHW fp16 in, NHWC fp16 out; whole passes of output channels,
// whole aligned runs of input columns under the kPix output pixels of a thread.
bool conv_first_supported(const ConvArgs& a) {
  return a.C == 3 && a.R == 3 && a.S == 3 && a.sh == 2 && a.sw == 2 && a.ph == 1 && a.pw == 1 && a.K % kPass == 0 &&
         a.K <= 128 && a.W % 8 == 0 && a.H % 2 == 0 && a.Wo == a.W / 2 && a.Ho == a.H / 2 && !(a.flags & F_RES) &&
         (long)a.N * a.Ho * a.Wo * a.K < (1L << 31) && (long)a.N * a.Ho < (1L << 31);
}

hipError_t launch_conv_first(const ConvArgs& a, hipStream_t st) {
  ConvArgs b = a;
  b.fd_howo = make_fastdiv((uint32_t)(a.Wo / kPix));   // thread index -> output row n * Ho + p
  b.fd_wo = make_fastdiv((uint32_t)a.Ho);              // output row -> image
  const long threads = (long)a.N * a.Ho * (a.Wo / kPix);
  const size_t lds_bytes = (size_t)a.K * 8;
  hipLaunchKernelGGL(conv_first_kernel, dim3((unsigned)((threads + 127) / 128)), dim3(128), lds_bytes, st, b);
  return hipGetLastError();
}

}  // namespace relay
