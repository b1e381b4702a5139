// Depthwise 3x3 conv2d, NHWC fp16, fp32 accumulation, fused scale/shift/relu epilogue
// (paper Section 4.1: the elementwise operators behind a contraction run in its kernel).
//
// Bandwidth-bound (4.5 FLOP/B at stride 1), so no MFMA.  Channels lie across lanes as 16-byte
// vectors of 8, every global access is a coalesced run along C.  A thread produces TW x TH
// outputs for its 8 channels from an input patch held in registers; the overlap between neighbouring threads' patches is served by the
// vector L1 / the XCD's L2, not by HBM.  The patch is fetched with raw buffer loads whose
// out-of-range offsets return zeros (no branches for the padding), all issued before the
// first use, and the multiply-adds take the fp16 operands directly (v_fma_mix_f32: fp16 x
// fp16 + fp32), with no conversion instructions.
// Workgroups are renumbered so that one XCD works through a contiguous range of rows: the
// rows two workgroups share are then fetched into one L2, not several.
#include "kernels.hpp"

namespace relay {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));

// acc += x.lo*w.lo (fp16 halves of 32-bit registers), fp32 accumulate
__device__ __forceinline__ void fma_mix_lo(float& acc, unsigned x, unsigned w) {
  asm("v_fma_mix_f32 %0, %1, %2, %0 op_sel:[0,0,0] op_sel_hi:[1,1,0]" : "+v"(acc) : "v"(x), "v"(w));
}
__device__ __forceinline__ void fma_mix_hi(float& acc, unsigned x, unsigned w) {
  asm("v_fma_mix_f32 %0, %1, %2, %0 op_sel:[1,1,0] op_sel_hi:[1,1,0]" : "+v"(acc) : "v"(x), "v"(w));
}

__device__ __forceinline__ int xcd_order(int bid, int nb) {
  const int xcd = bid & 7, idx = bid >> 3;
  const int per = nb >> 3, rem = nb & 7;
  return xcd < rem ? xcd * (per + 1) + idx : rem * (per + 1) + (xcd - rem) * per + idx;
}

typedef unsigned uintx4 __attribute__((ext_vector_type(4)));

// 16-byte load through a raw buffer descriptor: an offset at or beyond num_records reads zeros,
// which is how padding taps are handled without branches.
__device__ __forceinline__ uint4 buffer_load16(__amdgpu_buffer_rsrc_t rsrc, unsigned voff) {
  const uintx4 v = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)voff, 0, 0);
  return make_uint4(v[0], v[1], v[2], v[3]);
}

template <int STRIDE, int TH, int TW>
__global__ __launch_bounds__(256) void dwconv3x3_f16_kernel(const ConvArgs a) {
  constexpr int IH = (TH - 1) * STRIDE + 3, IW = (TW - 1) * STRIDE + 3;
  constexpr unsigned kOob = 0x80000000u;
  const int cvecs = a.C >> 3;
  const int tiles_w = (a.Wo + TW - 1) / TW, tiles_h = (a.Ho + TH - 1) / TH;
  const unsigned total = (unsigned)(a.N * tiles_h * tiles_w * cvecs);  // < 2^31: checked by the launcher
  unsigned idx = (unsigned)xcd_order(blockIdx.x, gridDim.x) * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int cv = (int)(idx % (unsigned)cvecs);
  idx /= (unsigned)cvecs;
  const int tw = (int)(idx % (unsigned)tiles_w);
  idx /= (unsigned)tiles_w;
  const int th = (int)(idx % (unsigned)tiles_h);
  const int n = (int)(idx / (unsigned)tiles_h);
  const int c0 = cv * 8;
  const int p0 = th * TH, q0 = tw * TW;
  const int ih0 = p0 * STRIDE - a.ph, iw0 = q0 * STRIDE - a.pw;

  const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<void*>(a.x), 0, (int)((unsigned)a.N * a.H * a.W * a.C * 2u), 0x00020000);
  const int pix_bytes = a.C * 2;
  const unsigned base = (unsigned)(((n * a.H + ih0) * a.W + iw0) * pix_bytes + c0 * 2);  // tap (0,0)

  // issue every load of the patch before the first use; a tap outside the image gets the
  // out-of-range marker as its offset
  bool cok[IW];
#pragma unroll
  for (int s = 0; s < IW; ++s) cok[s] = (unsigned)(iw0 + s) < (unsigned)a.W;
  uint4 xv[IH][IW];
#pragma unroll
  for (int r = 0; r < IH; ++r) {
    const bool rok = (unsigned)(ih0 + r) < (unsigned)a.H;
    const unsigned rbase = base + (unsigned)(r * a.W * pix_bytes);
#pragma unroll
    for (int s = 0; s < IW; ++s)
      xv[r][s] = buffer_load16(rs, (rok && cok[s]) ? rbase + (unsigned)(s * pix_bytes) : kOob);
  }
  const _Float16* w = static_cast<const _Float16*>(a.w) + c0;  // [r][s][c]
  uint4 wv[9];
#pragma unroll
  for (int t = 0; t < 9; ++t) wv[t] = *reinterpret_cast<const uint4*>(w + (long)t * a.C);
  float mul[8], add[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const float sc = (a.flags & F_BN) ? a.scale[c0 + e] : 1.f;
    const float sf = (a.flags & F_BN) ? a.shift[c0 + e] : 0.f;
    const float b = (a.flags & F_BIAS) ? a.bias[c0 + e] : 0.f;
    mul[e] = sc;
    add[e] = b * sc + sf;  // (acc + b)*sc + sf
  }
  float acc[TH][TW][8];
#pragma unroll
  for (int i = 0; i < TH; ++i)
#pragma unroll
    for (int j = 0; j < TW; ++j)
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[i][j][e] = 0.f;

#pragma unroll
  for (int fr = 0; fr < 3; ++fr)
#pragma unroll
    for (int fs = 0; fs < 3; ++fs) {
      const uint4 ww = wv[fr * 3 + fs];
      const unsigned wr[4] = {ww.x, ww.y, ww.z, ww.w};
#pragma unroll
      for (int i = 0; i < TH; ++i)
#pragma unroll
        for (int j = 0; j < TW; ++j) {
          const uint4 xx = xv[i * STRIDE + fr][j * STRIDE + fs];
          const unsigned xr[4] = {xx.x, xx.y, xx.z, xx.w};
#pragma unroll
          for (int h = 0; h < 4; ++h) {
            fma_mix_lo(acc[i][j][2 * h], xr[h], wr[h]);
            fma_mix_hi(acc[i][j][2 * h + 1], xr[h], wr[h]);
          }
        }
    }

  const float lo = (a.flags & F_RELU) ? 0.f : -__builtin_inff();  // relu as a max with a uniform bound
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
      for (int e = 0; e < 8; ++e) o[e] = (_Float16)fmaxf(acc[i][j][e] * mul[e] + add[e], lo);
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

// 2x4 (stride 1) and 2x2 (stride 2) outputs per thread: measured faster than smaller patches
// on every MobileNet layer, including the 7x7 ones.
hipError_t launch_dwconv_f16(const ConvArgs& a, hipStream_t st) {
  if (a.sh == 1) return launch_dw<1, 2, 4>(a, st);
  return launch_dw<2, 2, 2>(a, st);
}

}  // namespace relay
