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
#include "dw_math.hpp"
#include "kernels.hpp"
#include "lds_dma.hpp"

namespace relay {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));

typedef unsigned uintx4 __attribute__((ext_vector_type(4)));

// 16-byte load through a raw buffer descriptor: an offset at or beyond num_records reads zeros,
// which is how padding taps are handled without branches.
__device__ __forceinline__ uint4 buffer_load16(__amdgpu_buffer_rsrc_t rsrc, unsigned voff) {
  const uintx4 v = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)voff, 0, 0);
  return make_uint4(v[0], v[1], v[2], v[3]);
}

template <int STRIDE, int TH, int TW>
__global__ __launch_bounds__(256) void dwconv3x3_f16_kernel(const ConvArgs a) {
  // all arguments as one batch of scalar loads with one wait (the compiler would load them where first used)
  asm volatile("" ::"s"(a.x), "s"(a.w), "s"(a.y), "s"(a.bias), "s"(a.scale), "s"(a.shift), "s"(a.N), "s"(a.H), "s"(a.W),
               "s"(a.C), "s"(a.Ho), "s"(a.Wo), "s"(a.sh), "s"(a.ph), "s"(a.pw), "s"(a.flags), "s"(a.fd_tiles_n.mul),
               "s"(a.fd_tiles_n.shift), "s"(a.fd_wo.mul), "s"(a.fd_wo.shift), "s"(a.fd_howo.mul), "s"(a.fd_howo.shift));
  constexpr int IH = (TH - 1) * STRIDE + 3, IW = (TW - 1) * STRIDE + 3;
  constexpr unsigned kOob = 0x80000000u;
  const int cvecs = a.C >> 3;
  const int tiles_w = (a.Wo + TW - 1) / TW, tiles_h = (a.Ho + TH - 1) / TH;
  const unsigned total = (unsigned)(a.N * tiles_h * tiles_w * cvecs);  // < 2^31: checked by the launcher
  unsigned idx = (unsigned)xcd_remap(blockIdx.x, gridDim.x) * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  // (divisions by multiply-high with the launcher's constants -- fd_tiles_n: cvecs, fd_wo: tiles_w, fd_howo:
  // tiles_h --: three software divisions per thread sat in front of the first load)
  const unsigned i1 = fast_div(idx, a.fd_tiles_n), i2 = fast_div(i1, a.fd_wo);
  const int cv = (int)(idx - i1 * (unsigned)cvecs);
  const int tw = (int)(i1 - i2 * (unsigned)tiles_w);
  const int n = (int)fast_div(i2, a.fd_howo);
  const int th = (int)i2 - n * tiles_h;
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
      *reinterpret_cast<uint4*>(y + ((long)p * a.Wo + q) * a.C) = scale_shift_narrow8(acc[i][j], mul, add, lo);
    }
  }
}

// ---- stride 1, wide images: the input patch of a workgroup goes through LDS.
//
// A workgroup of NT threads owns (2*MTH) x 28 output pixels x (8*CBV) channels of one image.
// Its input patch, (2*MTH + 2) x 30 pixels, is fetched once with global->LDS loads (lane i of
// an instruction writes 16 bytes at base + 16*i; the patch is stored as [pixel][channel
// vector], so one instruction moves 64/CBV whole pixels; taps in the padding get an
// out-of-range offset and arrive as zeros).  A thread then reads the 4 x 6 patch of its 2 x 4
// outputs from LDS instead of from the vector L1: the patch is requested from L2 about 1.3
// times per input element (the halo) instead of 3 times.  28 columns divide the 112-, 56- and
// 28-pixel rows of the workloads; other widths run with a ragged last tile.  Measured: the
// same kernel without its multiply-adds streams at 5.2 TB/s; the 9 fp32 FMAs per output
// element that the vector ALUs must issue are what is left of the gap to the HBM rate.
template <int CBV, int MTH, int NT>
__global__ __launch_bounds__(NT) void dwconv3x3_s1_lds_kernel(const ConvArgs a) {
  // all arguments as one batch of scalar loads with one wait (the compiler would load them where first used)
  asm volatile("" ::"s"(a.x), "s"(a.w), "s"(a.y), "s"(a.bias), "s"(a.scale), "s"(a.shift), "s"(a.N), "s"(a.H), "s"(a.W),
               "s"(a.C), "s"(a.Ho), "s"(a.Wo), "s"(a.sh), "s"(a.ph), "s"(a.pw), "s"(a.flags));
  constexpr int MTW = 7;                       // micro-tiles (2 x 4 outputs) across the workgroup tile
  constexpr int TH = 2 * MTH, TW = 4 * MTW;    // output tile
  constexpr int PH = TH + 2, PW = TW + 2;      // input patch
  constexpr int NV = PH * PW * CBV;            // 16-byte vectors of the patch
  constexpr int LOADS = (NV + NT - 1) / NT;    // load instructions per thread
  constexpr int NW = NT / 64;
  static_assert(MTH * MTW * CBV <= NT, "one thread per micro-tile and channel vector");
  __shared__ uint4 patch[LOADS * NT];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int cblocks = a.C / (8 * CBV);
  const int tiles_w = (a.Wo + TW - 1) / TW, tiles_h = (a.Ho + TH - 1) / TH;
  // (n, tile row, tile column, channel block), channel block fastest; divisions by multiply-high with the
  // launcher's constants (fd_tiles_n: cblocks, fd_wo: tiles_w, fd_howo: tiles_h)
  const unsigned t0 = (unsigned)xcd_remap(blockIdx.x, gridDim.x);
  const unsigned t1 = fast_div(t0, a.fd_tiles_n), t2 = fast_div(t1, a.fd_wo);
  const int cb = (int)(t0 - t1 * (unsigned)cblocks);
  const int tx = (int)(t1 - t2 * (unsigned)tiles_w);
  const int n = (int)fast_div(t2, a.fd_howo);
  const int ty = (int)t2 - n * tiles_h;
  const int oy0 = ty * TH, ox0 = tx * TW;
  const int iy0 = oy0 - a.ph, ix0 = ox0 - a.pw;  // input coordinates of patch pixel (0, 0)
  const int c0 = cb * 8 * CBV;

  const intx4 rs = make_rsrc(a.x, (unsigned)a.N * a.H * a.W * a.C * 2u);
  const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) uint4*)(&patch[0]);
#pragma unroll
  for (int j = 0; j < LOADS; ++j) {
    const int v = (j * NW + wave) * 64 + lane;  // vector index in the patch: pixel * CBV + channel vector
    const int pix = v / CBV, cv = v % CBV;
    const int py = pix / PW, px = pix - py * PW;
    const int iy = iy0 + py, ix = ix0 + px;
    const bool ok = v < NV && (unsigned)iy < (unsigned)a.H && (unsigned)ix < (unsigned)a.W;
    const unsigned off = ok ? (unsigned)((((n * a.H + iy) * a.W + ix) * a.C + c0 + cv * 8) * 2) : kOob;
    lds_dma16(rs, lds_base + (unsigned)((j * NW + wave) * 64) * 16u, off);
  }

  // this thread's micro-tile and channel vector; the filters and constants load while the patch is in flight
  const int cv = tid % CBV, mt = tid / CBV;
  const int mtx = mt % MTW, mty = mt / MTW;
  const bool active = mty < MTH;
  const int c = c0 + cv * 8;
  const _Float16* w = static_cast<const _Float16*>(a.w) + c;  // [r][s][c]
  uint4 wv[9];
#pragma unroll
  for (int k = 0; k < 9; ++k) wv[k] = *reinterpret_cast<const uint4*>(w + (long)k * a.C);
  float mul[8], add[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const float sc = (a.flags & F_BN) ? a.scale[c + e] : 1.f;
    const float sf = (a.flags & F_BN) ? a.shift[c + e] : 0.f;
    const float b = (a.flags & F_BIAS) ? a.bias[c + e] : 0.f;
    mul[e] = sc;
    add[e] = b * sc + sf;  // (acc + b)*sc + sf
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (!active) return;

  float acc[2][4][8];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[i][j][e] = 0.f;
  const uint4* pp = patch + ((mty * 2) * PW + mtx * 4) * CBV + cv;
#pragma unroll
  for (int r = 0; r < 4; ++r) {  // patch row: feeds output row i = r - fr for filter row fr
    uint4 xr[6];
#pragma unroll
    for (int q = 0; q < 6; ++q) xr[q] = pp[(r * PW + q) * CBV];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int fr = r - i;
      if (fr < 0 || fr > 2) continue;
#pragma unroll
      for (int fs = 0; fs < 3; ++fs) {
        const uint4 ww = wv[fr * 3 + fs];
        const unsigned wr[4] = {ww.x, ww.y, ww.z, ww.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const uint4 xx = xr[j + fs];
          const unsigned xh[4] = {xx.x, xx.y, xx.z, xx.w};
#pragma unroll
          for (int h = 0; h < 4; ++h) {
            fma_mix_lo(acc[i][j][2 * h], xh[h], wr[h]);
            fma_mix_hi(acc[i][j][2 * h + 1], xh[h], wr[h]);
          }
        }
      }
    }
  }

  const float lo = (a.flags & F_RELU) ? 0.f : -__builtin_inff();
  _Float16* y = static_cast<_Float16*>(a.y) + (long)n * a.Ho * a.Wo * a.C + c;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int p = oy0 + mty * 2 + i;
    if (p >= a.Ho) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int q = ox0 + mtx * 4 + j;
      if (q >= a.Wo) continue;
      *reinterpret_cast<uint4*>(y + ((long)p * a.Wo + q) * a.C) = scale_shift_narrow8(acc[i][j], mul, add, lo);
    }
  }
}

template <int CBV, int MTH, int NT>
hipError_t launch_dw_lds(const ConvArgs& a, hipStream_t st) {
  const long tiles = (long)a.N * ((a.Ho + 2 * MTH - 1) / (2 * MTH)) * ((a.Wo + 27) / 28) * (a.C / (8 * CBV));
  ConvArgs b = a;   // the kernel's index decoding divides by these three
  b.fd_tiles_n = make_fastdiv((uint32_t)(a.C / (8 * CBV)));
  b.fd_wo = make_fastdiv((uint32_t)((a.Wo + 27) / 28));
  b.fd_howo = make_fastdiv((uint32_t)((a.Ho + 2 * MTH - 1) / (2 * MTH)));
  hipLaunchKernelGGL((dwconv3x3_s1_lds_kernel<CBV, MTH, NT>), dim3((unsigned)tiles), dim3(NT), 0, st, b);
  return hipGetLastError();
}

template <int STRIDE, int TH, int TW>
hipError_t launch_dw(const ConvArgs& a, hipStream_t st) {
  const long total = (long)a.N * ((a.Ho + TH - 1) / TH) * ((a.Wo + TW - 1) / TW) * (a.C / 8);
  dim3 grid((unsigned)((total + 255) / 256)), block(256);
  ConvArgs b = a;   // the kernel's index decoding divides by these three
  b.fd_tiles_n = make_fastdiv((uint32_t)(a.C / 8));
  b.fd_wo = make_fastdiv((uint32_t)((a.Wo + TW - 1) / TW));
  b.fd_howo = make_fastdiv((uint32_t)((a.Ho + TH - 1) / TH));
  hipLaunchKernelGGL((dwconv3x3_f16_kernel<STRIDE, TH, TW>), grid, block, 0, st, b);
  return hipGetLastError();
}

}  // namespace

// 2x4 (stride 1) and 2x2 (stride 2) outputs per thread: measured faster than smaller patches
// on every MobileNet layer at batch 32, including the 7x7 ones.
hipError_t launch_dwconv_f16(const ConvArgs& a, hipStream_t st) {
  // rows of at least one 28-pixel tile and enough outputs to give every CU several workgroups: the LDS-staged
  // kernel (measured faster from 28 x 28 up at batch 32; small workgroups on the large images, where eight of
  // them share a CU and overlap their load, compute and store phases)
  const long vecs = (long)a.N * a.Ho * a.Wo * (a.C / 8);   // (pixel, 8-channel vector) outputs
  if (a.sh == 1 && a.sw == 1 && a.Wo >= 28 && a.Ho >= 8 && a.C % 32 == 0 && vecs >= 8 * 65536) {
    if (a.Wo >= 56) return launch_dw_lds<4, 4, 128>(a, st);
    return launch_dw_lds<4, 8, 256>(a, st);
  }
  // Few outputs (small batches, the deep layers): the large per-thread patches would leave most CUs without a
  // workgroup -- 14 x 14 x 512 at batch 1 is six workgroups of 2 x 4 patches -- and the layer's time is then the
  // latency of one thread's chain of loads, multiply-adds and stores; smaller patches spread it over the chip.
  if (a.sh == 1) {
    // (measured: 14 x 14 x 512 at batch 1, 12.5 k outputs, 6.0 -> 4.4 us with 1 x 1 patches; at batch 32, 401 k
    // outputs, 6.7 us with 2 x 4 patches against 12.2 us with 1 x 2)
    if (vecs >= 2 * 65536) return launch_dw<1, 2, 4>(a, st);
    if (vecs >= 65536) return launch_dw<1, 1, 2>(a, st);
    return launch_dw<1, 1, 1>(a, st);
  }
  if (vecs >= 65536) return launch_dw<2, 2, 2>(a, st);
  return launch_dw<2, 1, 1>(a, st);
}

}  // namespace relay
