// Internal interface between the C-ABI layer (api.cpp) and the gfx950 kernels.
// Launchers enqueue on the given stream and return the HIP status of the launch.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "fastdiv.hpp"

namespace relay {

enum : unsigned { F_BIAS = 1, F_BN = 2, F_RES = 4, F_RELU = 8 };
enum : int { ROUND_NEAREST = 0, ROUND_FLOOR = 1, ROUND_CEIL = 2, ROUND_STOCHASTIC = 3 };
// how the quantized epilogue scales the accumulator (paper Section 4.2: a scheme chooses its scaling)
//   QMODE_SHIFT   q = round(acc / 2^rshift)                                 (power-of-two scales)
//   QMODE_SCALED  q = round(acc * qmult[k] / 2^(31 + qshift[k])), ties up    (any scale, per output channel)
//   QMODE_ACC16   the accumulator is saturated to int16 first, then QMODE_SHIFT (16-bit accumulation scheme)
enum : int { QMODE_SHIFT = 0, QMODE_SCALED = 1, QMODE_ACC16 = 2 };

// Geometry and operands of one conv-like primitive function.
struct ConvArgs {
  const void* x;
  const void* w;
  void* y;
  const void* res;
  const float* bias;
  const float* scale;
  const float* shift;
  const int32_t* qbias;
  int N, H, W, C, K, R, S, sh, sw, ph, pw, Ho, Wo;
  // element strides of x along image, row and pixel (NHWC: H*W*C, W*C, C).  The row-packed
  // stem path views a [.., Wp, 4] tensor as 32- or 64-"channel" pixels that overlap: then
  // xs_w = 4 while C is the chunk length.
  int xs_n, xs_h, xs_w;
  // host-computed constants of the implicit-GEMM prologue
  float rcp_wo, rcp_ho;   // 1/Wo, 1/Ho
  unsigned tap_spread;    // bit r*S set for every filter row r (R*S <= 32)
  int param_vec;          // per-channel constants are 16-byte aligned and K % 8 == 0: vector loads
  int n_major;            // tile order: consecutive workgroups share an output-channel tile (else a pixel tile)
  FastDiv fd_wo, fd_howo;           // division by Wo and by Ho*Wo (tile decoding in the prologue)
  FastDiv fd_tiles_m, fd_tiles_n;   // ... by the tile counts of the launched kernel variant (set by its launcher)
  int M;        // N*Ho*Wo  (rows of the implicit GEMM)
  int Kred;     // R*S*C    (reduction length)
  int Kp;       // row pitch of the packed filters, elements
  int lshift, rshift;
  int round_mode;          // ROUND_* rule of the requantization acc / 2^rshift
  int round_add;           // what the deterministic rules add before the shift (0 when rshift == 0)
  int qmode;               // QMODE_* of the quantized epilogue
  int clip_lo, clip_hi;    // bounds of the code type: -127 .. 127 (signed), 0 .. 255 (unsigned)
  const int32_t* qmult;    // QMODE_SCALED: per-channel multiplier [K] and shift [K]
  const int32_t* qshift;
  unsigned seed_lo, seed_hi;  // key of the stochastic rounding draws
  unsigned flags;
  // Output channel segments (parallel convolution combination and concatenation views, paper
  // Section 4.4): channel ch in [seg_end[i-1], seg_end[i]) of output pixel m is stored at
  // seg_y[i] + m*seg_ld[i] + (ch - seg_end[i-1]) elements; boundaries are multiples of 8.
  // nseg == 0: the plain tensor y with pixel pitch K.  Only the direct-to-LDS kernels read these.
  // Fused 3x3 / stride 2 / pad 1 max pool behind the conv (direct-to-LDS implicit GEMM, 256-pixel
  // tiles): a workgroup computes the 15 x 17 conv outputs under a 7 x 8 block of pooled outputs
  // and writes only those.  pool != 0: y is the pooled tensor [N][Ho/2][Wo/2][K].
  int pool;
  int pool_tiles_img, pool_tiles_row;   // 7 x 8 blocks per image and per row of blocks
  FastDiv fd_pool_img, fd_pool_row;
  // Reduction split over workgroups (direct-to-LDS implicit GEMM only): `split` workgroups share one
  // output tile, each reducing a contiguous run of chunks; they leave raw partial tiles in ws_part
  // ([tile][split][BM][BN] accumulator words) and count themselves in ws_cnt[tile]; the workgroup
  // that arrives last adds the partials in split order and runs the epilogue, then puts the
  // counter back to zero.  split <= 1: one workgroup per tile, nothing of this is touched.
  int split;
  // host-side only: upper bound on the workgroups a persistent kernel launches (0: one per workgroup
  // slot of the chip)
  int max_wgs;
  unsigned* ws_part;
  unsigned* ws_cnt;
  // seg_centre bit i: segment i is a 1x1 convolution embedded at the centre tap of the R x S window
  // (same stride, padding R/2, S/2 reads the same input pixel): its tiles reduce over that tap's
  // chunks only.  seg_norelu bit i: no relu for segment i although F_RELU is set.
  unsigned seg_centre, seg_norelu;
  int nseg;
  int seg_end[4];
  int seg_ld[4];
  void* seg_y[4];
};

// A depthwise 3x3 conv2d (pad 1, stride 1 or 2, NHWC fp16, filters [r][s][c]) with its fused tail and the 1x1
// conv2d that consumes it, as one kernel.  `pw` describes the 1x1 conv over the depthwise output
// (N x Ho x Wo pixels of C channels -> K channels; w, bias, scale, shift, flags, y; its x is unused).
struct DwPwArgs {
  const void* x;
  const void* dw_w;
  const float* dw_bias;
  const float* dw_scale;
  const float* dw_shift;
  unsigned dw_flags;
  int N, H, W, C, Ho, Wo, stride;
  int tiles_x, tiles_y, tiles_n;   // set by the launcher of the kernel variant,
  FastDiv fd_x, fd_y, fd_n;        // with the divisions by them
  ConvArgs pw;
};

// Row pitch (elements) of packed filters for a reduction of kred elements of esize bytes:
// whole 128-byte groups.
inline int packed_pitch(int kred, int esize) {
  const int per = 128 / esize;
  return (kred + per - 1) / per * per;
}

hipError_t launch_conv_direct_f32(const ConvArgs& a, hipStream_t st);
// tile < 0: pick by heuristic.
hipError_t launch_conv_igemm(const ConvArgs& a, bool is_i8, int tile, hipStream_t st);
int igemm_tile_count();
// Name, as a kernel trace prints it, of the instantiation launch_conv_igemm would use.
void igemm_kernel_name(const ConvArgs& a, bool is_i8, int tile, char* buf, size_t len);
// The direct-to-LDS variant (conv_igemm_dma.hip) and the shapes it takes.
bool igemm_dma_supported(const ConvArgs& a, bool is_i8);
hipError_t launch_conv_igemm_dma(const ConvArgs& a, bool is_i8, int tile, hipStream_t st);
// How many workgroups should share a tile's reduction for this layer (1: none; `want` > 0 forces a
// count, clamped to the number of chunks) and the bytes of zero-initialised device memory that takes:
// counters first (counter_bytes, a multiple of 256), then the partial tiles.
int igemm_dma_plan_split(const ConvArgs& a, bool is_i8, int tile, int want, size_t* counter_bytes, size_t* total_bytes);
// conv + 3x3/s2/p1 max pool in one launch (a.pool set up by fill_pool_args); false: shape not taken
bool igemm_dma_pool_supported(const ConvArgs& a, bool is_i8);
void fill_pool_args(ConvArgs& a);
hipError_t launch_conv_igemm_dma_pool(const ConvArgs& a, bool is_i8, hipStream_t st);
void igemm_dma_pool_kernel_name(bool is_i8, char* buf, size_t len);
int igemm_dma_tile_count();
void igemm_dma_kernel_name(const ConvArgs& a, bool is_i8, int tile, char* buf, size_t len);
// The 3x3 / stride 1 / pad 1 kernel that stages the activations once per channel chunk (conv_halo.hip).
bool conv_halo_supported(const ConvArgs& a, bool is_i8, int variant);
int conv_halo_pick(const ConvArgs& a, bool is_i8);  // variant, or -1: leave the layer to the implicit-GEMM kernel
int conv_halo_variant_count();
hipError_t launch_conv_halo(const ConvArgs& a, bool is_i8, int variant, hipStream_t st);
void conv_halo_kernel_name(const ConvArgs& a, bool is_i8, int variant, char* buf, size_t len);
// The persistent 3x3 / stride 1 / pad 1 kernel whose workgroups stream tile after tile (conv_stream.hip).
bool conv_stream_supported(const ConvArgs& a, bool is_i8, int variant);
int conv_stream_pick(const ConvArgs& a, bool is_i8);  // variant, or -1
int conv_stream_variant_count();
hipError_t launch_conv_stream(const ConvArgs& a, bool is_i8, int variant, hipStream_t st);
void conv_stream_kernel_name(const ConvArgs& a, bool is_i8, int variant, char* buf, size_t len);
// The first layer of an image network: 3 channels, 3x3 / stride 2 / pad 1, NCHW fp16 in, NHWC fp16 out (conv_first.hip).
bool conv_first_supported(const ConvArgs& a);
size_t conv_first_packed_bytes(int K);
hipError_t launch_pack_first_filters(const void* w_oihw, void* out, int K, hipStream_t st);
hipError_t launch_conv_first(const ConvArgs& a, hipStream_t st);   // a.w: the packed filters
hipError_t launch_dwconv_f16(const ConvArgs& a, hipStream_t st);
// The depthwise conv and its 1x1 conv in one launch (dwpw.hip).
int dwpw_variant_count();
bool dwpw_supported(const DwPwArgs& a, int variant);
int dwpw_pick(const DwPwArgs& a);   // variant expected to beat the two separate launches, or -1
int dwpw_any(const DwPwArgs& a);    // dwpw_pick, else any variant that takes the shape, or -1
hipError_t launch_dwpw(const DwPwArgs& a, int variant, hipStream_t st);
void dwpw_kernel_name(int variant, char* buf, size_t len);
hipError_t launch_dense(int m, int n, int k, bool is_f16, const void* x, const void* w, const float* bias,
                        int act, void* y, hipStream_t st);
hipError_t launch_pack_filters(const void* w_oihw, void* w_packed, int K, int Csrc, int C, int R, int S,
                               int Kp, int esize, hipStream_t st);
hipError_t launch_pack_dw_filters(const void* w_crs, void* w_rsc, int C, int RS, hipStream_t st);
hipError_t launch_maxpool(bool is_i8, int N, int C, int H, int W, int R, int stride, int pad, int Ho, int Wo,
                          const void* x, void* y, hipStream_t st);
// one unfused elementwise operator on an fp16 NHWC tensor of npix pixels x c channels (c % 8 == 0)
hipError_t launch_elementwise_f16(int op, long npix, int c, const void* x, const float* p0, const float* p1,
                                  const void* other, void* y, hipStream_t st);
// w_out[k][c][i] = w[k][c][i] * scale[axis_in ? c : k] for i < rs, product in fp64, one rounding to the filter type
hipError_t launch_fold_scale_axis(bool is_f16, int K, int C, int RS, bool axis_in, const void* w, const float* scale,
                                  void* w_out, hipStream_t st);
// out[k] = bias[k]*scale[k] + shift[k] (bias may be NULL: 0), fp64 arithmetic, fp32 result
hipError_t launch_fold_bias(int K, const float* bias, const float* scale, const float* shift, float* out,
                            hipStream_t st);
hipError_t launch_avgpool_f16(int N, int C, int HW, const void* x, void* y, hipStream_t st);
hipError_t launch_nchw_to_nhwc(int esize, int N, int C, int H, int W, int Cpad, const void* x, void* y,
                               hipStream_t st);
// [N,C<=4,H,W] -> zero-padded [N, H+2ph, Wp, 4]
hipError_t launch_pack_input_nhwc4(int esize, int N, int C, int H, int W, int ph, int pw, int Wp, const void* x,
                                   void* y, hipStream_t st);
// OIHW [K][Csrc<=4][R][S] -> [K][Kp] with reduction index r*ck + s*4 + c, zero elsewhere
// Q and simQ of the quantization flow (paper Section 4.2) on n elements; src_f16: x is fp16, else fp32
hipError_t launch_quantize(bool src_f16, long n, const void* x, float rho, int beta, int sigma, int mode,
                           unsigned seed_lo, unsigned seed_hi, int8_t* y, hipStream_t st);
hipError_t launch_sim_quantize(long n, const float* x, float rho, int beta, int sigma, int mode, unsigned seed_lo,
                               unsigned seed_hi, float* y, hipStream_t st);
// Calibration and realization of the quantization flow (realize.hip).  RealizedConv mirrors the
// public relay_realized_conv; `cell` is one zero-initialised-by-the-launcher word of device scratch.
struct RealizedConv {
  float rho_w;
  int out_rshift, residual_lshift, status;
};
enum : int { REALIZE_BAD_OUT_SHIFT = 1, REALIZE_BAD_RES_SHIFT = 2, REALIZE_BIAS_OVERFLOW = 4 };
hipError_t launch_pow2_range(int esize, long n, const void* x, float* rho, unsigned* cell, hipStream_t st);
hipError_t launch_realize_conv(int K, long per_k, const float* w, const float* bias, const float* scale,
                               const float* shift, float rho_x, float rho_y, float rho_r, int8_t* wq, int32_t* bias_q,
                               RealizedConv* out, float* folded, unsigned* cell, hipStream_t st);
// further quantization schemes (qschemes.hip): unsigned activations re-coded into a padded signed tensor,
// the zero-point term of the bias, the 16/32 direct convolution
hipError_t launch_recode_u8_padded(const void* x, void* y, int N, int H, int W, int C, int ph, int pw, hipStream_t st);
hipError_t launch_fold_zero_point(int K, long per_k, const int8_t* w, const int32_t* bias, int zero_point, int32_t* out, hipStream_t st);
hipError_t launch_qconv16_direct(const ConvArgs& a, hipStream_t st);
// measured ceilings (probe.hip): register-only matrix-instruction loop, streaming copy
hipError_t launch_probe_grid_barrier(int workgroups, int rounds, unsigned spin_limit, unsigned* cells, float* data, hipStream_t st);
hipError_t launch_probe_mfma(bool is_i8, int iters, int workgroups, unsigned* out, hipStream_t st);
hipError_t launch_probe_copy(const void* src, void* dst, long bytes, hipStream_t st);
hipError_t launch_pack_filters_rows(const void* w_oihw, void* w_packed, int K, int Csrc, int R, int S, int ck,
                                    int Kp, int esize, hipStream_t st);

}  // namespace relay
