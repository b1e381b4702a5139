/*
 * relay_fused.h -- C ABI of the fused primitive operators for MI355X (gfx950).
 *
 * A "fused primitive function" is what the paper's operator-fusion pass produces
 * (Section 4.1, "Extraction"): a contraction (conv2d, depthwise conv2d, dense) together
 * with the elementwise operators that post-dominate it, factored into one function whose
 * parameters are the group's free variables.  The compiled form of such a function uses
 * a fixed calling convention and preallocated inputs and outputs (Section 3.3,
 * "Backends"); the entry points below are that calling convention.
 *
 * Conventions common to every entry point
 *   - Every data pointer is a DEVICE pointer owned by the caller.  The library never
 *     allocates, frees or synchronises; work is enqueued on `hip_stream` (a hipStream_t
 *     passed as void*, NULL = the default stream) and the call returns at once.
 *   - Shapes are static and carried by value in the descriptor (the paper's lowered code
 *     is shape specific, Section 4.1 "Lowering").
 *   - Optional operands are NULL exactly when their flag bit is clear; a mismatch is
 *     RELAY_ERR_NULL.  Outputs must not alias inputs.
 *   - All argument checks run on the host before any HIP call.  A failed check returns
 *     a status and leaves a message for relay_last_error(); nothing is launched.
 *   - No C++ exception crosses this boundary.
 */
#ifndef RELAY_FUSED_H_
#define RELAY_FUSED_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  RELAY_OK = 0,
  RELAY_ERR_NULL = 1,        /* a required pointer is NULL, or an optional one disagrees with flags */
  RELAY_ERR_SHAPE = 2,       /* a non-positive extent, an empty output, padding >= kernel ... */
  RELAY_ERR_DTYPE = 3,       /* dtype not valid for this entry point */
  RELAY_ERR_UNSUPPORTED = 4, /* a valid request this library has no kernel for */
  RELAY_ERR_ALIGN = 5,       /* pointer or channel count not aligned for vector access */
  RELAY_ERR_WORKSPACE = 6,   /* workspace smaller than relay_workspace_bytes() asks */
  RELAY_ERR_DEVICE = 7       /* the HIP runtime refused the launch */
} relay_status;

typedef enum { RELAY_F32 = 0, RELAY_F16 = 1, RELAY_I8 = 2, RELAY_I16 = 3 /* the 16/32 scheme only */ } relay_dtype;
/* RELAY_NHWC4_PADDED: input of a first-layer conv with c <= 4 channels, stored [n][h + 2*pad_h]
 * [wp][4] with the zero border, wp - w - 2*pad_w slack columns and channels c..3 all zero
 * (relay_pack_input_nhwc4 writes it from NCHW; relay_nhwc4_padded_shape gives hp, wp).  The
 * filter row's taps and channels are then contiguous in memory and one filter row is one
 * reduction chunk of the MFMA kernel.  Output, residual: plain NHWC. */
typedef enum { RELAY_NCHW = 0, RELAY_NHWC = 1, RELAY_NHWC4_PADDED = 2 } relay_layout;

/* which elementwise operators are fused behind the contraction */
enum { RELAY_HAS_BIAS = 1, RELAY_HAS_BN = 2, RELAY_HAS_RESIDUAL = 4, RELAY_RELU = 8 };

/* Static type of a conv2d primitive function.  Dilation is 1.  Input [n,c,h,w], filters
 * [k,c,r,s] (depthwise: k == c, one [r,s] filter per channel).
 * Supported (dtype, layout): (F32, NCHW) direct kernel; (F16, NHWC) and (I8, NHWC)
 * implicit-GEMM MFMA kernels, which need c % 8 == 0 (F16) or c % 16 == 0 (I8): pad the
 * channel axis with zeros (relay_nchw_to_nhwc does); (F16 | I8, NHWC4_PADDED) for c <= 4. */
typedef struct {
  int32_t n, c, h, w;
  int32_t k, r, s;
  int32_t stride_h, stride_w, pad_h, pad_w;
  int32_t dtype;   /* relay_dtype  */
  int32_t layout;  /* relay_layout */
  uint32_t flags;  /* RELAY_HAS_* | RELAY_RELU */
} relay_conv2d_desc;

/* The shape relation of conv2d (paper Section 3.2, "Operators and Type Relations": an operator's
 * type carries a relation between the shapes of its arguments and of its result, enforced at every
 * call site; here it is evaluated on the static shapes of the descriptor):
 *   Ho = floor((h + 2*pad_h - r)/stride_h) + 1, Wo likewise.
 * d: host pointer; ho, wo: host pointers that receive the result.  Validates the geometry
 * (RELAY_ERR_NULL / _SHAPE / _DTYPE / _UNSUPPORTED as for the conv calls); touches no device. */
relay_status relay_conv2d_out_shape(const relay_conv2d_desc* d, int32_t* ho, int32_t* wo);

/* Lowered operators work on inputs and outputs that are allocated beforehand (paper Section 3.3,
 * "Backends"); the same holds for scratch memory, which the caller sizes with this query and owns.
 * Bytes of device scratch the conv entry points (relay_fused_conv2d_bias_bn_relu, relay_qconv2d_requant*)
 * can use for this descriptor (d, bytes: host pointers); 0 for most layers.  A layer with few output tiles and a long reduction
 * (the deep layers at small batch) is split along the reduction over several workgroups per tile, which
 * leave partial sums and a per-tile arrival count in the workspace; the last to arrive adds the partials
 * in a fixed order (results do not depend on timing; int8 stays bit-exact) and runs the fused tail.
 * Workspace contract of those entry points:
 *   workspace == NULL            the layer runs unsplit (always valid, slower for such layers)
 *   workspace != NULL            device memory, 256-byte aligned, workspace_bytes >= this size, else
 *                                RELAY_ERR_ALIGN / RELAY_ERR_WORKSPACE; its first bytes (the counts) must
 *                                be ZERO before the first call that uses it -- zero the whole buffer once;
 *                                every call leaves them zero again, so the buffer can be reused by later
 *                                calls in the same stream (or replayed from a graph) without clearing.
 * Calls that may overlap in time (different streams) need workspaces of their own. */
relay_status relay_workspace_bytes(const relay_conv2d_desc* d, size_t* bytes);

/* Size of the packed filter tensor, and the packing itself -- compile-time work in the
 * paper's terms (constant folding and layout alteration, Sections 3.3 and 5.3).
 * w_oihw: device, [k, c_src, r, s] in the descriptor's dtype with c_src <= d->c (channels
 * c_src..c-1 are filled with zeros).  w_packed: device, packed_bytes >= the size reported.
 * NHWC kernels read [k][r][s][c] with the reduction axis zero-padded to a whole number of
 * 64-byte chunks; the NCHW F32 kernel reads OIHW unchanged. */
relay_status relay_packed_weight_bytes(const relay_conv2d_desc* d, size_t* bytes);
relay_status relay_prepack_conv2d_weights(const relay_conv2d_desc* d, const void* w_oihw, int32_t c_src,
                                          void* w_packed, size_t packed_bytes, void* hip_stream);

/* Pre-padded 4-channel input of a RELAY_NHWC4_PADDED conv (F16 or I8): its extents, and the
 * conversion from NCHW [n,c,h,w] (descriptor geometry; an alteration of the operator's data layout
 * in the sense of paper Section 5.3, done per inference -- the filter packing above is the
 * compile-time one).  y: device, 16-byte aligned,
 * n*hp*wp*4 elements. */
relay_status relay_nhwc4_padded_shape(const relay_conv2d_desc* d, int32_t* hp, int32_t* wp);
relay_status relay_pack_input_nhwc4(const relay_conv2d_desc* d, const void* x_nchw, void* y, void* hip_stream);

/* conv2d -> [+bias[k]] -> [*bn_scale[k] + bn_shift[k]] -> [+residual] -> [relu] -> cast.
 * (paper Section 4.1; the order is this library's reading, the paper leaves it open.)
 * dtype F32 (NCHW) or F16 (NHWC, fp32 accumulation, output rounded to nearest even).
 * x [n,c,h,w]; residual and y [n,k,ho,wo] in the descriptor's layout and dtype;
 * bias / bn_scale / bn_shift: fp32 [k].  F16: x, w_packed, residual, y 16-byte aligned. */
relay_status relay_fused_conv2d_bias_bn_relu(const relay_conv2d_desc* d, const void* x, const void* w_packed,
                                             const float* bias, const float* bn_scale, const float* bn_shift,
                                             const void* residual, void* y, void* workspace,
                                             size_t workspace_bytes, void* hip_stream);

/* Quantized conv2d (paper Section 4.2, "Realize": Q = cast(clip(round(x * 2^-s)))
 * expanded into elementwise operators and fused behind the convolution):
 *   acc = conv2d(x_i8, w_i8) in int32  [+ bias[k]]  [+ residual_i8 * 2^residual_lshift]
 *   q   = out_rshift == 0 ? acc : (acc + 2^(out_rshift-1)) >> out_rshift   (arithmetic shift:
 *         round to nearest, ties toward +infinity)
 *   q   = min(max(q, -127), 127);  [relu: q = max(q, 0)];  y = (int8) q
 * d->dtype == RELAY_I8, layout NHWC, d->flags may hold HAS_BIAS | HAS_RESIDUAL | RELU.
 * 0 <= out_rshift <= 31, 0 <= residual_lshift <= 23.  Precondition: |acc| < 2^31 (wraps
 * silently otherwise).  x, w_packed 16-byte aligned; y, residual 8-byte aligned. */
relay_status relay_qconv2d_requant(const relay_conv2d_desc* d, const int8_t* x, const int8_t* w_packed,
                                   const int32_t* bias, const int8_t* residual, int32_t residual_lshift,
                                   int32_t out_rshift, int8_t* y, void* workspace, size_t workspace_bytes,
                                   void* hip_stream);

/* Rounding strategies of the quantization flow (paper Section 4.2 names nearest, floor, ceiling
 * and stochastic rounding as choices of a quantization scheme). */
typedef enum {
  RELAY_ROUND_NEAREST = 0,    /* ties toward +infinity: floor(t + 1/2) */
  RELAY_ROUND_FLOOR = 1,
  RELAY_ROUND_CEIL = 2,
  RELAY_ROUND_STOCHASTIC = 3  /* up with probability frac(t) */
} relay_round_mode;

/* relay_qconv2d_requant with a rounding strategy for acc / 2^out_rshift (paper Section 4.2: a
 * quantization scheme chooses its rounding):
 *   nearest: (acc + 2^(s-1)) >> s;  floor: acc >> s;  ceiling: (acc + 2^s - 1) >> s;
 *   stochastic: (acc + u) >> s with u = the low s bits of the element's random word.
 * Random words come from Philox-4x32-10 (Salmon et al., SC'11), a counter-based generator:
 * output element e = ((n*ho + p)*wo + q)*k + channel (its NHWC position) takes word e mod 4 of
 * the block with counter (e div 4 low word, high word, 0, 0) and key (seed low word, seed high
 * word), so a result depends on (seed, position) only, not on the launch shape.
 * Precondition as for relay_qconv2d_requant: |acc| < 2^31 (bias and residual included); the rounding
 * addend is never added to acc in 32 bits, so every mode is exact for all 0 <= out_rshift <= 31.
 * Everything else as relay_qconv2d_requant, which is this call with RELAY_ROUND_NEAREST. */
relay_status relay_qconv2d_requant_rounding(const relay_conv2d_desc* d, const int8_t* x, const int8_t* w_packed,
                                            const int32_t* bias, const int8_t* residual, int32_t residual_lshift,
                                            int32_t out_rshift, int32_t round_mode, uint64_t seed, int8_t* y,
                                            void* workspace, size_t workspace_bytes, void* hip_stream);

/* Further quantization schemes (paper Section 4.2: a scheme chooses its integer types, signed or
 * unsigned, and the realized operator scales by "multiplication and rounding"; the accuracy table of
 * Section 5.4 lists m/n = 8/16 and 16/32 -- m-bit multiplies accumulated in n bits -- beside 8/32).
 * Each is relay_qconv2d_requant with another tail or other operand types; operands, alignment,
 * workspace and errors as there unless said otherwise.  This library's readings of what the paper
 * leaves open are stated with each call.
 *
 * relay_qconv2d_requant_scaled: a general (not power-of-two) scale per output channel,
 *     q = floor(acc * mult[k] / 2^(31 + rshift[k]) + 1/2)          (ties toward +infinity)
 *   mult, rshift: device int32 [k], 0 < mult[k] < 2^31, 0 <= rshift[k] <= 31 (not checked on the
 *   device; relay_quantize_multiplier produces such pairs).  The product is formed in 64 bits.
 * relay_quantize_multiplier: host helper, scale = mult / 2^31 * 2^-rshift with 2^30 <= mult < 2^31,
 *   mult rounded to nearest; 2^-32 < scale < 1, else RELAY_ERR_SHAPE.  mult, rshift: host pointers.
 * relay_qconv2d_requant_acc16: the 8/16 scheme.  The matrix cores accumulate in 32 bits; the scheme's
 *   16-bit accumulator is the exact sum (bias and residual included) saturated to [-32768, 32767]
 *   before the rounding shift -- equal to a 16-bit accumulation whenever that does not overflow,
 *   which is the scheme's precondition, and defined beyond it.
 * relay_qconv2d_requant_i16: the 16/32 scheme.  d->dtype == RELAY_I16, NHWC, c % 8 == 0, k % 4 == 0;
 *   x, y int16 [n,h,w,c] / [n,ho,wo,k]; w_packed from relay_prepack_conv2d_weights with the same
 *   descriptor; tail [+bias] -> round(acc / 2^out_rshift) -> clip +-32767 -> [relu].  Precondition:
 *   the sums fit int32 (they wrap otherwise).  Runs on the vector ALUs (no 16-bit integer matrix form).
 * relay_qconv2d_requant_u8: unsigned 8-bit activations (codes 0..255, zero padding = code 0) with
 *   signed 8-bit filters on the signed matrix cores: the activations are re-coded (x - 128) into a
 *   physically padded signed copy in `workspace` whose border holds -128, and the constant
 *   128 * sum(w[k]) is part of the bias.  d: the I8 NHWC descriptor of the convolution with
 *   RELAY_HAS_BIAS set and no residual, c % 16 == 0; bias_zp [k] = relay_fold_zero_point(w, bias, 128);
 *   out_unsigned 1: y holds uint8 codes clipped to [0, 255] (which contains the relu), 0: int8 codes
 *   clipped to +-127 [and relu].  workspace: device, 16-byte aligned, at least
 *   relay_qconv2d_u8_workspace_bytes(d), else RELAY_ERR_WORKSPACE.  Two launches.
 * relay_fold_zero_point: out[k] = bias[k] (NULL: 0) + zero_point * sum_i w[k][i] over the OIHW int8
 *   filters (per_k = c*r*s), exact; device pointers; compile-time work. */
relay_status relay_qconv2d_requant_scaled(const relay_conv2d_desc* d, const int8_t* x, const int8_t* w_packed,
                                          const int32_t* bias, const int8_t* residual, int32_t residual_lshift,
                                          const int32_t* mult, const int32_t* rshift, int8_t* y, void* workspace,
                                          size_t workspace_bytes, void* hip_stream);
relay_status relay_quantize_multiplier(double scale, int32_t* mult, int32_t* rshift);
relay_status relay_qconv2d_requant_acc16(const relay_conv2d_desc* d, const int8_t* x, const int8_t* w_packed,
                                         const int32_t* bias, const int8_t* residual, int32_t residual_lshift,
                                         int32_t out_rshift, int8_t* y, void* workspace, size_t workspace_bytes,
                                         void* hip_stream);
relay_status relay_qconv2d_requant_i16(const relay_conv2d_desc* d, const int16_t* x, const int16_t* w_packed,
                                       const int32_t* bias, int32_t out_rshift, int16_t* y, void* hip_stream);
relay_status relay_qconv2d_u8_workspace_bytes(const relay_conv2d_desc* d, size_t* bytes);
relay_status relay_fold_zero_point(int32_t k, int64_t per_k, const int8_t* w, const int32_t* bias, int32_t zero_point,
                                   int32_t* out, void* hip_stream);
relay_status relay_qconv2d_requant_u8(const relay_conv2d_desc* d, const uint8_t* x, const int8_t* w_packed,
                                      const int32_t* bias_zp, int32_t out_rshift, int32_t out_unsigned, void* y,
                                      void* workspace, size_t workspace_bytes, void* hip_stream);

/* The quantization operators themselves (paper Section 4.2), elementwise over n_elems values:
 *   code = clip(round(x / rho * 2^(beta - sigma)), qtype)
 *          qtype signed (sigma >= 1): [-(2^(beta-1) - 1), 2^(beta-1) - 1];  unsigned (sigma == 0): [0, 2^beta - 1]
 *          (the section lets a scheme choose between signed and unsigned integers)
 *   relay_quantize       ("Realize", Q):    y = (int8) code, or (uint8) code in the same bytes for
 *                                           sigma == 0            x: F32 or F16, 2 <= beta <= 8
 *   relay_sim_quantize   ("Annotate", simQ): y_f32 = code * rho / 2^(beta - sigma)   x: F32, 2 <= beta <= 24
 * beta = bits of the target type, sigma = bits that carry no magnitude (1 for a signed type, 0 for an unsigned one),
 * rho > 0 = the range mapped onto full scale (this library's reading of the three parameters).
 * The code is decided in fp32 in the order written: IEEE division, exact scaling by the power of
 * two, then the rounding rule (nearest = floor(t + 0.5f); stochastic = floor(t + w * 2^-24) with
 * w the top 24 bits of the element's random word, element index = position in x).
 * x and y 16-byte aligned (relay_quantize: y 8-byte); y must not alias x. */
relay_status relay_quantize(int64_t n_elems, int32_t src_dtype, const void* x, float rho, int32_t beta,
                            int32_t sigma, int32_t round_mode, uint64_t seed, int8_t* y, void* hip_stream);
relay_status relay_sim_quantize(int64_t n_elems, const float* x, float rho, int32_t beta, int32_t sigma,
                                int32_t round_mode, uint64_t seed, float* y, void* hip_stream);

/* Depthwise conv2d as a fused primitive function (paper Section 4.1, "Extraction": the contraction
 * with the elementwise operators that post-dominate it; MobileNet, one of the vision models of
 * Section 5.1, is built from such layers):
 *   y[n,c,p,q] = sum_{r,s} x[n,c,p*stride-pad+r,q*stride-pad+s] * w[c,r,s]
 *   -> [+bias[c]] -> [*bn_scale[c] + bn_shift[c]] -> [relu] -> cast to fp16 (nearest even).
 * d: k == c, 3x3, stride 1 or 2 (equal in both directions), F16, NHWC, c % 8 == 0, no residual;
 * fp32 accumulation.  x [n,h,w,c], y [n,ho,wo,c] device, 16-byte aligned, caller-owned; bias /
 * bn_scale / bn_shift fp32 [c] device or NULL with the flag clear.  w_rsc: filters repacked
 * [r][s][c] by relay_prepack_dwconv_weights from w_crs [c][r][s] (both device; compile-time work).
 * Errors: RELAY_ERR_SHAPE (k != c, input above 2^31-1 bytes), _UNSUPPORTED (window, stride,
 * residual, layout), _DTYPE, _ALIGN, _NULL, _DEVICE; nothing is launched on an error. */
relay_status relay_prepack_dwconv_weights(const relay_conv2d_desc* d, const void* w_crs, void* w_rsc,
                                          void* hip_stream);
relay_status relay_fused_dwconv_bias_relu(const relay_conv2d_desc* d, const void* x, const void* w_rsc,
                                          const float* bias, const float* bn_scale, const float* bn_shift,
                                          void* y, void* hip_stream);

/* The first layer of an image network as a fused primitive function (paper Section 4.1: conv2d with the
 * elementwise operators behind it; Section 5.2: the cost of every launch and of every tensor that goes
 * through memory), read from the image as it arrives:
 *   y[n,p,q,k] = sum_{c,r,s} x[n,c,2p-1+r,2q-1+s] * w[k,c,r,s] -> [+bias] -> [*bn_scale + bn_shift] -> [relu] -> fp16
 * with fp32 accumulation.  d: F16, layout RELAY_NCHW (the layout of x; y is NHWC), c == 3, 3x3, stride 2,
 * pad 1, k % 16 == 0, k <= 128, w % 8 == 0, h even, no residual.  x_nchw [n,3,h,w] and y_nhwc [n,h/2,w/2,k]
 * device, 16-byte aligned, caller-owned, distinct; bias / bn_scale / bn_shift fp32 [k] device or NULL with
 * the flag clear.  No layout conversion or padded copy of the image is needed in front of this call.
 * w_packed: the filters as relay_prepack_first_layer_weights writes them from w_oihw [k,3,3,3] fp16 (both
 * device; compile-time work; relay_first_layer_packed_weight_bytes bytes, 16-byte aligned): pairs of
 * filter taps per output channel, in the order the kernel's two-element dot products consume them.  The
 * kernel reads this table through the scalar cache: it must be complete before the launch and is
 * never written by it.
 * relay_conv2d_first_layer_supported: 1 where these calls take the descriptor, else 0 (and RELAY_OK).
 * Errors: RELAY_ERR_DTYPE, _UNSUPPORTED (layout, window, stride, padding, channel counts, sizes, residual,
 * aliasing), _SHAPE, _NULL, _ALIGN, _DEVICE; nothing is launched on an error. */
relay_status relay_conv2d_first_layer_supported(const relay_conv2d_desc* d, int32_t* supported);
relay_status relay_first_layer_packed_weight_bytes(const relay_conv2d_desc* d, size_t* bytes);
relay_status relay_prepack_first_layer_weights(const relay_conv2d_desc* d, const void* w_oihw, void* w_packed,
                                               void* hip_stream);
relay_status relay_fused_conv2d_first_layer(const relay_conv2d_desc* d, const void* x_nchw, const void* w_packed,
                                            const float* bias, const float* bn_scale, const float* bn_shift,
                                            void* y_nhwc, void* hip_stream);

/* A depthwise conv2d and the 1x1 conv2d that consumes it, each with its fused tail, as ONE launch
 * (paper Section 4.1: a primitive function is one kernel; Section 5.2: the cost of every extra launch and
 * every intermediate that goes through memory; MobileNet's separable block, Section 5.1):
 *   t = fp16( relay_fused_dwconv_bias_relu(dw, x, dw_w_rsc, dw_bias, dw_scale, dw_shift) )
 *   y[n,p,q,k'] = sum_c t[n,p,q,c] * pw_w[k',c] -> [+pw_bias] -> [*pw_scale + pw_shift] -> [relu] -> fp16
 * t never leaves the chip; both reductions run in the order of the two separate entry points, so the result
 * equals theirs bit for bit.  dw: as for relay_fused_dwconv_bias_relu, additionally padding 1 and
 * c % 32 == 0.  k: output channels of the 1x1 conv (a multiple of 8); pw_flags: RELAY_HAS_BIAS / _HAS_BN /
 * _RELU.  pw_w_packed: the 1x1 filters [k][c] packed by relay_prepack_conv2d_weights for a 1x1 / stride 1 /
 * F16 / NHWC descriptor of c input channels.  x [n,h,w,c], y [n,ho,wo,k] device, 16-byte aligned,
 * caller-owned, distinct.  Per-channel arrays fp32 device ([c] for dw_*, [k] for pw_*) or NULL with the
 * flag clear.  relay_set_conv_tile(300 + v) forces kernel variant v for the calling thread.
 * Errors: as relay_fused_dwconv_bias_relu, plus RELAY_ERR_UNSUPPORTED (padding, c % 32, residual flag, no
 * variant for the stride) and _SHAPE (k); nothing is launched on an error. */
relay_status relay_fused_dwconv_pwconv(const relay_conv2d_desc* dw, const void* x, const void* dw_w_rsc,
                                       const float* dw_bias, const float* dw_scale, const float* dw_shift,
                                       int32_t k, uint32_t pw_flags, const void* pw_w_packed,
                                       const float* pw_bias, const float* pw_scale, const float* pw_shift,
                                       void* y, void* hip_stream);

/* Whether the single launch above is expected to be faster than relay_fused_dwconv_bias_relu followed by
 * the 1x1 relay_fused_conv2d_bias_bn_relu (paper Section 4.1: fusion is a choice the compiler makes per
 * group of operators; Section 5.2 measures what it buys): *pays = 1 on the layers that stream from
 * memory (many pixels, at most 256 channels), 0 on the deep layers, where the single launch would have to
 * recompute the depthwise tile once per tile of output channels.  From measurements on MI355X; host-only,
 * nothing is launched.  dw, k as for relay_fused_dwconv_pwconv; same errors for shapes it does not take. */
relay_status relay_dwconv_pwconv_fusion_pays(const relay_conv2d_desc* dw, int32_t k, int32_t* pays);
/* Profiling aid (paper Section 4.1 "Lowering": the lowered code is specific to the shape): the name, as a
 * kernel trace prints it, of the variant relay_fused_dwconv_pwconv runs for this shape. */
relay_status relay_dwconv_pwconv_kernel_name(const relay_conv2d_desc* dw, int32_t k, char* buf, size_t len);

/* dense as a fused primitive function (paper Section 4.1: a contraction with its elementwise tail;
 * Section 3.3 "Backends": operators are lowered to dense linear algebra kernels; the classifier
 * layers of the vision models of Section 5.1):
 *   y[m,j] = sum_i x[m,i] * w[j,i]  [+ bias[j]]  [act: 0 none, 1 relu].
 * dtype F16 (fp32 accumulation, result rounded to nearest even; k % 8 == 0) or F32 (k % 4 == 0).
 * x [m,k], w [n,k] (one row per output unit; the orientation is this library's reading), y [m,n]:
 * device, row-major, caller-owned, x and w 16-byte aligned; bias fp32 [n] device or NULL.
 * Errors: RELAY_ERR_SHAPE (non-positive or above 2^31-1 elements), _DTYPE, _UNSUPPORTED (act),
 * _ALIGN, _NULL, _DEVICE.  y must not alias x or w. */
relay_status relay_fused_dense_bias_act(int32_t m, int32_t n, int32_t k, int32_t dtype, const void* x,
                                        const void* w, const float* bias, int32_t act, void* y,
                                        void* hip_stream);

/* Window operators that only chain the real layer shapes of the vision models of paper Section 5.1
 * (standard architectures; the fusion rule of Section 4.1 leaves them as groups of their own).
 * NHWC; F16 needs c % 8 == 0, I8 c % 16 == 0.  x, y: device, 16-byte aligned, caller-owned.
 *   relay_maxpool2d       y[n,p,q,c] = max over the r x r window at stride `stride`, padding `pad`
 *                         (padding never wins the maximum); F16 or I8
 *   relay_global_avgpool  y[n,c] = mean over the hw pixels of image n, fp32 sum, F16 */
relay_status relay_maxpool2d(int32_t dtype, int32_t n, int32_t c, int32_t h, int32_t w, int32_t r,
                             int32_t stride, int32_t pad, const void* x, void* y, void* hip_stream);
relay_status relay_global_avgpool(int32_t dtype, int32_t n, int32_t c, int32_t hw, const void* x, void* y,
                                  void* hip_stream);

/* A convolution primitive function with the 3x3 / stride 2 / pad 1 max pool that follows it run
 * as ONE launch: the conv output never reaches memory.  This carries the operator fusion of
 * paper Section 4.1 one operator past the elementwise tail (a window operator whose input tile
 * the workgroup already holds); the result equals relay_fused_conv2d_bias_bn_relu (or
 * relay_qconv2d_requant) followed by relay_maxpool2d(r=3, stride=2, pad=1) bit for bit, because
 * each conv output is finished and narrowed exactly as there before the maximum is taken.
 *   d          the CONVOLUTION (F16 or I8; NHWC or NHWC4_PADDED; flags without HAS_RESIDUAL;
 *              I8 also without HAS_BN), with conv output ho % 14 == 0, wo % 16 == 0, k % 8 == 0
 *   y_pooled   [n, ho/2, wo/2, k] NHWC in d->dtype; F16 16-byte, I8 8-byte aligned
 *   the other operands as in the unpooled calls; the quantized call rounds to nearest.
 * relay_conv2d_maxpool_fusable writes 1 if these calls take the descriptor, else 0 (the calls
 * themselves return RELAY_ERR_UNSUPPORTED and launch nothing).
 * relay_conv2d_maxpool_kernel_name: the kernel a trace shows for these calls (cf. relay_conv2d_kernel_name). */
relay_status relay_conv2d_maxpool_fusable(const relay_conv2d_desc* d, int32_t* fusable);
relay_status relay_conv2d_maxpool_kernel_name(const relay_conv2d_desc* d, char* buf, size_t len);
relay_status relay_fused_conv2d_bn_relu_maxpool(const relay_conv2d_desc* d, const void* x, const void* w_packed,
                                                const float* bias, const float* bn_scale, const float* bn_shift,
                                                void* y_pooled, void* hip_stream);
relay_status relay_qconv2d_requant_maxpool(const relay_conv2d_desc* d, const int8_t* x, const int8_t* w_packed,
                                           const int32_t* bias, int32_t out_rshift, int8_t* y_pooled,
                                           void* hip_stream);

/* One UNFUSED elementwise operator on an fp16 NHWC tensor [n_pixels, c] (c % 8 == 0): what runs
 * behind a convolution when operator fusion is switched off.  The paper measures fusion against
 * such a pipeline (Section 5.2); this entry point exists for that comparison and for checking
 * that the fused operators equal the unfused sequence.  Reads x, writes y (fp16, round to
 * nearest even); y may alias x.
 *   RELAY_EW_BIAS_ADD     y = x + p0[channel]
 *   RELAY_EW_SCALE_SHIFT  y = x * p0[channel] + p1[channel]
 *   RELAY_EW_ADD          y = x + other            (other: fp16, same shape)
 *   RELAY_EW_RELU         y = max(x, 0)
 * Operands an operator does not use must be NULL.  Tensors 16-byte aligned. */
typedef enum { RELAY_EW_BIAS_ADD = 0, RELAY_EW_SCALE_SHIFT = 1, RELAY_EW_ADD = 2, RELAY_EW_RELU = 3 } relay_elementwise_op;
relay_status relay_elementwise_f16(int32_t op, int64_t n_pixels, int32_t c, const void* x, const float* p0,
                                   const float* p1, const void* other, void* y, void* hip_stream);
/* Parallel convolution combination (paper Section 4.4, "Parallel convolution combination"):
 * several convolutions that read the same tensor with the same window, stride and padding and
 * carry the same elementwise tail run as ONE launch over their filters stacked along the
 * output-channel axis.  Each member's result is a channel range ("segment") of that launch and
 * is stored straight into the member's own tensor -- which may itself be a channel range of a
 * wider NHWC tensor, so a later concatenation along channels costs nothing -- and the input may
 * likewise be a channel range of a wider tensor.
 *   d            NHWC, F16; c = channels read per pixel, k = channels of all segments together;
 *                flags as for relay_fused_conv2d_bias_bn_relu, without RELAY_HAS_RESIDUAL
 *   x, x_ld      first channel read of pixel (0,0,0) (device); pixel p of the input starts at
 *                x + p*x_ld elements.  x_ld >= c, multiple of 8
 *   w_packed     the members' packed filters one after another (packing is row-per-output-channel,
 *                so the members' relay_prepack_conv2d_weights results are simply concatenated)
 *   bias, bn_scale, bn_shift   [k], the members' constants one after another; NULL iff flag clear
 *   nseg         1..4 segments; seg_channels[i] > 0, multiple of 8, summing to k (host array)
 *   seg_y[i]     where channel 0 of segment i of output pixel 0 goes (device pointers, host array);
 *   seg_ld[i]    output pixel m of segment i starts at seg_y[i] + m*seg_ld[i] elements;
 *                seg_ld[i] >= seg_channels[i], multiple of 8 (host array)
 * Output ranges must not overlap each other or the input (not checked beyond pointer equality).
 * RELAY_ERR_UNSUPPORTED for shapes outside the direct-to-LDS kernels (c % 32 != 0, r*s > 32).
 * All pointers 16-byte aligned.  Nothing is allocated; the call only enqueues on hip_stream. */
relay_status relay_fused_conv2d_combined(const relay_conv2d_desc* d, const void* x, int32_t x_ld,
                                         const void* w_packed, const float* bias, const float* bn_scale,
                                         const float* bn_shift, int32_t nseg, const int32_t* seg_channels,
                                         void* const* seg_y, const int32_t* seg_ld, void* hip_stream);

/* The quantized form of relay_fused_conv2d_combined (paper Section 4.4, "Parallel convolution
 * combination", on the realized int8 convolutions of Section 4.2): d->dtype == RELAY_I8, flags
 * HAS_BIAS | RELU; x int8 with x_ld a multiple of 16, c % 64 == 0; bias int32 [k] over all segments;
 * segments of int8 with seg_channels / seg_ld multiples of 8 and seg_y 8-byte aligned.  Scaling of the
 * tail: mult == rshift == NULL -> one power-of-two shift out_rshift for every member (as
 * relay_qconv2d_requant); else per output channel round(acc * mult[k] / 2^(31 + rshift[k])) as
 * relay_qconv2d_requant_scaled, so that every member keeps its own scale (device int32 [k] each).
 * Clip +-127, [relu].  Bit-equal to the members' separate launches. */
relay_status relay_qconv2d_combined(const relay_conv2d_desc* d, const int8_t* x, int32_t x_ld, const int8_t* w_packed,
                                    const int32_t* bias, const int32_t* mult, const int32_t* rshift, int32_t out_rshift,
                                    int32_t nseg, const int32_t* seg_channels, void* const* seg_y, const int32_t* seg_ld,
                                    void* hip_stream);

/* relay_fused_conv2d_combined (paper Section 4.4, "Parallel convolution combination") for members
 * whose windows and tails differ in two ways that occur in residual networks (a stride-2 3x3 convolution and the 1x1 shortcut convolution beside it
 * read the same tensor): a 1x1 convolution with the same stride and no padding reads, for every
 * output pixel, the input pixel under the CENTRE tap of an odd r x s window padded by (r/2, s/2),
 * so it is that window with zeros everywhere else; and one member may end in relu while another
 * does not.  Per segment (host arrays of nseg entries):
 *   seg_window[i]  RELAY_WINDOW_FULL: the descriptor's window.  RELAY_WINDOW_CENTRE: a 1x1
 *                  convolution; its filters sit at the centre tap of rows packed for the r x s
 *                  window (prepack the 1x1 filters embedded in zeros), and its tiles reduce over
 *                  that tap only, so the zeros cost nothing.  Such a segment begins at and holds
 *                  a multiple of 128 channels.
 *   seg_relu[i]    1: relu (d->flags must hold RELAY_RELU), 0: none.
 * Everything else as relay_fused_conv2d_combined. */
typedef enum { RELAY_WINDOW_FULL = 0, RELAY_WINDOW_CENTRE = 1 } relay_segment_window;
relay_status relay_fused_conv2d_combined_windows(const relay_conv2d_desc* d, const void* x, int32_t x_ld,
                                                 const void* w_packed, const float* bias, const float* bn_scale,
                                                 const float* bn_shift, int32_t nseg, const int32_t* seg_channels,
                                                 void* const* seg_y, const int32_t* seg_ld,
                                                 const int32_t* seg_window, const int32_t* seg_relu,
                                                 void* hip_stream);

/* Axis scale folding (paper Section 4.4, "Axis scale folding"): a multiplication by a
 * per-channel constant before or after a convolution is moved into the convolution's constant
 * filters ahead of time, leaving no multiplication in the operator's tail.
 *   relay_fold_scale_axis: w_out[k][c][r][s] = w[k][c][r][s] * scale[axis == RELAY_FOLD_OUT ? k : c]
 *     on OIHW filters (device, F16 or F32; rs = r*s), scale [k] resp. [c] fp32 (device).  The
 *     product is formed exactly (fp64) and rounded once to the filter type.  w_out may equal w.
 *   relay_fold_bias: out[k] = bias[k]*scale[k] + shift[k] (bias NULL: 0), fp64 arithmetic rounded
 *     to fp32 -- the bias that replaces "add bias, scale, shift" once scale sits in the filters. */
typedef enum { RELAY_FOLD_OUT = 0, RELAY_FOLD_IN = 1 } relay_fold_axis;
relay_status relay_fold_scale_axis(int32_t dtype, int32_t k, int32_t c, int32_t rs, int32_t axis, const void* w,
                                   const float* scale, void* w_out, void* hip_stream);
relay_status relay_fold_bias(int32_t k, const float* bias, const float* scale, const float* shift, float* out,
                             void* hip_stream);

/* The compile-time half of the quantization flow on the device (paper Section 4.2, "Calibrate" and
 * "Realize", after the axis scale folding of Section 4.4), 8-bit signed scheme (beta = 8, sigma = 1)
 * with power-of-two ranges: a tensor with range rho holds code * rho / 2^7.
 *
 * relay_calibrate_pow2_range: the "no overflow" rule for one tensor -- *rho_out = the smallest
 *   power of two that no |x[i]| exceeds (2^-20 for a tensor of zeros; NaN is ignored).
 *   x: device, F32 or F16, n_elems values; rho_out: DEVICE float; cell: DEVICE scratch of 4 bytes
 *   (4-byte aligned; the call clears it).
 *
 * relay_realize_conv: one convolution with filters w [k][per_k] (OIHW flattened, per_k = c*r*s),
 *   tail [+bias] -> [*scale + shift], input range rho_x, output range rho_y, residual range
 *   rho_res (0: no residual operand); all device pointers, fp32:
 *     w'[k][i]  = w[k][i] * scale[k]           (exact product, one rounding to fp32; scale NULL: w)
 *     rho_w     = smallest power of two >= max |w'|
 *     wq        = Q(w', rho_w, 8, 1), round to nearest            -> int8 [k][per_k]
 *     unit      = rho_x * rho_w / 2^14                            (worth of one accumulator count)
 *     bias_q[k] = floor((bias[k]*scale[k] + shift[k]) / unit + 1/2)   -> int32 [k]  (fp64; bias NULL: 0;
 *                 scale NULL: bias[k]; bias_q NULL allowed when bias and shift are both NULL)
 *     out_rshift = log2(2^7 rho_y / (rho_x rho_w)),  residual_lshift = log2(2^7 rho_res / (rho_x rho_w))
 *   out: DEVICE relay_realized_conv; status is 0 or an OR of RELAY_REALIZE_* bits (a shift that is not
 *   an integer in the range relay_qconv2d_requant takes, a bias outside int32 -- stored as 0).
 *   workspace: device, 16-byte aligned, at least k*per_k*4 + 16 bytes (the folded filters and the
 *   maximum), else RELAY_ERR_WORKSPACE.  scale and shift are given together or not at all.
 * Both calls only enqueue kernels on hip_stream; the caller copies the few result words back when
 * it needs them on the host.  Errors: RELAY_ERR_NULL, _SHAPE (extents, non-positive or infinite
 * ranges), _DTYPE, _ALIGN, _WORKSPACE, _DEVICE. */
typedef struct {
  float rho_w;
  int32_t out_rshift, residual_lshift, status;
} relay_realized_conv;
enum { RELAY_REALIZE_BAD_OUT_SHIFT = 1, RELAY_REALIZE_BAD_RES_SHIFT = 2, RELAY_REALIZE_BIAS_OVERFLOW = 4 };
relay_status relay_calibrate_pow2_range(int32_t dtype, int64_t n_elems, const void* x, float* rho_out, void* cell,
                                        void* hip_stream);
relay_status relay_realize_conv(int32_t k, int64_t per_k, const float* w, const float* bias, const float* scale,
                                const float* shift, float rho_x, float rho_y, float rho_res, int8_t* wq,
                                int32_t* bias_q, relay_realized_conv* out, void* workspace, size_t workspace_bytes,
                                void* hip_stream);

/* For callers that cannot allocate device memory (code under HIP-graph capture, serving loops and
 * harnesses that forbid hipMalloc): relay_fused_conv2d_bias_bn_relu for F16 NHWC / NHWC4_PADDED
 * descriptors with the reduction-split scratch (see relay_workspace_bytes) taken from a static
 * device array inside the library instead of a caller workspace.  Same operands, same results bit
 * for bit as that call given a workspace.  Nothing is allocated or freed, by this call or by any
 * routine it uses.  Limits: relay_workspace_bytes(d) must not exceed RELAY_STATIC_SCRATCH_BYTES, else
 * RELAY_ERR_WORKSPACE and nothing is launched (every ResNet-18 / MobileNet layer at any batch fits).
 * Every GPU the library runs on holds one such array until the process ends; all calls on a GPU
 * share it, so two of these calls that may overlap in time on one GPU (different streams or
 * threads) race -- serialise them, or use the workspace form.  The arrival counters at its start are
 * cleared by a small kernel ahead of each launch that uses them. */
#define RELAY_STATIC_SCRATCH_BYTES (4u << 20)
relay_status relay_fused_conv2d_bias_bn_relu_static(const relay_conv2d_desc* d, const void* x, const void* w_packed,
                                                    const float* bias, const float* bn_scale, const float* bn_shift,
                                                    const void* residual, void* y, void* hip_stream);

/* Layout alteration of an activation tensor (paper Section 5.3 lists the alteration of operator
 * data layouts among the compiler's passes): [n,c,h,w] -> [n,h,w,c_pad], channels c..c_pad-1 zero.
 * Any dtype; c_pad >= c; x, y device, y must not alias x. */
relay_status relay_nchw_to_nhwc(int32_t dtype, int32_t n, int32_t c, int32_t h, int32_t w, int32_t c_pad,
                                const void* x, void* y, void* hip_stream);

/* Tuning aid (the library's stand-in for the schedule search of paper Section 4.1, "Lowering":
 * which schedule a fused operator gets is a choice made per shape and platform): force the
 * implicit-GEMM workgroup tile of later fp16 / int8 conv calls made BY THE CALLING THREAD
 * (0 .. count-1, largest first; 100 + v: variant v of the 3x3 stride-1 kernel; -1 = choose by
 * layer shape, the default; -2 = by layer shape without the 3x3 stride-1 kernel).  The setting is
 * thread-local: other threads' calls are unaffected and nothing is shared between threads.
 * Results do not depend on the tile (int8: bit for bit). */
relay_status relay_set_conv_tile(int32_t tile);
/* Tuning aid (paper Section 4.1, "Lowering", as above), thread-local like relay_set_conv_tile: workgroups per output tile of the calling
 * thread's later conv calls that are given a workspace (0 = choose by layer shape, the default;
 * 1 = never split; n <= 64, clamped to the number of reduction chunks).  relay_workspace_bytes
 * called from the same thread follows the setting. */
relay_status relay_set_conv_split(int32_t split);
/* Tuning aid (paper Section 4.1, "Lowering", as above), thread-local: upper bound on the number of
 * workgroups in the grid of the persistent 3x3 stride-1 kernel, whose workgroups each walk a list
 * of output tiles (0 = one per workgroup slot of the chip, the default).  A smaller grid leaves
 * compute units to other streams and makes every workgroup walk more tiles; results do not depend
 * on it. */
relay_status relay_set_conv_workgroups(int32_t workgroups);

/* Measurement aids for the roofline figures (paper Section 5.1 states how its measurements are
 * taken; these give the chip's measured ceilings to set beside the nominal ones):
 *   relay_probe_mfma  every wave of `workgroups` workgroups of 256 threads runs `iters` rounds of four
 *                     independent 32x32 matrix instructions (F16: 32x32x16, I8: 32x32x32) on registers
 *                     only: 2 * 32*32*K * 4 * iters * 4 * workgroups operations per launch.
 *                     out: device, 4 bytes (practically never written).
 *   relay_probe_copy  dst[i] = src[i] over `bytes` bytes (a multiple of 16) in 16-byte pieces, a
 *                     grid-stride loop of 4096 workgroups: reads and writes `bytes` each.
 *   relay_probe_grid_barrier  one launch of `workgroups` (1..1024) workgroups of 256 threads that meet in
 *                     `rounds` barriers across the whole grid: a device-scope release and an atomic arrival,
 *                     a bounded poll (at most spin_limit device-scope loads per wait), an acquire -- what a
 *                     boundary between dependent layers inside ONE launch costs, to set beside the cost
 *                     of a kernel boundary (paper Section 5.2, launch overhead at small batch).  cells: 16
 *                     bytes on the device, zero before the first launch; a launch whose waits all
 *                     succeed leaves cells[0] = cells[2] = 0 for the next one.  cells[1] != 0 afterwards:
 *                     a wait ran out (every workgroup then leaves; clear cells before the next launch).
 *                     data: NULL, or workgroups * 256 floats that every thread adds to before each barrier
 *                     (gives the release something to write back).  rounds == 0: an empty kernel.
 * Device pointers owned by the caller; only enqueue on hip_stream. */
relay_status relay_probe_grid_barrier(int32_t workgroups, int32_t rounds, uint32_t spin_limit, void* cells, void* data,
                                      void* hip_stream);
relay_status relay_probe_mfma(int32_t dtype, int32_t iters, int32_t workgroups, void* out, void* hip_stream);
relay_status relay_probe_copy(const void* src, void* dst, int64_t bytes, void* hip_stream);

/* Profiling aid (lowered code is specific to shape and platform, paper Section 4.1 "Lowering": this
 * tells which specialisation a shape gets): the name, as a kernel trace prints it, of the
 * implicit-GEMM kernel variant a fp16 / int8 descriptor runs on (template arguments give the workgroup's wave grid and
 * per-wave MFMA tile).  buf receives a NUL-terminated string of at most len bytes. */
relay_status relay_conv2d_kernel_name(const relay_conv2d_desc* d, char* buf, size_t len);

/* Part of the fixed calling convention (paper Section 3.3, "Backends"): every entry point returns a
 * relay_status and raises nothing; this returns the message of the calling thread's last failed
 * call (thread-local static storage owned by the library, never NULL, valid until that thread's
 * next failing call). */
const char* relay_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* RELAY_FUSED_H_ */
