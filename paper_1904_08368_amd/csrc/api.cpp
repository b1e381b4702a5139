// C-ABI layer: argument checks on the host, then dispatch to the gfx950 kernels.
// Every check runs before the first HIP call, so the error paths are testable on a
// machine without a GPU.
#include <atomic>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>

#include "../../include/relay_fused.h"
#include "../../include/relay_fusion.h"
#include "fusion.hpp"
#include "kernels.hpp"

namespace {

thread_local char g_err[256] = "";

relay_status fail(relay_status st, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return st;
}

int esize_of(int dtype) { return dtype == RELAY_F32 ? 4 : (dtype == RELAY_F16 || dtype == RELAY_I16) ? 2 : dtype == RELAY_I8 ? 1 : 0; }

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

constexpr long kMaxElems = (1L << 31) - 1;  // kernels index activations with 32-bit element offsets

// Geometry checks shared by every conv-like entry point.
relay_status check_geometry(const relay_conv2d_desc* d, int* ho, int* wo) {
  if (!d) return fail(RELAY_ERR_NULL, "descriptor is NULL");
  if (d->n <= 0 || d->c <= 0 || d->h <= 0 || d->w <= 0 || d->k <= 0 || d->r <= 0 || d->s <= 0)
    return fail(RELAY_ERR_SHAPE, "non-positive extent (n=%d c=%d h=%d w=%d k=%d r=%d s=%d)", d->n, d->c, d->h, d->w,
                d->k, d->r, d->s);
  if (d->stride_h <= 0 || d->stride_w <= 0) return fail(RELAY_ERR_SHAPE, "stride must be positive");
  if (d->pad_h < 0 || d->pad_w < 0) return fail(RELAY_ERR_SHAPE, "padding must be non-negative");
  if (d->pad_h >= d->r || d->pad_w >= d->s)
    return fail(RELAY_ERR_SHAPE, "padding (%d,%d) must be smaller than the kernel (%d,%d)", d->pad_h, d->pad_w, d->r,
                d->s);
  if (d->h + 2 * d->pad_h < d->r || d->w + 2 * d->pad_w < d->s)
    return fail(RELAY_ERR_SHAPE, "kernel larger than the padded input: empty output");
  if (esize_of(d->dtype) == 0) return fail(RELAY_ERR_DTYPE, "unknown dtype %d", d->dtype);
  if (d->layout != RELAY_NCHW && d->layout != RELAY_NHWC && d->layout != RELAY_NHWC4_PADDED)
    return fail(RELAY_ERR_UNSUPPORTED, "unknown layout %d", d->layout);
  if (d->flags & ~(uint32_t)(RELAY_HAS_BIAS | RELAY_HAS_BN | RELAY_HAS_RESIDUAL | RELAY_RELU))
    return fail(RELAY_ERR_UNSUPPORTED, "unknown flag bits 0x%x", d->flags);
  const int oh = (d->h + 2 * d->pad_h - d->r) / d->stride_h + 1;
  const int ow = (d->w + 2 * d->pad_w - d->s) / d->stride_w + 1;
  if ((long)d->n * d->c * d->h * d->w > kMaxElems || (long)d->n * d->k * oh * ow > kMaxElems ||
      (long)d->k * d->c * d->r * d->s > kMaxElems)
    return fail(RELAY_ERR_SHAPE, "tensor exceeds 2^31-1 elements");
  *ho = oh;
  *wo = ow;
  return RELAY_OK;
}

relay_status check_optional(const void* p, bool wanted, const char* name) {
  if (wanted && !p) return fail(RELAY_ERR_NULL, "%s is NULL but its flag is set", name);
  if (!wanted && p) return fail(RELAY_ERR_NULL, "%s is given but its flag is clear", name);
  return RELAY_OK;
}

// width of the pre-padded NHWC4 input: the padded row rounded up to 8 pixels
int nhwc4_padded_w(const relay_conv2d_desc* d) { return (d->w + 2 * d->pad_w + 7) & ~7; }
// reduction elements per filter row in the row-packed stem path: one 64-byte chunk
int nhwc4_row_chunk(const relay_conv2d_desc* d) { return 64 / esize_of(d->dtype); }

relay::ConvArgs make_args(const relay_conv2d_desc* d, int ho, int wo) {
  relay::ConvArgs a;
  memset(&a, 0, sizeof(a));
  a.N = d->n; a.H = d->h; a.W = d->w; a.C = d->c; a.K = d->k; a.R = d->r; a.S = d->s;
  a.sh = d->stride_h; a.sw = d->stride_w; a.ph = d->pad_h; a.pw = d->pad_w;
  a.Ho = ho; a.Wo = wo;
  a.M = d->n * ho * wo;
  a.flags = d->flags;
  if (d->layout == RELAY_NHWC4_PADDED) {
    // Row-packed view: the s taps and 4 channels of one filter row are contiguous in the
    // padded NHWC4 tensor, so a whole filter row (padded to one 64-byte chunk) is one
    // "pixel" of C = chunk channels; pixels overlap (xs_w = 4) and nothing is out of range.
    const int wp = nhwc4_padded_w(d), hp = d->h + 2 * d->pad_h;
    a.C = nhwc4_row_chunk(d);
    a.S = 1;
    a.ph = a.pw = 0;
    a.H = hp;
    a.W = wp;
    a.xs_w = 4;
    a.xs_h = wp * 4;
    a.xs_n = hp * wp * 4;
  } else {
    a.xs_w = d->c;
    a.xs_h = d->w * d->c;
    a.xs_n = d->h * d->w * d->c;
  }
  a.clip_lo = -127;
  a.clip_hi = 127;
  a.Kred = a.R * a.S * a.C;
  a.Kp = relay::packed_pitch(a.Kred, esize_of(d->dtype));
  a.fd_wo = relay::make_fastdiv((uint32_t)wo);
  a.fd_howo = relay::make_fastdiv((uint32_t)(ho * wo));
  a.rcp_wo = 1.0f / (float)wo;
  a.rcp_ho = 1.0f / (float)ho;
  if (a.R * a.S <= 32)
    for (int r = 0; r < a.R; ++r) a.tap_spread |= 1u << (r * a.S);
  return a;
}

// Tuning overrides of the calling thread (relay_set_conv_tile / relay_set_conv_split): thread-local, so
// that threads cannot disturb each other's calls and nothing is shared between them.
thread_local int g_force_tile = -1;
thread_local int g_force_split = 0;  // 0: by layer shape; n >= 1: n workgroups per tile where the kernel can split
thread_local int g_max_wgs = 0;      // 0: fill the chip; n >= 1: at most n workgroups in a persistent kernel's grid

// after the operand pointers are in place
void finish_args(relay::ConvArgs& a) {
  const bool al = aligned(a.bias, 16) && aligned(a.scale, 16) && aligned(a.shift, 16) && aligned(a.qbias, 16);
  a.param_vec = (al && (a.K & 7) == 0) ? 1 : 0;
  a.max_wgs = g_max_wgs;
  // an XCD works through a run of consecutive tiles: let the run share whichever operand is
  // larger, so that the XCD's L2 only has to hold a slab of it
  a.n_major = (size_t)a.K * a.Kred > (size_t)a.N * a.H * a.W * a.C ? 1 : 0;
}

relay_status device_status(hipError_t e, const char* what) {
  if (e == hipSuccess) return RELAY_OK;
  return fail(RELAY_ERR_DEVICE, "%s: %s", what, hipGetErrorString(e));
}

// implicit-GEMM paths: which (dtype, layout, channel count) combinations have a kernel
relay_status check_igemm_support(const relay_conv2d_desc* d) {
  if (d->layout == RELAY_NHWC4_PADDED) {
    if (d->c > 4) return fail(RELAY_ERR_SHAPE, "the pre-padded NHWC4 layout holds at most 4 channels (c=%d)", d->c);
    if (d->s * 4 > nhwc4_row_chunk(d) || d->r > 32)
      return fail(RELAY_ERR_UNSUPPORTED, "filter %dx%d too large for the row-packed path", d->r, d->s);
    if ((long)d->n * (d->h + 2 * d->pad_h) * nhwc4_padded_w(d) * 4 * esize_of(d->dtype) > 0x7fffffffL)
      return fail(RELAY_ERR_SHAPE, "padded input exceeds 2^31-1 bytes");
    return RELAY_OK;
  }
  if (d->layout != RELAY_NHWC)
    return fail(RELAY_ERR_UNSUPPORTED, "fp16 / int8 conv2d needs NHWC activations");
  const int ve = d->dtype == RELAY_I8 ? 16 : 8;
  if (d->c % ve) return fail(RELAY_ERR_ALIGN, "c=%d must be a multiple of %d (pad the channel axis)", d->c, ve);
  return RELAY_OK;
}

}  // namespace

// ---- the allocation-free variant: reduction-split scratch in a static device array ----------------
// `scratch` is the name of the device array in device code; in host code the name is only a handle
// for hipGetSymbolAddress.  Each GPU holds its own copy at its own address: the address is looked
// up once per device (with that device current) and host code uses only that pointer.
static __device__ __align__(256) unsigned char scratch[RELAY_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

__global__ void clear_words_kernel(unsigned* p, int n) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0u;
}

// device address of `scratch` on the current device
relay_status scratch_address(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return device_status(e, "hipGetDevice");
  if (dev < 0 || dev >= kMaxDevices) return fail(RELAY_ERR_DEVICE, "device ordinal %d outside 0..%d", dev, kMaxDevices - 1);
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) return device_status(e == hipSuccess ? hipErrorInvalidSymbol : e, "hipGetSymbolAddress(scratch)");
    g_scratch_ptr[dev].store(p, std::memory_order_release);  // (two threads racing here store the same address)
  }
  *out = p;
  return RELAY_OK;
}
}  // namespace

extern "C" {

const char* relay_last_error(void) { return g_err; }

relay_status relay_conv2d_out_shape(const relay_conv2d_desc* d, int32_t* ho, int32_t* wo) {
  if (!ho || !wo) return fail(RELAY_ERR_NULL, "output pointers are NULL");
  int oh, ow;
  relay_status st = check_geometry(d, &oh, &ow);
  if (st != RELAY_OK) return st;
  *ho = oh;
  *wo = ow;
  return RELAY_OK;
}

// Split of the reduction over workgroups for this layer (1: none) and the workspace it takes.
// Only the direct-to-LDS implicit GEMM splits; a layer that goes to another kernel gets 1.
static int plan_split(const relay::ConvArgs& a, bool is_i8, size_t* counter_bytes, size_t* total_bytes);

relay_status relay_workspace_bytes(const relay_conv2d_desc* d, size_t* bytes) {
  if (!bytes) return fail(RELAY_ERR_NULL, "bytes is NULL");
  int oh, ow;
  relay_status st = check_geometry(d, &oh, &ow);
  if (st != RELAY_OK) return st;
  *bytes = 0;  // most layers keep their partial sums in registers
  if ((d->dtype == RELAY_F16 || d->dtype == RELAY_I8) && check_igemm_support(d) == RELAY_OK) {
    const relay::ConvArgs a = make_args(d, oh, ow);
    size_t cb = 0;
    plan_split(a, d->dtype == RELAY_I8, &cb, bytes);
  }
  return RELAY_OK;
}

relay_status relay_packed_weight_bytes(const relay_conv2d_desc* d, size_t* bytes) {
  if (!bytes) return fail(RELAY_ERR_NULL, "bytes is NULL");
  int oh, ow;
  relay_status st = check_geometry(d, &oh, &ow);
  if (st != RELAY_OK) return st;
  const int es = esize_of(d->dtype);
  if (d->dtype == RELAY_F32) {
    if (d->layout != RELAY_NCHW) return fail(RELAY_ERR_UNSUPPORTED, "fp32 conv2d is NCHW only");
    *bytes = (size_t)d->k * d->c * d->r * d->s * es;
  } else {
    if ((st = check_igemm_support(d)) != RELAY_OK) return st;
    const int kred = d->layout == RELAY_NHWC4_PADDED ? d->r * nhwc4_row_chunk(d) : d->r * d->s * d->c;
    *bytes = (size_t)d->k * relay::packed_pitch(kred, es) * es;
  }
  return RELAY_OK;
}

relay_status relay_nhwc4_padded_shape(const relay_conv2d_desc* d, int32_t* hp, int32_t* wp) {
  if (!hp || !wp) return fail(RELAY_ERR_NULL, "output pointers are NULL");
  int oh, ow;
  relay_status st = check_geometry(d, &oh, &ow);
  if (st != RELAY_OK) return st;
  if (d->c > 4) return fail(RELAY_ERR_SHAPE, "the pre-padded NHWC4 layout holds at most 4 channels (c=%d)", d->c);
  *hp = d->h + 2 * d->pad_h;
  *wp = nhwc4_padded_w(d);
  return RELAY_OK;
}

relay_status relay_pack_input_nhwc4(const relay_conv2d_desc* d, const void* x_nchw, void* y, void* hip_stream) {
  int oh, ow;
  relay_status st = check_geometry(d, &oh, &ow);
  if (st != RELAY_OK) return st;
  if (d->dtype != RELAY_F16 && d->dtype != RELAY_I8) return fail(RELAY_ERR_DTYPE, "NHWC4 packing takes F16 or I8");
  if (d->c > 4) return fail(RELAY_ERR_SHAPE, "the pre-padded NHWC4 layout holds at most 4 channels (c=%d)", d->c);
  if (!x_nchw || !y) return fail(RELAY_ERR_NULL, "x_nchw and y are required");
  if (x_nchw == y) return fail(RELAY_ERR_UNSUPPORTED, "output must not alias an input");
  if (!aligned(y, 16)) return fail(RELAY_ERR_ALIGN, "y must be 16-byte aligned");
  if ((long)d->n * (d->h + 2 * d->pad_h) * nhwc4_padded_w(d) * 4 * esize_of(d->dtype) > 0x7fffffffL)
    return fail(RELAY_ERR_SHAPE, "padded input exceeds 2^31-1 bytes");
  return device_status(relay::launch_pack_input_nhwc4(esize_of(d->dtype), d->n, d->c, d->h, d->w, d->pad_h, d->pad_w,
                                                      nhwc4_padded_w(d), x_nchw, y, static_cast<hipStream_t>(hip_stream)),
                       "NHWC4 input packing");
}

relay_status relay_prepack_conv2d_weights(const relay_conv2d_desc* d, const void* w_oihw, int32_t c_src,
                                          void* w_packed, size_t packed_bytes, void* hip_stream) {
  size_t need = 0;
  relay_status st = relay_packed_weight_bytes(d, &need);
  if (st != RELAY_OK) return st;
  if (!w_oihw || !w_packed) return fail(RELAY_ERR_NULL, "weight pointer is NULL");
  if (c_src <= 0 || c_src > d->c) return fail(RELAY_ERR_SHAPE, "c_src=%d must lie in 1..c=%d", c_src, d->c);
  if (packed_bytes < need) return fail(RELAY_ERR_WORKSPACE, "packed buffer has %zu bytes, %zu needed", packed_bytes, need);
  const int es = esize_of(d->dtype);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  if (d->dtype == RELAY_F32) {
    if (c_src != d->c) return fail(RELAY_ERR_SHAPE, "fp32 NCHW filters are not channel-padded");
    return device_status(hipMemcpyAsync(w_packed, w_oihw, need, hipMemcpyDeviceToDevice, s), "filter copy");
  }
  if (!aligned(w_packed, 16)) return fail(RELAY_ERR_ALIGN, "w_packed must be 16-byte aligned");
  if (d->layout == RELAY_NHWC4_PADDED) {
    const int ck = nhwc4_row_chunk(d);
    return device_status(relay::launch_pack_filters_rows(w_oihw, w_packed, d->k, c_src, d->r, d->s, ck,
                                                         relay::packed_pitch(d->r * ck, es), es, s),
                         "filter packing");
  }
  const int kp = relay::packed_pitch(d->r * d->s * d->c, es);
  return device_status(relay::launch_pack_filters(w_oihw, w_packed, d->k, c_src, d->c, d->r, d->s, kp, es, s),
                       "filter packing");
}

// g_force_tile: -1 heuristics; -2 heuristics without the 3x3 stride-1 kernels; 0.. a tile of the
// implicit-GEMM kernels; kHaloBase + v the halo kernel's variant v, kStreamBase + v the persistent
// kernel's variant v (where they apply)
constexpr int kHaloBase = 100;
constexpr int kStreamBase = 200;
constexpr int kDwPwBase = 300;   // ... of the fused depthwise + 1x1 kernel (its own entry point)

relay_status relay_set_conv_tile(int32_t tile) {
  const int most = relay::igemm_dma_tile_count() > relay::igemm_tile_count() ? relay::igemm_dma_tile_count()
                                                                             : relay::igemm_tile_count();
  const bool halo = (tile >= kHaloBase && tile < kHaloBase + relay::conv_halo_variant_count()) ||
                    (tile >= kStreamBase && tile < kStreamBase + relay::conv_stream_variant_count()) ||
                    (tile >= kDwPwBase && tile < kDwPwBase + relay::dwpw_variant_count());
  if (tile >= most && !halo) return fail(RELAY_ERR_UNSUPPORTED, "no tile %d", tile);
  g_force_tile = tile < -1 ? -2 : tile;
  return RELAY_OK;
}

// which variant of the persistent 3x3 stride-1 kernel runs this layer, or -1
static int stream_choice(const relay::ConvArgs& a, bool is_i8) {
  if (g_force_tile >= kStreamBase && g_force_tile < kDwPwBase)
    return relay::conv_stream_supported(a, is_i8, g_force_tile - kStreamBase) ? g_force_tile - kStreamBase : -1;
  return g_force_tile == -1 ? relay::conv_stream_pick(a, is_i8) : -1;
}

// which halo variant runs this layer, or -1
static int halo_choice(const relay::ConvArgs& a, bool is_i8) {
  if (stream_choice(a, is_i8) >= 0) return -1;
  if (g_force_tile >= kStreamBase) return -1;
  if (g_force_tile >= kHaloBase) return relay::conv_halo_supported(a, is_i8, g_force_tile - kHaloBase) ? g_force_tile - kHaloBase : -1;
  return g_force_tile == -1 ? relay::conv_halo_pick(a, is_i8) : -1;
}

static int plan_split(const relay::ConvArgs& a, bool is_i8, size_t* counter_bytes, size_t* total_bytes) {
  *counter_bytes = *total_bytes = 0;
  if (stream_choice(a, is_i8) >= 0 || halo_choice(a, is_i8) >= 0 || !relay::igemm_dma_supported(a, is_i8)) return 1;
  return relay::igemm_dma_plan_split(a, is_i8, g_force_tile, g_force_split, counter_bytes, total_bytes);
}

relay_status relay_set_conv_workgroups(int32_t workgroups) {
  if (workgroups < 0 || workgroups > (1 << 20)) return fail(RELAY_ERR_UNSUPPORTED, "workgroups=%d outside 0..2^20", workgroups);
  g_max_wgs = workgroups;
  return RELAY_OK;
}

relay_status relay_set_conv_split(int32_t split) {
  if (split < 0 || split > 64) return fail(RELAY_ERR_UNSUPPORTED, "split=%d outside 0..64", split);
  g_force_split = split;
  return RELAY_OK;
}

// Takes the caller's workspace into the arguments if this layer splits its reduction.
static relay_status use_workspace(relay::ConvArgs& a, bool is_i8, void* workspace, size_t workspace_bytes) {
  a.split = 1;
  if (!workspace) return RELAY_OK;  // without a workspace every tile is reduced by one workgroup
  size_t cb = 0, need = 0;
  const int split = plan_split(a, is_i8, &cb, &need);
  if (split <= 1) return RELAY_OK;
  if (!aligned(workspace, 256)) return fail(RELAY_ERR_ALIGN, "workspace must be 256-byte aligned");
  if (workspace_bytes < need)
    return fail(RELAY_ERR_WORKSPACE, "workspace has %zu bytes, relay_workspace_bytes asks for %zu", workspace_bytes, need);
  a.split = split;
  a.ws_cnt = static_cast<unsigned*>(workspace);
  a.ws_part = reinterpret_cast<unsigned*>(static_cast<char*>(workspace) + cb);
  return RELAY_OK;
}

static hipError_t launch_igemm(const relay::ConvArgs& a, bool is_i8, hipStream_t s) {
  const int sv = stream_choice(a, is_i8);
  if (sv >= 0) return relay::launch_conv_stream(a, is_i8, sv, s);
  const int hv = halo_choice(a, is_i8);
  if (hv >= 0) return relay::launch_conv_halo(a, is_i8, hv, s);
  if (relay::igemm_dma_supported(a, is_i8)) return relay::launch_conv_igemm_dma(a, is_i8, g_force_tile, s);
  if (a.xs_w != a.C) return hipErrorInvalidValue;  // the register-staged kernel reads plain NHWC only
  return relay::launch_conv_igemm(a, is_i8, g_force_tile, s);
}

relay_status relay_conv2d_kernel_name(const relay_conv2d_desc* d, char* buf, size_t len) {
  if (!buf || len == 0) return fail(RELAY_ERR_NULL, "name buffer is NULL or empty");
  int ho, wo;
  relay_status st = check_geometry(d, &ho, &wo);
  if (st != RELAY_OK) return st;
  if (d->dtype != RELAY_F16 && d->dtype != RELAY_I8) return fail(RELAY_ERR_DTYPE, "only the MFMA paths have kernel variants");
  if ((st = check_igemm_support(d)) != RELAY_OK) return st;
  relay::ConvArgs a = make_args(d, ho, wo);
  const bool i8 = d->dtype == RELAY_I8;
  if (stream_choice(a, i8) >= 0)
    relay::conv_stream_kernel_name(a, i8, stream_choice(a, i8), buf, len);
  else if (halo_choice(a, i8) >= 0)
    relay::conv_halo_kernel_name(a, i8, halo_choice(a, i8), buf, len);
  else if (relay::igemm_dma_supported(a, i8))
    relay::igemm_dma_kernel_name(a, i8, g_force_tile, buf, len);
  else
    relay::igemm_kernel_name(a, i8, g_force_tile, buf, len);
  return RELAY_OK;
}

relay_status relay_fused_conv2d_bias_bn_relu(const relay_conv2d_desc* d, const void* x, const void* w_packed,
                                             const float* bias, const float* bn_scale, const float* bn_shift,
                                             const void* residual, void* y, void* workspace,
                                             size_t workspace_bytes, void* hip_stream) {
  int ho, wo;
  relay_status st = check_geometry(d, &ho, &wo);
  if (st != RELAY_OK) return st;
  if (d->dtype != RELAY_F32 && d->dtype != RELAY_F16)
    return fail(RELAY_ERR_DTYPE, "float conv2d takes F32 or F16 (int8 goes through relay_qconv2d_requant)");
  if (!x || !w_packed || !y) return fail(RELAY_ERR_NULL, "x, w_packed and y are required");
  if ((st = check_optional(bias, d->flags & RELAY_HAS_BIAS, "bias")) != RELAY_OK) return st;
  if ((st = check_optional(bn_scale, d->flags & RELAY_HAS_BN, "bn_scale")) != RELAY_OK) return st;
  if ((st = check_optional(bn_shift, d->flags & RELAY_HAS_BN, "bn_shift")) != RELAY_OK) return st;
  if ((st = check_optional(residual, d->flags & RELAY_HAS_RESIDUAL, "residual")) != RELAY_OK) return st;
  if (y == x || y == residual) return fail(RELAY_ERR_UNSUPPORTED, "output must not alias an input");
  relay::ConvArgs a = make_args(d, ho, wo);
  a.x = x; a.w = w_packed; a.y = y; a.res = residual; a.bias = bias; a.scale = bn_scale; a.shift = bn_shift;
  finish_args(a);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  if (d->dtype == RELAY_F32) {
    if (d->layout != RELAY_NCHW) return fail(RELAY_ERR_UNSUPPORTED, "fp32 conv2d is NCHW only");
    if (!aligned(x, 4) || !aligned(w_packed, 4) || !aligned(y, 4)) return fail(RELAY_ERR_ALIGN, "fp32 pointers must be 4-byte aligned");
    return device_status(relay::launch_conv_direct_f32(a, s), "conv2d fp32 launch");
  }
  if ((st = check_igemm_support(d)) != RELAY_OK) return st;
  if (!aligned(x, 16) || !aligned(w_packed, 16) || !aligned(y, 16) || (residual && !aligned(residual, 16)))
    return fail(RELAY_ERR_ALIGN, "fp16 tensors must be 16-byte aligned");
  if ((st = use_workspace(a, false, workspace, workspace_bytes)) != RELAY_OK) return st;
  return device_status(launch_igemm(a, false, s), "conv2d fp16 launch");
}

// ---- the allocation-free variant of the fp16 conv (scratch: the static device array declared at the top)
relay_status relay_fused_conv2d_bias_bn_relu_static(const relay_conv2d_desc* d, const void* x, const void* w_packed,
                                                    const float* bias, const float* bn_scale, const float* bn_shift,
                                                    const void* residual, void* y, void* hip_stream) {
  int ho, wo;
  relay_status st = check_geometry(d, &ho, &wo);
  if (st != RELAY_OK) return st;
  if (d->dtype != RELAY_F16) return fail(RELAY_ERR_DTYPE, "the allocation-free conv2d takes F16");
  if (!x || !w_packed || !y) return fail(RELAY_ERR_NULL, "x, w_packed and y are required");
  if ((st = check_optional(bias, d->flags & RELAY_HAS_BIAS, "bias")) != RELAY_OK) return st;
  if ((st = check_optional(bn_scale, d->flags & RELAY_HAS_BN, "bn_scale")) != RELAY_OK) return st;
  if ((st = check_optional(bn_shift, d->flags & RELAY_HAS_BN, "bn_shift")) != RELAY_OK) return st;
  if ((st = check_optional(residual, d->flags & RELAY_HAS_RESIDUAL, "residual")) != RELAY_OK) return st;
  if (y == x || y == residual) return fail(RELAY_ERR_UNSUPPORTED, "output must not alias an input");
  if ((st = check_igemm_support(d)) != RELAY_OK) return st;
  if (!aligned(x, 16) || !aligned(w_packed, 16) || !aligned(y, 16) || (residual && !aligned(residual, 16)))
    return fail(RELAY_ERR_ALIGN, "fp16 tensors must be 16-byte aligned");
  relay::ConvArgs a = make_args(d, ho, wo);
  a.x = x; a.w = w_packed; a.y = y; a.res = residual; a.bias = bias; a.scale = bn_scale; a.shift = bn_shift;
  finish_args(a);
  size_t cb = 0, need = 0;
  const int split = plan_split(a, false, &cb, &need);
  if (need > RELAY_STATIC_SCRATCH_BYTES)
    return fail(RELAY_ERR_WORKSPACE, "this layer's reduction split needs %zu bytes of scratch, the static array holds %u", need,
                (unsigned)RELAY_STATIC_SCRATCH_BYTES);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  a.split = 1;
  if (split > 1) {
    void* base = nullptr;
    if ((st = scratch_address(&base)) != RELAY_OK) return st;
    a.split = split;
    a.ws_cnt = static_cast<unsigned*>(base);
    a.ws_part = reinterpret_cast<unsigned*>(static_cast<char*>(base) + cb);
    // the arrival counters must start at zero whatever an earlier call left behind; a fill kernel,
    // not a memset, so that the call can be recorded into a HIP graph
    const int words = (int)(cb / sizeof(unsigned));
    hipLaunchKernelGGL(clear_words_kernel, dim3((words + 255) / 256), dim3(256), 0, s, a.ws_cnt, words);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return device_status(e, "scratch clear launch");
  }
  return device_status(launch_igemm(a, false, s), "conv2d fp16 launch");
}

// ---- the first layer of an image network, read from the NCHW image -----------------------------------
static relay_status first_layer_args(const relay_conv2d_desc* d, relay::ConvArgs* out) {
  int ho, wo;
  relay_status st = check_geometry(d, &ho, &wo);
  if (st != RELAY_OK) return st;
  if (d->dtype != RELAY_F16) return fail(RELAY_ERR_DTYPE, "the first-layer conv2d takes F16");
  if (d->layout != RELAY_NCHW) return fail(RELAY_ERR_UNSUPPORTED, "the first-layer conv2d reads an NCHW image (layout RELAY_NCHW)");
  relay::ConvArgs a = make_args(d, ho, wo);
  if (!relay::conv_first_supported(a))
    return fail(RELAY_ERR_UNSUPPORTED,
                "the first-layer conv2d takes c == 3, 3x3 / stride 2 / pad 1, k %% 16 == 0, k <= 128, w %% 8 == 0, h even, no "
                "residual, an output below 2^31 elements (c=%d r=%d s=%d stride=%d pad=%d k=%d h=%d w=%d)",
                d->c, d->r, d->s, d->stride_h, d->pad_h, d->k, d->h, d->w);
  *out = a;
  return RELAY_OK;
}

relay_status relay_conv2d_first_layer_supported(const relay_conv2d_desc* d, int32_t* supported) {
  if (!supported) return fail(RELAY_ERR_NULL, "supported is NULL");
  int ho, wo;
  relay_status st = check_geometry(d, &ho, &wo);
  if (st != RELAY_OK) return st;
  const relay::ConvArgs a = make_args(d, ho, wo);
  *supported = (d->dtype == RELAY_F16 && d->layout == RELAY_NCHW && relay::conv_first_supported(a)) ? 1 : 0;
  return RELAY_OK;
}

relay_status relay_first_layer_packed_weight_bytes(const relay_conv2d_desc* d, size_t* bytes) {
  if (!bytes) return fail(RELAY_ERR_NULL, "bytes is NULL");
  relay::ConvArgs a;
  relay_status st = first_layer_args(d, &a);
  if (st != RELAY_OK) return st;
  *bytes = relay::conv_first_packed_bytes(a.K);
  return RELAY_OK;
}

relay_status relay_prepack_first_layer_weights(const relay_conv2d_desc* d, const void* w_oihw, void* w_packed,
                                               void* hip_stream) {
  relay::ConvArgs a;
  relay_status st = first_layer_args(d, &a);
  if (st != RELAY_OK) return st;
  if (!w_oihw || !w_packed) return fail(RELAY_ERR_NULL, "w_oihw and w_packed are required");
  if (!aligned(w_oihw, 2) || !aligned(w_packed, 16)) return fail(RELAY_ERR_ALIGN, "w_oihw must be 2-byte, w_packed 16-byte aligned");
  return device_status(relay::launch_pack_first_filters(w_oihw, w_packed, a.K, static_cast<hipStream_t>(hip_stream)),
                       "first-layer filter packing launch");
}

relay_status relay_fused_conv2d_first_layer(const relay_conv2d_desc* d, const void* x_nchw, const void* w_packed,
                                            const float* bias, const float* bn_scale, const float* bn_shift,
                                            void* y_nhwc, void* hip_stream) {
  relay::ConvArgs a;
  relay_status st = first_layer_args(d, &a);
  if (st != RELAY_OK) return st;
  if (!x_nchw || !w_packed || !y_nhwc) return fail(RELAY_ERR_NULL, "x_nchw, w_packed and y_nhwc are required");
  if ((st = check_optional(bias, d->flags & RELAY_HAS_BIAS, "bias")) != RELAY_OK) return st;
  if ((st = check_optional(bn_scale, d->flags & RELAY_HAS_BN, "bn_scale")) != RELAY_OK) return st;
  if ((st = check_optional(bn_shift, d->flags & RELAY_HAS_BN, "bn_shift")) != RELAY_OK) return st;
  if (y_nhwc == x_nchw) return fail(RELAY_ERR_UNSUPPORTED, "output must not alias an input");
  if (!aligned(x_nchw, 16) || !aligned(y_nhwc, 16) || !aligned(w_packed, 16))
    return fail(RELAY_ERR_ALIGN, "x_nchw, w_packed and y_nhwc must be 16-byte aligned");
  a.x = x_nchw; a.w = w_packed; a.y = y_nhwc; a.bias = bias; a.scale = bn_scale; a.shift = bn_shift;
  return device_status(relay::launch_conv_first(a, static_cast<hipStream_t>(hip_stream)), "first-layer conv2d launch");
}

// quantized form of a combined launch: the int32 bias and the scaling rule of the tail (NULL: the float form)
struct CombinedQuant {
  const int32_t* bias;
  const int32_t* mult;     // per-channel multiplier and shift (QMODE_SCALED), or NULL: one power-of-two shift
  const int32_t* rshift_k;
  int out_rshift;
};
static relay_status combined_conv(const relay_conv2d_desc* d, const void* x, int32_t x_ld, const void* w_packed,
                                  const float* bias, const float* bn_scale, const float* bn_shift, int32_t nseg,
                                  const int32_t* seg_channels, void* const* seg_y, const int32_t* seg_ld,
                                  const int32_t* seg_window, const int32_t* seg_relu, void* hip_stream,
                                  const CombinedQuant* q = nullptr);

relay_status relay_fused_conv2d_combined(const relay_conv2d_desc* d, const void* x, int32_t x_ld,
                                         const void* w_packed, const float* bias, const float* bn_scale,
                                         const float* bn_shift, int32_t nseg, const int32_t* seg_channels,
                                         void* const* seg_y, const int32_t* seg_ld, void* hip_stream) {
  return combined_conv(d, x, x_ld, w_packed, bias, bn_scale, bn_shift, nseg, seg_channels, seg_y, seg_ld, nullptr,
                       nullptr, hip_stream);
}

relay_status relay_fused_conv2d_combined_windows(const relay_conv2d_desc* d, const void* x, int32_t x_ld,
                                                 const void* w_packed, const float* bias, const float* bn_scale,
                                                 const float* bn_shift, int32_t nseg, const int32_t* seg_channels,
                                                 void* const* seg_y, const int32_t* seg_ld,
                                                 const int32_t* seg_window, const int32_t* seg_relu,
                                                 void* hip_stream) {
  if (!seg_window || !seg_relu) return fail(RELAY_ERR_NULL, "seg_window and seg_relu are required");
  return combined_conv(d, x, x_ld, w_packed, bias, bn_scale, bn_shift, nseg, seg_channels, seg_y, seg_ld, seg_window,
                       seg_relu, hip_stream);
}

relay_status relay_qconv2d_combined(const relay_conv2d_desc* d, const int8_t* x, int32_t x_ld, const int8_t* w_packed,
                                    const int32_t* bias, const int32_t* mult, const int32_t* rshift, int32_t out_rshift,
                                    int32_t nseg, const int32_t* seg_channels, void* const* seg_y, const int32_t* seg_ld,
                                    void* hip_stream) {
  if ((mult == nullptr) != (rshift == nullptr)) return fail(RELAY_ERR_NULL, "mult and rshift are given together or not at all");
  if (!mult && (out_rshift < 0 || out_rshift > 31)) return fail(RELAY_ERR_UNSUPPORTED, "out_rshift=%d outside 0..31", out_rshift);
  if (!aligned(mult, 4) || !aligned(rshift, 4) || !aligned(bias, 4)) return fail(RELAY_ERR_ALIGN, "bias, mult and rshift must be 4-byte aligned");
  const CombinedQuant q{bias, mult, rshift, out_rshift};
  return combined_conv(d, x, x_ld, w_packed, nullptr, nullptr, nullptr, nseg, seg_channels, seg_y, seg_ld, nullptr, nullptr,
                       hip_stream, &q);
}

static relay_status combined_conv(const relay_conv2d_desc* d, const void* x, int32_t x_ld, const void* w_packed,
                                  const float* bias, const float* bn_scale, const float* bn_shift, int32_t nseg,
                                  const int32_t* seg_channels, void* const* seg_y, const int32_t* seg_ld,
                                  const int32_t* seg_window, const int32_t* seg_relu, void* hip_stream,
                                  const CombinedQuant* q) {
  int ho, wo;
  relay_status st = check_geometry(d, &ho, &wo);
  if (st != RELAY_OK) return st;
  const bool i8 = q != nullptr;
  const int xa = i8 ? 16 : 8;   // channel granularity of the input view (one 16-byte vector)
  if (i8 && d->dtype != RELAY_I8) return fail(RELAY_ERR_DTYPE, "the combined quantized conv2d takes I8");
  if (i8 && (d->flags & RELAY_HAS_BN)) return fail(RELAY_ERR_UNSUPPORTED, "the quantized epilogue has no float scale/shift");
  if (!i8 && d->dtype != RELAY_F16) return fail(RELAY_ERR_DTYPE, "the combined conv2d takes F16");
  if (d->layout != RELAY_NHWC) return fail(RELAY_ERR_UNSUPPORTED, "the combined conv2d takes NHWC");
  if (d->flags & RELAY_HAS_RESIDUAL) return fail(RELAY_ERR_UNSUPPORTED, "the combined conv2d has no residual operand");
  if (!x || !w_packed || !seg_channels || !seg_y || !seg_ld)
    return fail(RELAY_ERR_NULL, "x, w_packed and the segment arrays are required");
  if ((st = check_optional(i8 ? (const void*)q->bias : (const void*)bias, d->flags & RELAY_HAS_BIAS, "bias")) != RELAY_OK) return st;
  if ((st = check_optional(bn_scale, d->flags & RELAY_HAS_BN, "bn_scale")) != RELAY_OK) return st;
  if ((st = check_optional(bn_shift, d->flags & RELAY_HAS_BN, "bn_shift")) != RELAY_OK) return st;
  if (nseg < 1 || nseg > 4) return fail(RELAY_ERR_SHAPE, "nseg=%d outside 1..4", nseg);
  if (x_ld < d->c || x_ld % xa) return fail(RELAY_ERR_SHAPE, "x_ld=%d must be a multiple of %d and at least c=%d", x_ld, xa, d->c);
  if ((long)d->n * d->h * d->w * x_ld > kMaxElems) return fail(RELAY_ERR_SHAPE, "input view exceeds 2^31-1 elements");
  relay::ConvArgs a = make_args(d, ho, wo);
  long total = 0;
  for (int i = 0; i < nseg; ++i) {
    if (seg_channels[i] <= 0 || seg_channels[i] % 8)
      return fail(RELAY_ERR_SHAPE, "segment %d has %d channels: must be a positive multiple of 8", i, seg_channels[i]);
    if (seg_ld[i] < seg_channels[i] || seg_ld[i] % 8)
      return fail(RELAY_ERR_SHAPE, "seg_ld[%d]=%d must be a multiple of 8 and at least %d", i, seg_ld[i], seg_channels[i]);
    if (!seg_y[i]) return fail(RELAY_ERR_NULL, "seg_y[%d] is NULL", i);
    if (!aligned(seg_y[i], i8 ? 8 : 16)) return fail(RELAY_ERR_ALIGN, "seg_y[%d] must be %d-byte aligned", i, i8 ? 8 : 16);
    if (seg_y[i] == x) return fail(RELAY_ERR_UNSUPPORTED, "output must not alias an input");
    for (int j = 0; j < i; ++j)
      if (seg_y[j] == seg_y[i]) return fail(RELAY_ERR_UNSUPPORTED, "segments %d and %d share an address", j, i);
    if ((long)a.M * seg_ld[i] > kMaxElems) return fail(RELAY_ERR_SHAPE, "output view %d exceeds 2^31-1 elements", i);
    if (seg_window) {
      if (seg_window[i] != RELAY_WINDOW_FULL && seg_window[i] != RELAY_WINDOW_CENTRE)
        return fail(RELAY_ERR_UNSUPPORTED, "seg_window[%d]=%d is not a relay_segment_window", i, seg_window[i]);
      if (seg_window[i] == RELAY_WINDOW_CENTRE) {
        // the tiles of such a segment stop at its boundaries whatever tile the kernel takes (at most 128 channels wide)
        if (total % 128 || seg_channels[i] % 128)
          return fail(RELAY_ERR_SHAPE, "centre-tap segment %d must begin at and hold a multiple of 128 channels", i);
        if (!(d->r & 1) || !(d->s & 1) || d->pad_h != d->r / 2 || d->pad_w != d->s / 2)
          return fail(RELAY_ERR_UNSUPPORTED, "centre-tap segments need an odd window padded by half its size");
        a.seg_centre |= 1u << i;
      }
      if (seg_relu[i] != 0 && seg_relu[i] != 1) return fail(RELAY_ERR_UNSUPPORTED, "seg_relu[%d] must be 0 or 1", i);
      if (seg_relu[i] && !(d->flags & RELAY_RELU))
        return fail(RELAY_ERR_UNSUPPORTED, "seg_relu[%d] is set but the descriptor has no RELAY_RELU", i);
      if (!seg_relu[i] && (d->flags & RELAY_RELU)) a.seg_norelu |= 1u << i;
    }
    total += seg_channels[i];
    a.seg_end[i] = (int)total;
    a.seg_ld[i] = seg_ld[i];
    a.seg_y[i] = seg_y[i];
  }
  if (total != d->k) return fail(RELAY_ERR_SHAPE, "segments hold %ld channels, the descriptor k=%d", total, d->k);
  if ((st = check_igemm_support(d)) != RELAY_OK) return st;
  if (!aligned(x, 16) || !aligned(w_packed, 16)) return fail(RELAY_ERR_ALIGN, "x and w_packed must be 16-byte aligned");
  a.nseg = nseg;
  a.xs_w = x_ld;
  a.xs_h = d->w * x_ld;
  a.xs_n = d->h * d->w * x_ld;
  a.x = x; a.w = w_packed; a.y = seg_y[0]; a.bias = bias; a.scale = bn_scale; a.shift = bn_shift;
  if (i8) {
    a.qbias = q->bias;
    a.round_mode = RELAY_ROUND_NEAREST;
    if (q->mult) {
      a.qmode = relay::QMODE_SCALED; a.qmult = q->mult; a.qshift = q->rshift_k;
    } else {
      a.rshift = q->out_rshift;
      a.round_add = q->out_rshift == 0 ? 0 : 1 << (q->out_rshift - 1);
    }
  }
  finish_args(a);
  if (!relay::igemm_dma_supported(a, i8))
    return fail(RELAY_ERR_UNSUPPORTED, "the combined conv2d needs c %% %d == 0 and r*s <= 32 (c=%d, r=%d, s=%d)", i8 ? 64 : 32, d->c,
                d->r, d->s);
  return device_status(launch_igemm(a, i8, static_cast<hipStream_t>(hip_stream)), "combined conv2d launch");
}

relay_status relay_fold_scale_axis(int32_t dtype, int32_t k, int32_t c, int32_t rs, int32_t axis, const void* w,
                                   const float* scale, void* w_out, void* hip_stream) {
  if (dtype != RELAY_F16 && dtype != RELAY_F32) return fail(RELAY_ERR_DTYPE, "scale folding takes F16 or F32 filters");
  if (k <= 0 || c <= 0 || rs <= 0) return fail(RELAY_ERR_SHAPE, "non-positive extent (k=%d c=%d rs=%d)", k, c, rs);
  if ((long)k * c * rs > kMaxElems) return fail(RELAY_ERR_SHAPE, "filters exceed 2^31-1 elements");
  if (axis != RELAY_FOLD_OUT && axis != RELAY_FOLD_IN) return fail(RELAY_ERR_UNSUPPORTED, "unknown axis %d", axis);
  if (!w || !scale || !w_out) return fail(RELAY_ERR_NULL, "w, scale and w_out are required");
  if (!aligned(w, esize_of(dtype)) || !aligned(w_out, esize_of(dtype)) || !aligned(scale, 4))
    return fail(RELAY_ERR_ALIGN, "pointers must be aligned to their element size");
  return device_status(relay::launch_fold_scale_axis(dtype == RELAY_F16, k, c, rs, axis == RELAY_FOLD_IN, w, scale,
                                                     w_out, static_cast<hipStream_t>(hip_stream)),
                       "scale folding");
}

relay_status relay_fold_bias(int32_t k, const float* bias, const float* scale, const float* shift, float* out,
                             void* hip_stream) {
  if (k <= 0) return fail(RELAY_ERR_SHAPE, "k=%d must be positive", k);
  if (!scale || !shift || !out) return fail(RELAY_ERR_NULL, "scale, shift and out are required");
  if (!aligned(scale, 4) || !aligned(shift, 4) || !aligned(out, 4) || !aligned(bias, 4))
    return fail(RELAY_ERR_ALIGN, "pointers must be 4-byte aligned");
  return device_status(relay::launch_fold_bias(k, bias, scale, shift, out, static_cast<hipStream_t>(hip_stream)),
                       "bias folding");
}

relay_status relay_qconv2d_requant(const relay_conv2d_desc* d, const int8_t* x, const int8_t* w_packed,
                                   const int32_t* bias, const int8_t* residual, int32_t residual_lshift,
                                   int32_t out_rshift, int8_t* y, void* workspace, size_t workspace_bytes,
                                   void* hip_stream) {
  return relay_qconv2d_requant_rounding(d, x, w_packed, bias, residual, residual_lshift, out_rshift,
                                        RELAY_ROUND_NEAREST, 0, y, workspace, workspace_bytes, hip_stream);
}

// The quantized conv behind all of its entry points: the scaling rule of the tail (qmode, with its
// per-channel operands) and the bounds of the code type are the only things they differ in.
static relay_status qconv_common(const relay_conv2d_desc* d, const int8_t* x, const int8_t* w_packed, const int32_t* bias,
                                 const int8_t* residual, int32_t residual_lshift, int32_t out_rshift, int32_t round_mode,
                                 uint64_t seed, int qmode, const int32_t* qmult, const int32_t* qshift, int clip_lo,
                                 int clip_hi, void* y, void* workspace, size_t workspace_bytes, void* hip_stream);

relay_status relay_qconv2d_requant_rounding(const relay_conv2d_desc* d, const int8_t* x, const int8_t* w_packed,
                                            const int32_t* bias, const int8_t* residual, int32_t residual_lshift,
                                            int32_t out_rshift, int32_t round_mode, uint64_t seed, int8_t* y,
                                            void* workspace, size_t workspace_bytes, void* hip_stream) {
  return qconv_common(d, x, w_packed, bias, residual, residual_lshift, out_rshift, round_mode, seed, relay::QMODE_SHIFT, nullptr,
                      nullptr, -127, 127, y, workspace, workspace_bytes, hip_stream);
}

relay_status relay_qconv2d_requant_scaled(const relay_conv2d_desc* d, const int8_t* x, const int8_t* w_packed,
                                          const int32_t* bias, const int8_t* residual, int32_t residual_lshift,
                                          const int32_t* mult, const int32_t* rshift, int8_t* y, void* workspace,
                                          size_t workspace_bytes, void* hip_stream) {
  if (!mult || !rshift) return fail(RELAY_ERR_NULL, "mult and rshift are required");
  if (!aligned(mult, 4) || !aligned(rshift, 4)) return fail(RELAY_ERR_ALIGN, "mult and rshift must be 4-byte aligned");
  return qconv_common(d, x, w_packed, bias, residual, residual_lshift, 0, RELAY_ROUND_NEAREST, 0, relay::QMODE_SCALED, mult, rshift,
                      -127, 127, y, workspace, workspace_bytes, hip_stream);
}

relay_status relay_qconv2d_requant_acc16(const relay_conv2d_desc* d, const int8_t* x, const int8_t* w_packed,
                                         const int32_t* bias, const int8_t* residual, int32_t residual_lshift,
                                         int32_t out_rshift, int8_t* y, void* workspace, size_t workspace_bytes,
                                         void* hip_stream) {
  return qconv_common(d, x, w_packed, bias, residual, residual_lshift, out_rshift, RELAY_ROUND_NEAREST, 0, relay::QMODE_ACC16,
                      nullptr, nullptr, -127, 127, y, workspace, workspace_bytes, hip_stream);
}

relay_status relay_fold_zero_point(int32_t k, int64_t per_k, const int8_t* w, const int32_t* bias, int32_t zero_point,
                                   int32_t* out, void* hip_stream) {
  if (k <= 0 || per_k <= 0 || (long)k * per_k > kMaxElems) return fail(RELAY_ERR_SHAPE, "bad filter extent (k=%d per_k=%lld)", k, (long long)per_k);
  if (!w || !out) return fail(RELAY_ERR_NULL, "w and out are required");
  if (zero_point < -255 || zero_point > 255) return fail(RELAY_ERR_UNSUPPORTED, "zero_point=%d outside -255..255", zero_point);
  if (!aligned(bias, 4) || !aligned(out, 4)) return fail(RELAY_ERR_ALIGN, "bias and out must be 4-byte aligned");
  return device_status(relay::launch_fold_zero_point(k, per_k, w, bias, zero_point, out, static_cast<hipStream_t>(hip_stream)),
                       "zero-point folding");
}

relay_status relay_qconv2d_u8_workspace_bytes(const relay_conv2d_desc* d, size_t* bytes) {
  if (!bytes) return fail(RELAY_ERR_NULL, "bytes is NULL");
  int ho, wo;
  relay_status st = check_geometry(d, &ho, &wo);
  if (st != RELAY_OK) return st;
  if (d->dtype != RELAY_I8 || d->layout != RELAY_NHWC) return fail(RELAY_ERR_DTYPE, "unsigned activations take an I8 NHWC descriptor");
  *bytes = (size_t)d->n * (d->h + 2 * d->pad_h) * (d->w + 2 * d->pad_w) * d->c;
  return RELAY_OK;
}

relay_status relay_qconv2d_requant_u8(const relay_conv2d_desc* d, const uint8_t* x, const int8_t* w_packed,
                                      const int32_t* bias_zp, int32_t out_rshift, int32_t out_unsigned, void* y,
                                      void* workspace, size_t workspace_bytes, void* hip_stream) {
  size_t need = 0;
  relay_status st = relay_qconv2d_u8_workspace_bytes(d, &need);
  if (st != RELAY_OK) return st;
  if (d->flags & RELAY_HAS_RESIDUAL) return fail(RELAY_ERR_UNSUPPORTED, "the unsigned-activation conv2d has no residual operand");
  if (!(d->flags & RELAY_HAS_BIAS)) return fail(RELAY_ERR_NULL, "bias_zp (bias + 128 * sum of the filters) is required: set RELAY_HAS_BIAS");
  if (out_unsigned != 0 && out_unsigned != 1) return fail(RELAY_ERR_UNSUPPORTED, "out_unsigned must be 0 or 1");
  if (!x || !workspace) return fail(RELAY_ERR_NULL, "x and workspace are required");
  if (d->c % 16) return fail(RELAY_ERR_ALIGN, "c=%d must be a multiple of 16 (pad the channel axis)", d->c);
  if (!aligned(x, 16) || !aligned(workspace, 16)) return fail(RELAY_ERR_ALIGN, "x and workspace must be 16-byte aligned");
  if (workspace_bytes < need) return fail(RELAY_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, need);
  if (need > 0x7fffffffu) return fail(RELAY_ERR_SHAPE, "padded input exceeds 2^31-1 bytes");
  // the signed conv over the physically padded copy: same filters, no padding left
  relay_conv2d_desc d2 = *d;
  d2.h = d->h + 2 * d->pad_h;
  d2.w = d->w + 2 * d->pad_w;
  d2.pad_h = d2.pad_w = 0;
  // validate the conv call before anything is launched (the checks touch no pointer)
  if (!w_packed || !y || !bias_zp) return fail(RELAY_ERR_NULL, "w_packed, bias_zp and y are required");
  if (out_rshift < 0 || out_rshift > 31) return fail(RELAY_ERR_UNSUPPORTED, "out_rshift=%d outside 0..31", out_rshift);
  if (!aligned(w_packed, 16) || !aligned(y, 8) || !aligned(bias_zp, 4))
    return fail(RELAY_ERR_ALIGN, "w_packed must be 16-byte, y 8-byte, bias_zp 4-byte aligned");
  if (y == (const void*)x || y == workspace) return fail(RELAY_ERR_UNSUPPORTED, "output must not alias an input");
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  st = device_status(relay::launch_recode_u8_padded(x, workspace, d->n, d->h, d->w, d->c, d->pad_h, d->pad_w, s), "activation re-coding");
  if (st != RELAY_OK) return st;
  return qconv_common(&d2, static_cast<const int8_t*>(workspace), w_packed, bias_zp, nullptr, 0, out_rshift, RELAY_ROUND_NEAREST, 0,
                      relay::QMODE_SHIFT, nullptr, nullptr, out_unsigned ? 0 : -127, out_unsigned ? 255 : 127, y, nullptr, 0, hip_stream);
}

relay_status relay_qconv2d_requant_i16(const relay_conv2d_desc* d, const int16_t* x, const int16_t* w_packed,
                                       const int32_t* bias, int32_t out_rshift, int16_t* y, void* hip_stream) {
  int ho, wo;
  relay_status st = check_geometry(d, &ho, &wo);
  if (st != RELAY_OK) return st;
  if (d->dtype != RELAY_I16) return fail(RELAY_ERR_DTYPE, "the 16/32 conv2d takes I16");
  if (d->layout != RELAY_NHWC) return fail(RELAY_ERR_UNSUPPORTED, "the 16/32 conv2d needs NHWC activations");
  if (d->flags & (RELAY_HAS_BN | RELAY_HAS_RESIDUAL)) return fail(RELAY_ERR_UNSUPPORTED, "the 16/32 conv2d takes a bias and relu only");
  if (d->c % 8 || d->k % 4) return fail(RELAY_ERR_ALIGN, "c=%d must be a multiple of 8 and k=%d of 4", d->c, d->k);
  if (!x || !w_packed || !y) return fail(RELAY_ERR_NULL, "x, w_packed and y are required");
  if ((st = check_optional(bias, d->flags & RELAY_HAS_BIAS, "bias")) != RELAY_OK) return st;
  if (out_rshift < 0 || out_rshift > 31) return fail(RELAY_ERR_UNSUPPORTED, "out_rshift=%d outside 0..31", out_rshift);
  if (!aligned(x, 16) || !aligned(w_packed, 16) || !aligned(y, 8) || !aligned(bias, 4))
    return fail(RELAY_ERR_ALIGN, "x / w_packed must be 16-byte aligned, y 8-byte, bias 4-byte");
  if ((const void*)y == (const void*)x) return fail(RELAY_ERR_UNSUPPORTED, "output must not alias an input");
  relay::ConvArgs a = make_args(d, ho, wo);
  a.x = x; a.w = w_packed; a.y = y; a.qbias = bias;
  a.rshift = out_rshift;
  a.round_add = out_rshift == 0 ? 0 : 1 << (out_rshift - 1);
  return device_status(relay::launch_qconv16_direct(a, static_cast<hipStream_t>(hip_stream)), "16/32 conv2d launch");
}

relay_status relay_quantize_multiplier(double scale, int32_t* mult, int32_t* rshift) {
  if (!mult || !rshift) return fail(RELAY_ERR_NULL, "mult and rshift are required");
  if (!(scale > 0.0) || !(scale < 1.0)) return fail(RELAY_ERR_SHAPE, "scale must lie in (2^-32, 1)");
  int e = 0;
  const double m = frexp(scale, &e);   // scale = m * 2^e, 0.5 <= m < 1
  long long M = (long long)floor(ldexp(m, 31) + 0.5);
  if (M == (1ll << 31)) {              // m rounded up to 1
    M = 1ll << 30;
    ++e;
  }
  int s = -e;
  if (s == -1) {                       // so close to 1 that M rounded up to 2^31: the largest representable scale
    M = (1ll << 31) - 1;
    s = 0;
  }
  if (s < 0 || s > 31) return fail(RELAY_ERR_SHAPE, "scale must lie in (2^-32, 1)");
  *mult = (int32_t)M;
  *rshift = s;
  return RELAY_OK;
}

static relay_status qconv_common(const relay_conv2d_desc* d, const int8_t* x, const int8_t* w_packed, const int32_t* bias,
                                 const int8_t* residual, int32_t residual_lshift, int32_t out_rshift, int32_t round_mode,
                                 uint64_t seed, int qmode, const int32_t* qmult, const int32_t* qshift, int clip_lo,
                                 int clip_hi, void* y, void* workspace, size_t workspace_bytes, void* hip_stream) {
  int ho, wo;
  relay_status st = check_geometry(d, &ho, &wo);
  if (st != RELAY_OK) return st;
  if (d->dtype != RELAY_I8) return fail(RELAY_ERR_DTYPE, "quantized conv2d takes I8");
  if (d->flags & RELAY_HAS_BN) return fail(RELAY_ERR_UNSUPPORTED, "the quantized epilogue has no float scale/shift");
  if (!x || !w_packed || !y) return fail(RELAY_ERR_NULL, "x, w_packed and y are required");
  if ((st = check_optional(bias, d->flags & RELAY_HAS_BIAS, "bias")) != RELAY_OK) return st;
  if ((st = check_optional(residual, d->flags & RELAY_HAS_RESIDUAL, "residual")) != RELAY_OK) return st;
  if (out_rshift < 0 || out_rshift > 31) return fail(RELAY_ERR_UNSUPPORTED, "out_rshift=%d outside 0..31", out_rshift);
  if (residual_lshift < 0 || residual_lshift > 23)
    return fail(RELAY_ERR_UNSUPPORTED, "residual_lshift=%d outside 0..23", residual_lshift);
  if (round_mode < RELAY_ROUND_NEAREST || round_mode > RELAY_ROUND_STOCHASTIC)
    return fail(RELAY_ERR_UNSUPPORTED, "round_mode=%d is not a relay_round_mode", round_mode);
  if (y == x || y == residual) return fail(RELAY_ERR_UNSUPPORTED, "output must not alias an input");
  if ((st = check_igemm_support(d)) != RELAY_OK) return st;
  if (!aligned(x, 16) || !aligned(w_packed, 16) || !aligned(y, 8) || (residual && !aligned(residual, 8)) ||
      (bias && !aligned(bias, 4)))
    return fail(RELAY_ERR_ALIGN, "int8 x / w_packed must be 16-byte aligned, y / residual 8-byte, bias 4-byte aligned");
  relay::ConvArgs a = make_args(d, ho, wo);
  a.x = x; a.w = w_packed; a.y = y; a.res = residual; a.qbias = bias;
  a.lshift = residual_lshift; a.rshift = out_rshift;
  a.round_mode = round_mode; a.seed_lo = (unsigned)seed; a.seed_hi = (unsigned)(seed >> 32);
  a.round_add = out_rshift == 0 ? 0
                : round_mode == RELAY_ROUND_NEAREST ? 1 << (out_rshift - 1)
                : round_mode == RELAY_ROUND_CEIL ? (int)((1u << out_rshift) - 1u) : 0;
  a.qmode = qmode; a.qmult = qmult; a.qshift = qshift; a.clip_lo = clip_lo; a.clip_hi = clip_hi;
  finish_args(a);
  if ((st = use_workspace(a, true, workspace, workspace_bytes)) != RELAY_OK) return st;
  return device_status(launch_igemm(a, true, static_cast<hipStream_t>(hip_stream)), "qconv2d launch");
}

// ---- conv2d + 3x3 / stride 2 / pad 1 max pool in one launch -------------------------------------

static relay_status check_pool_fusable(const relay_conv2d_desc* d, int* ho, int* wo, relay::ConvArgs* out) {
  relay_status st = check_geometry(d, ho, wo);
  if (st != RELAY_OK) return st;
  if (d->dtype != RELAY_F16 && d->dtype != RELAY_I8) return fail(RELAY_ERR_DTYPE, "the pooled conv2d takes F16 or I8");
  if (d->flags & RELAY_HAS_RESIDUAL) return fail(RELAY_ERR_UNSUPPORTED, "the pooled conv2d has no residual operand");
  if (d->dtype == RELAY_I8 && (d->flags & RELAY_HAS_BN))
    return fail(RELAY_ERR_UNSUPPORTED, "the quantized epilogue has no float scale/shift");
  if ((st = check_igemm_support(d)) != RELAY_OK) return st;
  relay::ConvArgs a = make_args(d, *ho, *wo);
  if (!relay::igemm_dma_pool_supported(a, d->dtype == RELAY_I8))
    return fail(RELAY_ERR_UNSUPPORTED,
                "the pooled conv2d needs a conv output of ho %% 14 == 0 and wo %% 16 == 0 and k %% 8 == 0 (ho=%d wo=%d k=%d)",
                *ho, *wo, d->k);
  relay::fill_pool_args(a);
  *out = a;
  return RELAY_OK;
}

relay_status relay_conv2d_maxpool_fusable(const relay_conv2d_desc* d, int32_t* fusable) {
  if (!fusable) return fail(RELAY_ERR_NULL, "fusable is NULL");
  int ho, wo;
  relay::ConvArgs a;
  *fusable = check_pool_fusable(d, &ho, &wo, &a) == RELAY_OK ? 1 : 0;
  return RELAY_OK;
}

relay_status relay_conv2d_maxpool_kernel_name(const relay_conv2d_desc* d, char* buf, size_t len) {
  if (!buf || len == 0) return fail(RELAY_ERR_NULL, "name buffer is NULL or empty");
  int ho, wo;
  relay::ConvArgs a;
  const relay_status st = check_pool_fusable(d, &ho, &wo, &a);
  if (st != RELAY_OK) return st;
  relay::igemm_dma_pool_kernel_name(d->dtype == RELAY_I8, buf, len);
  return RELAY_OK;
}

relay_status relay_fused_conv2d_bn_relu_maxpool(const relay_conv2d_desc* d, const void* x, const void* w_packed,
                                                const float* bias, const float* bn_scale, const float* bn_shift,
                                                void* y_pooled, void* hip_stream) {
  int ho, wo;
  relay::ConvArgs a;
  relay_status st = check_pool_fusable(d, &ho, &wo, &a);
  if (st != RELAY_OK) return st;
  if (d->dtype != RELAY_F16) return fail(RELAY_ERR_DTYPE, "the float pooled conv2d takes F16");
  if (!x || !w_packed || !y_pooled) return fail(RELAY_ERR_NULL, "x, w_packed and y_pooled are required");
  if ((st = check_optional(bias, d->flags & RELAY_HAS_BIAS, "bias")) != RELAY_OK) return st;
  if ((st = check_optional(bn_scale, d->flags & RELAY_HAS_BN, "bn_scale")) != RELAY_OK) return st;
  if ((st = check_optional(bn_shift, d->flags & RELAY_HAS_BN, "bn_shift")) != RELAY_OK) return st;
  if (y_pooled == x) return fail(RELAY_ERR_UNSUPPORTED, "output must not alias an input");
  if (!aligned(x, 16) || !aligned(w_packed, 16) || !aligned(y_pooled, 16))
    return fail(RELAY_ERR_ALIGN, "fp16 tensors must be 16-byte aligned");
  a.x = x; a.w = w_packed; a.y = y_pooled; a.bias = bias; a.scale = bn_scale; a.shift = bn_shift;
  finish_args(a);
  return device_status(relay::launch_conv_igemm_dma_pool(a, false, static_cast<hipStream_t>(hip_stream)),
                       "pooled conv2d fp16 launch");
}

relay_status relay_qconv2d_requant_maxpool(const relay_conv2d_desc* d, const int8_t* x, const int8_t* w_packed,
                                           const int32_t* bias, int32_t out_rshift, int8_t* y_pooled,
                                           void* hip_stream) {
  int ho, wo;
  relay::ConvArgs a;
  relay_status st = check_pool_fusable(d, &ho, &wo, &a);
  if (st != RELAY_OK) return st;
  if (d->dtype != RELAY_I8) return fail(RELAY_ERR_DTYPE, "the quantized pooled conv2d takes I8");
  if (!x || !w_packed || !y_pooled) return fail(RELAY_ERR_NULL, "x, w_packed and y_pooled are required");
  if ((st = check_optional(bias, d->flags & RELAY_HAS_BIAS, "bias")) != RELAY_OK) return st;
  if (out_rshift < 0 || out_rshift > 31) return fail(RELAY_ERR_UNSUPPORTED, "out_rshift=%d outside 0..31", out_rshift);
  if (y_pooled == x) return fail(RELAY_ERR_UNSUPPORTED, "output must not alias an input");
  if (!aligned(x, 16) || !aligned(w_packed, 16) || !aligned(y_pooled, 8) || (bias && !aligned(bias, 4)))
    return fail(RELAY_ERR_ALIGN, "int8 x / w_packed must be 16-byte aligned, y_pooled 8-byte, bias 4-byte aligned");
  a.x = x; a.w = w_packed; a.y = y_pooled; a.qbias = bias;
  a.rshift = out_rshift;
  a.round_mode = RELAY_ROUND_NEAREST;
  a.round_add = out_rshift == 0 ? 0 : 1 << (out_rshift - 1);
  finish_args(a);
  return device_status(relay::launch_conv_igemm_dma_pool(a, true, static_cast<hipStream_t>(hip_stream)),
                       "pooled qconv2d launch");
}

static relay_status check_dw(const relay_conv2d_desc* d, int* ho, int* wo) {
  relay_status st = check_geometry(d, ho, wo);
  if (st != RELAY_OK) return st;
  if (d->dtype != RELAY_F16) return fail(RELAY_ERR_DTYPE, "depthwise conv2d takes F16");
  if (d->layout != RELAY_NHWC) return fail(RELAY_ERR_UNSUPPORTED, "depthwise conv2d needs NHWC activations");
  if (d->k != d->c) return fail(RELAY_ERR_SHAPE, "depthwise conv2d needs k == c (k=%d c=%d)", d->k, d->c);
  if (d->c % 8) return fail(RELAY_ERR_ALIGN, "c=%d must be a multiple of 8", d->c);
  if (d->r != 3 || d->s != 3) return fail(RELAY_ERR_UNSUPPORTED, "depthwise kernel must be 3x3");
  if (d->stride_h != d->stride_w || (d->stride_h != 1 && d->stride_h != 2))
    return fail(RELAY_ERR_UNSUPPORTED, "depthwise stride must be 1 or 2");
  if (d->flags & RELAY_HAS_RESIDUAL) return fail(RELAY_ERR_UNSUPPORTED, "depthwise conv2d has no residual input");
  if ((long)d->n * d->h * d->w * d->c * 2 > 0x7fffffffL)  // 32-bit buffer offsets, 2^31 marks "out of range"
    return fail(RELAY_ERR_SHAPE, "depthwise input exceeds 2^31-1 bytes");
  return RELAY_OK;
}

relay_status relay_prepack_dwconv_weights(const relay_conv2d_desc* d, const void* w_crs, void* w_rsc,
                                          void* hip_stream) {
  int ho, wo;
  relay_status st = check_dw(d, &ho, &wo);
  if (st != RELAY_OK) return st;
  if (!w_crs || !w_rsc) return fail(RELAY_ERR_NULL, "weight pointer is NULL");
  if (!aligned(w_rsc, 16)) return fail(RELAY_ERR_ALIGN, "w_rsc must be 16-byte aligned");
  return device_status(relay::launch_pack_dw_filters(w_crs, w_rsc, d->c, d->r * d->s, static_cast<hipStream_t>(hip_stream)),
                       "depthwise filter packing");
}

relay_status relay_fused_dwconv_bias_relu(const relay_conv2d_desc* d, const void* x, const void* w_rsc,
                                          const float* bias, const float* bn_scale, const float* bn_shift,
                                          void* y, void* hip_stream) {
  int ho, wo;
  relay_status st = check_dw(d, &ho, &wo);
  if (st != RELAY_OK) return st;
  if (!x || !w_rsc || !y) return fail(RELAY_ERR_NULL, "x, w_rsc and y are required");
  if ((st = check_optional(bias, d->flags & RELAY_HAS_BIAS, "bias")) != RELAY_OK) return st;
  if ((st = check_optional(bn_scale, d->flags & RELAY_HAS_BN, "bn_scale")) != RELAY_OK) return st;
  if ((st = check_optional(bn_shift, d->flags & RELAY_HAS_BN, "bn_shift")) != RELAY_OK) return st;
  if (y == x) return fail(RELAY_ERR_UNSUPPORTED, "output must not alias an input");
  if (!aligned(x, 16) || !aligned(w_rsc, 16) || !aligned(y, 16)) return fail(RELAY_ERR_ALIGN, "fp16 tensors must be 16-byte aligned");
  relay::ConvArgs a = make_args(d, ho, wo);
  a.x = x; a.w = w_rsc; a.y = y; a.bias = bias; a.scale = bn_scale; a.shift = bn_shift;
  return device_status(relay::launch_dwconv_f16(a, static_cast<hipStream_t>(hip_stream)), "depthwise launch");
}

// validation and kernel arguments shared by the fused depthwise + 1x1 entry point and its query (pointers may be NULL in the query)
static relay_status dwpw_args(const relay_conv2d_desc* dw, int32_t k, uint32_t pw_flags, relay::DwPwArgs* out) {
  int ho, wo;
  relay_status st = check_dw(dw, &ho, &wo);
  if (st != RELAY_OK) return st;
  if (dw->pad_h != 1 || dw->pad_w != 1) return fail(RELAY_ERR_UNSUPPORTED, "the fused depthwise + 1x1 kernel takes padding 1");
  if (dw->c % 32) return fail(RELAY_ERR_UNSUPPORTED, "c=%d must be a multiple of 32", dw->c);
  if (k <= 0 || k % 8) return fail(RELAY_ERR_SHAPE, "k=%d must be a positive multiple of 8", k);
  if (pw_flags & ~(RELAY_HAS_BIAS | RELAY_HAS_BN | RELAY_RELU))
    return fail(RELAY_ERR_UNSUPPORTED, "the 1x1 conv takes bias, scale/shift and relu only (flags=0x%x)", pw_flags);
  if ((long)dw->n * ho * wo * k > kMaxElems) return fail(RELAY_ERR_SHAPE, "output exceeds 2^31-1 elements");
  relay_conv2d_desc pd;
  memset(&pd, 0, sizeof(pd));
  pd.n = dw->n; pd.c = dw->c; pd.h = ho; pd.w = wo; pd.k = k; pd.r = pd.s = 1;
  pd.stride_h = pd.stride_w = 1;
  pd.dtype = RELAY_F16; pd.layout = RELAY_NHWC; pd.flags = pw_flags;
  relay::DwPwArgs& a = *out;
  memset(&a, 0, sizeof(a));
  a.dw_flags = dw->flags;
  a.N = dw->n; a.H = dw->h; a.W = dw->w; a.C = dw->c; a.Ho = ho; a.Wo = wo; a.stride = dw->stride_h;
  a.pw = make_args(&pd, ho, wo);
  return RELAY_OK;
}

relay_status relay_dwconv_pwconv_fusion_pays(const relay_conv2d_desc* dw, int32_t k, int32_t* pays) {
  if (!pays) return fail(RELAY_ERR_NULL, "pays is NULL");
  relay::DwPwArgs a;
  const relay_status st = dwpw_args(dw, k, 0, &a);
  if (st != RELAY_OK) return st;
  *pays = relay::dwpw_pick(a) >= 0 ? 1 : 0;
  return RELAY_OK;
}

relay_status relay_dwconv_pwconv_kernel_name(const relay_conv2d_desc* dw, int32_t k, char* buf, size_t len) {
  if (!buf || len == 0) return fail(RELAY_ERR_NULL, "name buffer is NULL or empty");
  relay::DwPwArgs a;
  const relay_status st = dwpw_args(dw, k, 0, &a);
  if (st != RELAY_OK) return st;
  const int variant = g_force_tile >= kDwPwBase ? g_force_tile - kDwPwBase : relay::dwpw_any(a);
  if (variant < 0 || !relay::dwpw_supported(a, variant))
    return fail(RELAY_ERR_UNSUPPORTED, "no fused depthwise + 1x1 kernel variant takes this shape (variant %d)", variant);
  relay::dwpw_kernel_name(variant, buf, len);
  return RELAY_OK;
}

relay_status relay_fused_dwconv_pwconv(const relay_conv2d_desc* dw, const void* x, const void* dw_w_rsc, const float* dw_bias,
                                       const float* dw_scale, const float* dw_shift, int32_t k, uint32_t pw_flags,
                                       const void* pw_w_packed, const float* pw_bias, const float* pw_scale,
                                       const float* pw_shift, void* y, void* hip_stream) {
  relay::DwPwArgs a;
  relay_status st = dwpw_args(dw, k, pw_flags, &a);
  if (st != RELAY_OK) return st;
  if (!x || !dw_w_rsc || !pw_w_packed || !y) return fail(RELAY_ERR_NULL, "x, dw_w_rsc, pw_w_packed and y are required");
  if ((st = check_optional(dw_bias, dw->flags & RELAY_HAS_BIAS, "dw_bias")) != RELAY_OK) return st;
  if ((st = check_optional(dw_scale, dw->flags & RELAY_HAS_BN, "dw_scale")) != RELAY_OK) return st;
  if ((st = check_optional(dw_shift, dw->flags & RELAY_HAS_BN, "dw_shift")) != RELAY_OK) return st;
  if ((st = check_optional(pw_bias, pw_flags & RELAY_HAS_BIAS, "pw_bias")) != RELAY_OK) return st;
  if ((st = check_optional(pw_scale, pw_flags & RELAY_HAS_BN, "pw_scale")) != RELAY_OK) return st;
  if ((st = check_optional(pw_shift, pw_flags & RELAY_HAS_BN, "pw_shift")) != RELAY_OK) return st;
  if (y == x) return fail(RELAY_ERR_UNSUPPORTED, "output must not alias an input");
  if (!aligned(x, 16) || !aligned(dw_w_rsc, 16) || !aligned(pw_w_packed, 16) || !aligned(y, 16))
    return fail(RELAY_ERR_ALIGN, "fp16 tensors must be 16-byte aligned");
  a.x = x; a.dw_w = dw_w_rsc; a.dw_bias = dw_bias; a.dw_scale = dw_scale; a.dw_shift = dw_shift;
  a.pw.w = pw_w_packed; a.pw.y = y; a.pw.bias = pw_bias; a.pw.scale = pw_scale; a.pw.shift = pw_shift;
  finish_args(a.pw);
  const int variant = g_force_tile >= kDwPwBase ? g_force_tile - kDwPwBase : relay::dwpw_any(a);
  if (variant < 0 || !relay::dwpw_supported(a, variant))
    return fail(RELAY_ERR_UNSUPPORTED, "no fused depthwise + 1x1 kernel variant takes this shape (variant %d)", variant);
  return device_status(relay::launch_dwpw(a, variant, static_cast<hipStream_t>(hip_stream)), "depthwise + 1x1 launch");
}

relay_status relay_fused_dense_bias_act(int32_t m, int32_t n, int32_t k, int32_t dtype, const void* x,
                                        const void* w, const float* bias, int32_t act, void* y,
                                        void* hip_stream) {
  if (m <= 0 || n <= 0 || k <= 0) return fail(RELAY_ERR_SHAPE, "non-positive extent (m=%d n=%d k=%d)", m, n, k);
  if (dtype != RELAY_F16 && dtype != RELAY_F32) return fail(RELAY_ERR_DTYPE, "dense takes F16 or F32");
  if (act != 0 && act != 1) return fail(RELAY_ERR_UNSUPPORTED, "act=%d (0 none, 1 relu)", act);
  if (!x || !w || !y) return fail(RELAY_ERR_NULL, "x, w and y are required");
  if ((long)m * k > kMaxElems || (long)n * k > kMaxElems || (long)m * n > kMaxElems)
    return fail(RELAY_ERR_SHAPE, "tensor exceeds 2^31-1 elements");
  const int ve = dtype == RELAY_F16 ? 8 : 4;
  if (k % ve) return fail(RELAY_ERR_ALIGN, "k=%d must be a multiple of %d", k, ve);
  if (!aligned(x, 16) || !aligned(w, 16) || !aligned(y, dtype == RELAY_F16 ? 2 : 4))
    return fail(RELAY_ERR_ALIGN, "x and w must be 16-byte aligned");
  if (y == x || y == w) return fail(RELAY_ERR_UNSUPPORTED, "output must not alias an input");
  if (dtype == RELAY_F16 && m >= 16 && k % 64 == 0) {
    // With a batch, dense is a 1x1 convolution over m one-pixel images; a weight row of whole
    // 128-byte groups is already the packed filter layout, so the MFMA kernel takes it as is.
    relay_conv2d_desc d;
    memset(&d, 0, sizeof(d));
    d.n = m; d.c = k; d.h = 1; d.w = 1; d.k = n; d.r = 1; d.s = 1;
    d.stride_h = d.stride_w = 1;
    d.dtype = RELAY_F16; d.layout = RELAY_NHWC;
    d.flags = (bias ? RELAY_HAS_BIAS : 0u) | (act == 1 ? RELAY_RELU : 0u);
    relay::ConvArgs a = make_args(&d, 1, 1);
    a.x = x; a.w = w; a.y = y; a.bias = bias;
    finish_args(a);
    if (relay::igemm_dma_supported(a, false))
      return device_status(relay::launch_conv_igemm_dma(a, false, -1, static_cast<hipStream_t>(hip_stream)),
                           "dense launch");
  }
  return device_status(relay::launch_dense(m, n, k, dtype == RELAY_F16, x, w, bias, act, y, static_cast<hipStream_t>(hip_stream)),
                       "dense launch");
}

relay_status relay_elementwise_f16(int32_t op, int64_t n_pixels, int32_t c, const void* x, const float* p0,
                                   const float* p1, const void* other, void* y, void* hip_stream) {
  if (op < RELAY_EW_BIAS_ADD || op > RELAY_EW_RELU) return fail(RELAY_ERR_UNSUPPORTED, "op=%d is not a relay_elementwise_op", op);
  if (n_pixels <= 0 || c <= 0 || n_pixels * c > kMaxElems) return fail(RELAY_ERR_SHAPE, "bad extent (n_pixels=%lld c=%d)", (long long)n_pixels, c);
  if (c % 8) return fail(RELAY_ERR_ALIGN, "c=%d must be a multiple of 8", c);
  if (!x || !y) return fail(RELAY_ERR_NULL, "x and y are required");
  const bool need_p0 = op == RELAY_EW_BIAS_ADD || op == RELAY_EW_SCALE_SHIFT, need_p1 = op == RELAY_EW_SCALE_SHIFT,
             need_other = op == RELAY_EW_ADD;
  if ((p0 != nullptr) != need_p0 || (p1 != nullptr) != need_p1 || (other != nullptr) != need_other)
    return fail(RELAY_ERR_NULL, "operands of op %d: p0 %s, p1 %s, other %s", op, need_p0 ? "required" : "must be NULL",
                need_p1 ? "required" : "must be NULL", need_other ? "required" : "must be NULL");
  if (!aligned(x, 16) || !aligned(y, 16) || (other && !aligned(other, 16)))
    return fail(RELAY_ERR_ALIGN, "fp16 tensors must be 16-byte aligned");
  return device_status(relay::launch_elementwise_f16(op, n_pixels, c, x, p0, p1, other, y, static_cast<hipStream_t>(hip_stream)),
                       "elementwise launch");
}

static relay_status check_quantize(int64_t n, const void* x, const void* y, float rho, int beta, int max_beta, int sigma,
                                   int round_mode) {
  if (n <= 0 || n > ((int64_t)1 << 40)) return fail(RELAY_ERR_SHAPE, "n_elems=%lld outside 1..2^40", (long long)n);
  if (!x || !y) return fail(RELAY_ERR_NULL, "x and y are required");
  if (!(rho > 0.f) || rho > 3.0e38f) return fail(RELAY_ERR_SHAPE, "rho must be positive and finite");
  if (beta < 2 || beta > max_beta) return fail(RELAY_ERR_UNSUPPORTED, "beta=%d outside 2..%d", beta, max_beta);
  if (sigma < 0 || sigma > beta) return fail(RELAY_ERR_UNSUPPORTED, "sigma=%d outside 0..beta", sigma);
  if (round_mode < RELAY_ROUND_NEAREST || round_mode > RELAY_ROUND_STOCHASTIC)
    return fail(RELAY_ERR_UNSUPPORTED, "round_mode=%d is not a relay_round_mode", round_mode);
  if (x == y) return fail(RELAY_ERR_UNSUPPORTED, "output must not alias the input");
  return RELAY_OK;
}

relay_status relay_quantize(int64_t n_elems, int32_t src_dtype, const void* x, float rho, int32_t beta, int32_t sigma,
                            int32_t round_mode, uint64_t seed, int8_t* y, void* hip_stream) {
  if (src_dtype != RELAY_F32 && src_dtype != RELAY_F16) return fail(RELAY_ERR_DTYPE, "quantize takes F32 or F16 input");
  relay_status st = check_quantize(n_elems, x, y, rho, beta, 8, sigma, round_mode);
  if (st != RELAY_OK) return st;
  if (!aligned(x, 16) || !aligned(y, 8)) return fail(RELAY_ERR_ALIGN, "x must be 16-byte and y 8-byte aligned");
  return device_status(relay::launch_quantize(src_dtype == RELAY_F16, n_elems, x, rho, beta, sigma, round_mode,
                                              (unsigned)seed, (unsigned)(seed >> 32), y,
                                              static_cast<hipStream_t>(hip_stream)),
                       "quantize launch");
}

relay_status relay_sim_quantize(int64_t n_elems, const float* x, float rho, int32_t beta, int32_t sigma,
                                int32_t round_mode, uint64_t seed, float* y, void* hip_stream) {
  relay_status st = check_quantize(n_elems, x, y, rho, beta, 24, sigma, round_mode);
  if (st != RELAY_OK) return st;
  if (!aligned(x, 16) || !aligned(y, 16)) return fail(RELAY_ERR_ALIGN, "x and y must be 16-byte aligned");
  return device_status(relay::launch_sim_quantize(n_elems, x, rho, beta, sigma, round_mode, (unsigned)seed,
                                                  (unsigned)(seed >> 32), y, static_cast<hipStream_t>(hip_stream)),
                       "sim_quantize launch");
}

relay_status relay_calibrate_pow2_range(int32_t dtype, int64_t n_elems, const void* x, float* rho_out, void* cell,
                                        void* hip_stream) {
  if (dtype != RELAY_F32 && dtype != RELAY_F16) return fail(RELAY_ERR_DTYPE, "calibration takes F32 or F16 tensors");
  if (n_elems <= 0 || n_elems > ((int64_t)1 << 40)) return fail(RELAY_ERR_SHAPE, "n_elems=%lld outside 1..2^40", (long long)n_elems);
  if (!x || !rho_out || !cell) return fail(RELAY_ERR_NULL, "x, rho_out and cell are required");
  if (!aligned(x, esize_of(dtype)) || !aligned(rho_out, 4) || !aligned(cell, 4))
    return fail(RELAY_ERR_ALIGN, "pointers must be aligned to their element size");
  return device_status(relay::launch_pow2_range(esize_of(dtype), n_elems, x, rho_out, static_cast<unsigned*>(cell),
                                                static_cast<hipStream_t>(hip_stream)),
                       "range calibration");
}

static_assert(sizeof(relay_realized_conv) == sizeof(relay::RealizedConv), "public and internal result records differ");
static_assert((int)RELAY_REALIZE_BAD_OUT_SHIFT == (int)relay::REALIZE_BAD_OUT_SHIFT &&
                  (int)RELAY_REALIZE_BAD_RES_SHIFT == (int)relay::REALIZE_BAD_RES_SHIFT &&
                  (int)RELAY_REALIZE_BIAS_OVERFLOW == (int)relay::REALIZE_BIAS_OVERFLOW,
              "public and internal status bits differ");

relay_status relay_realize_conv(int32_t k, int64_t per_k, const float* w, const float* bias, const float* scale,
                                const float* shift, float rho_x, float rho_y, float rho_res, int8_t* wq,
                                int32_t* bias_q, relay_realized_conv* out, void* workspace, size_t workspace_bytes,
                                void* hip_stream) {
  if (k <= 0 || per_k <= 0 || per_k > kMaxElems || (long)k * per_k > kMaxElems)
    return fail(RELAY_ERR_SHAPE, "bad filter extent (k=%d per_k=%lld)", k, (long long)per_k);
  if (!w || !wq || !out || !workspace) return fail(RELAY_ERR_NULL, "w, wq, out and workspace are required");
  if ((scale == nullptr) != (shift == nullptr)) return fail(RELAY_ERR_NULL, "scale and shift are given together or not at all");
  if ((bias || shift) && !bias_q) return fail(RELAY_ERR_NULL, "bias_q is required when the tail adds a bias or a shift");
  if (!(rho_x > 0.f) || !(rho_y > 0.f) || !(rho_res >= 0.f) || rho_x > 3.0e38f || rho_y > 3.0e38f || rho_res > 3.0e38f)
    return fail(RELAY_ERR_SHAPE, "ranges must be positive and finite (rho_res may be 0: no residual)");
  if (!aligned(w, 4) || !aligned(bias, 4) || !aligned(scale, 4) || !aligned(shift, 4) || !aligned(bias_q, 4) ||
      !aligned(out, 4) || !aligned(workspace, 16))
    return fail(RELAY_ERR_ALIGN, "fp32 / int32 pointers must be 4-byte and the workspace 16-byte aligned");
  const size_t need = (size_t)k * (size_t)per_k * 4 + 16;
  if (workspace_bytes < need) return fail(RELAY_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, need);
  if ((const void*)wq == (const void*)w) return fail(RELAY_ERR_UNSUPPORTED, "output must not alias an input");
  // layout of the workspace: the maximum's cell first (16 bytes), then the folded filters
  unsigned* cell = static_cast<unsigned*>(workspace);
  float* folded = reinterpret_cast<float*>(static_cast<char*>(workspace) + 16);
  return device_status(relay::launch_realize_conv(k, per_k, w, bias, scale, shift, rho_x, rho_y, rho_res, wq,
                                                  (bias || shift) ? bias_q : nullptr,
                                                  reinterpret_cast<relay::RealizedConv*>(out), folded, cell,
                                                  static_cast<hipStream_t>(hip_stream)),
                       "realize launch");
}

relay_status relay_probe_mfma(int32_t dtype, int32_t iters, int32_t workgroups, void* out, void* hip_stream) {
  if (dtype != RELAY_F16 && dtype != RELAY_I8) return fail(RELAY_ERR_DTYPE, "the matrix-instruction probe takes F16 or I8");
  if (iters < 1 || iters > (1 << 24) || workgroups < 1 || workgroups > (1 << 20))
    return fail(RELAY_ERR_SHAPE, "iters=%d workgroups=%d outside their ranges", iters, workgroups);
  if (!out) return fail(RELAY_ERR_NULL, "out is required");
  if (!aligned(out, 4)) return fail(RELAY_ERR_ALIGN, "out must be 4-byte aligned");
  return device_status(relay::launch_probe_mfma(dtype == RELAY_I8, iters, workgroups, static_cast<unsigned*>(out),
                                                static_cast<hipStream_t>(hip_stream)),
                       "probe launch");
}

relay_status relay_probe_grid_barrier(int32_t workgroups, int32_t rounds, uint32_t spin_limit, void* cells, void* data,
                                      void* hip_stream) {
  // every workgroup must be resident at once, or the first barrier could never complete: 256 threads, no
  // LDS to speak of, a handful of registers -- eight such workgroups fit a compute unit; four per unit
  // of the smallest chip this library is built for is the limit taken here
  if (workgroups < 1 || workgroups > 1024) return fail(RELAY_ERR_UNSUPPORTED, "workgroups=%d outside 1..1024", workgroups);
  if (rounds < 0 || rounds > (1 << 20)) return fail(RELAY_ERR_UNSUPPORTED, "rounds=%d outside 0..2^20", rounds);
  if (spin_limit < 1) return fail(RELAY_ERR_UNSUPPORTED, "spin_limit must be at least 1");
  if (!cells) return fail(RELAY_ERR_NULL, "cells is NULL");
  if (!aligned(cells, 4) || (data && !aligned(data, 4))) return fail(RELAY_ERR_ALIGN, "cells and data must be 4-byte aligned");
  return device_status(relay::launch_probe_grid_barrier(workgroups, rounds, spin_limit, static_cast<unsigned*>(cells),
                                                        static_cast<float*>(data), static_cast<hipStream_t>(hip_stream)),
                       "grid barrier probe launch");
}

relay_status relay_probe_copy(const void* src, void* dst, int64_t bytes, void* hip_stream) {
  if (!src || !dst) return fail(RELAY_ERR_NULL, "src and dst are required");
  if (bytes < 16 || bytes % 16 || bytes > ((int64_t)1 << 40)) return fail(RELAY_ERR_SHAPE, "bytes=%lld must be a multiple of 16 in 16..2^40", (long long)bytes);
  if (!aligned(src, 16) || !aligned(dst, 16)) return fail(RELAY_ERR_ALIGN, "src and dst must be 16-byte aligned");
  if (src == dst) return fail(RELAY_ERR_UNSUPPORTED, "output must not alias the input");
  return device_status(relay::launch_probe_copy(src, dst, bytes, static_cast<hipStream_t>(hip_stream)), "probe launch");
}

relay_status relay_fuse_extract(int32_t n_ops, const int32_t* pattern, const int32_t* in_offsets,
                                const int32_t* in_nodes, int32_t* ipdom, int32_t* group) {
  if (!pattern || !in_offsets || !group) return fail(RELAY_ERR_NULL, "pattern, in_offsets and group are required");
  if (n_ops < 1 || n_ops > (1 << 20)) return fail(RELAY_ERR_SHAPE, "n_ops=%d outside 1..2^20", n_ops);
  if (in_offsets[0] != 0) return fail(RELAY_ERR_SHAPE, "in_offsets[0] must be 0");
  for (int32_t i = 0; i < n_ops; ++i) {
    if (pattern[i] < RELAY_PATTERN_OPAQUE || pattern[i] > RELAY_PATTERN_CONTRACTION)
      return fail(RELAY_ERR_UNSUPPORTED, "operator %d has unknown pattern %d", i, pattern[i]);
    if (in_offsets[i + 1] < in_offsets[i]) return fail(RELAY_ERR_SHAPE, "in_offsets decreases at operator %d", i);
  }
  if (in_offsets[n_ops] > 0 && !in_nodes) return fail(RELAY_ERR_NULL, "in_nodes is NULL");
  for (int32_t i = 0; i < n_ops; ++i)
    for (int32_t e = in_offsets[i]; e < in_offsets[i + 1]; ++e)
      if (in_nodes[e] < 0 || in_nodes[e] >= i)
        return fail(RELAY_ERR_SHAPE, "operator %d reads operator %d: inputs must be earlier operators", i, in_nodes[e]);
  std::vector<int32_t> ip, gr;
  relay::fuse_extract(n_ops, pattern, in_offsets, in_nodes, ip, gr);
  for (int32_t i = 0; i < n_ops; ++i) {
    if (ipdom) ipdom[i] = ip[i];
    group[i] = gr[i];
  }
  return RELAY_OK;
}

relay_status relay_maxpool2d(int32_t dtype, int32_t n, int32_t c, int32_t h, int32_t w, int32_t r, int32_t stride,
                             int32_t pad, const void* x, void* y, void* hip_stream) {
  if (n <= 0 || c <= 0 || h <= 0 || w <= 0 || r <= 0 || stride <= 0 || pad < 0 || pad >= r || h + 2 * pad < r ||
      w + 2 * pad < r)
    return fail(RELAY_ERR_SHAPE, "bad pooling geometry");
  if (dtype != RELAY_F16 && dtype != RELAY_I8) return fail(RELAY_ERR_DTYPE, "maxpool takes F16 or I8");
  const int ve = dtype == RELAY_I8 ? 16 : 8;
  if (c % ve) return fail(RELAY_ERR_ALIGN, "c=%d must be a multiple of %d", c, ve);
  if (!x || !y) return fail(RELAY_ERR_NULL, "x and y are required");
  if (!aligned(x, 16) || !aligned(y, 16)) return fail(RELAY_ERR_ALIGN, "tensors must be 16-byte aligned");
  if ((long)n * c * h * w > kMaxElems) return fail(RELAY_ERR_SHAPE, "tensor exceeds 2^31-1 elements");
  const int ho = (h + 2 * pad - r) / stride + 1, wo = (w + 2 * pad - r) / stride + 1;
  return device_status(relay::launch_maxpool(dtype == RELAY_I8, n, c, h, w, r, stride, pad, ho, wo, x, y,
                                             static_cast<hipStream_t>(hip_stream)),
                       "maxpool launch");
}

relay_status relay_global_avgpool(int32_t dtype, int32_t n, int32_t c, int32_t hw, const void* x, void* y,
                                  void* hip_stream) {
  if (n <= 0 || c <= 0 || hw <= 0) return fail(RELAY_ERR_SHAPE, "non-positive extent");
  if (dtype != RELAY_F16) return fail(RELAY_ERR_DTYPE, "global average pool takes F16");
  if (c % 8) return fail(RELAY_ERR_ALIGN, "c=%d must be a multiple of 8", c);
  if (!x || !y) return fail(RELAY_ERR_NULL, "x and y are required");
  if (!aligned(x, 16) || !aligned(y, 16)) return fail(RELAY_ERR_ALIGN, "tensors must be 16-byte aligned");
  if ((long)n * c * hw > kMaxElems) return fail(RELAY_ERR_SHAPE, "tensor exceeds 2^31-1 elements");
  return device_status(relay::launch_avgpool_f16(n, c, hw, x, y, static_cast<hipStream_t>(hip_stream)), "avgpool launch");
}

relay_status relay_nchw_to_nhwc(int32_t dtype, int32_t n, int32_t c, int32_t h, int32_t w, int32_t c_pad,
                                const void* x, void* y, void* hip_stream) {
  if (n <= 0 || c <= 0 || h <= 0 || w <= 0 || c_pad < c) return fail(RELAY_ERR_SHAPE, "bad layout-conversion shape");
  const int es = esize_of(dtype);
  if (!es) return fail(RELAY_ERR_DTYPE, "unknown dtype %d", dtype);
  if (!x || !y) return fail(RELAY_ERR_NULL, "x and y are required");
  if (x == y) return fail(RELAY_ERR_UNSUPPORTED, "output must not alias an input");
  if ((long)n * c_pad * h * w > kMaxElems) return fail(RELAY_ERR_SHAPE, "tensor exceeds 2^31-1 elements");
  return device_status(relay::launch_nchw_to_nhwc(es, n, c, h, w, c_pad, x, y, static_cast<hipStream_t>(hip_stream)),
                       "layout conversion launch");
}

}  // extern "C"
