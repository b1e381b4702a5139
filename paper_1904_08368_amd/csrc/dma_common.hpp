// Pieces shared by the direct-to-LDS conv kernels: the global->LDS load, wait and descriptor
// helpers, the per-lane epilogue constants and the finish-and-store of 8 consecutive channels.
#pragma once
#include "igemm_common.hpp"
#include "lds_dma.hpp"

namespace relay {

// 32-bit pattern of an accumulator element (taken by value: a bit cast applied directly to a
// vector-element lvalue is not reliable)
__device__ __forceinline__ unsigned as_u32(float f) { return __builtin_bit_cast(unsigned, f); }
__device__ __forceinline__ unsigned as_u32(int i) { return (unsigned)i; }

// floor(t / d) and remainder for 0 <= t < 2^22, d > 0: float reciprocal plus one fix-up step.
__device__ __forceinline__ void small_divmod(int t, int d, float rcp_d, int& q, int& r) {
  q = (int)((float)t * rcp_d);
  r = t - q * d;
  const int fix = (r >= d ? 1 : 0) - (r < 0 ? 1 : 0);  // selects, not branches: lanes differ
  q += fix;
  r -= fix * d;
}

// Epilogue constants of the 8 consecutive channels [ech, ech + 8) a lane owns after the
// transposition.  float: y = acc*mul + add with mul = scale (or 1), add = bias*scale + shift;
// int8: acc += ibias.
struct LaneParams {
  float mul[8], add[8];
  int ibias[8];
};

// Where a lane's 8 channels [ech, ech + 8) are stored: the tensor, its pixel pitch (elements) and
// the position of channel ech inside a pixel of it.  Worked out after the main loop, so that it
// occupies no registers there.
struct OutLoc {
  void* y;
  int ldy;
  int cho;
  int norelu;  // the segment stays without relu although the flags ask for one
};

__device__ __forceinline__ OutLoc locate_output(const ConvArgs& a, int ech) {
  OutLoc ol{nullptr, 0, 0, 0};  // unused for the plain tensor: finish_store8 addresses that from the arguments
  if (a.nseg) {  // (uniform) which output segment holds the lane's channels
    int begin = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (i < a.nseg) {
        if (ech >= begin && ech < a.seg_end[i]) {
          ol.y = a.seg_y[i];
          ol.ldy = a.seg_ld[i];
          ol.cho = ech - begin;
          ol.norelu = (int)((a.seg_norelu >> i) & 1u);
        }
        begin = a.seg_end[i];
      }
  }
  return ol;
}

// The loads of a lane's epilogue constants, kept apart from the arithmetic on them so that a
// kernel can issue them ahead of its first ring loads and touch the values only after those
// have been issued: the global-memory latency of the constants is then covered by the issue of
// the ring loads instead of stalling the prologue.
struct RawLaneParams {
  float sc[8], sf[8], bb[8];
  int ib[8];
};

template <bool IS_I8>
__device__ __forceinline__ void fetch_lane_params(const ConvArgs& a, int ech, RawLaneParams& rp) {
  if (a.param_vec) {  // two 16-byte loads per array
    const int c8 = ech < a.K ? ech : a.K - 8;
    if constexpr (IS_I8) {
      int4 b0 = make_int4(0, 0, 0, 0), b1 = b0;
      if (a.flags & F_BIAS) {
        b0 = *reinterpret_cast<const int4*>(a.qbias + c8);
        b1 = *reinterpret_cast<const int4*>(a.qbias + c8 + 4);
      }
      const int t[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
#pragma unroll
      for (int e = 0; e < 8; ++e) rp.ib[e] = t[e];
    } else {
      float4 s0 = make_float4(1.f, 1.f, 1.f, 1.f), s1 = s0;
      float4 f0 = make_float4(0.f, 0.f, 0.f, 0.f), f1 = f0, b0 = f0, b1 = f0;
      if (a.flags & F_BN) {
        s0 = *reinterpret_cast<const float4*>(a.scale + c8);
        s1 = *reinterpret_cast<const float4*>(a.scale + c8 + 4);
        f0 = *reinterpret_cast<const float4*>(a.shift + c8);
        f1 = *reinterpret_cast<const float4*>(a.shift + c8 + 4);
      }
      if (a.flags & F_BIAS) {
        b0 = *reinterpret_cast<const float4*>(a.bias + c8);
        b1 = *reinterpret_cast<const float4*>(a.bias + c8 + 4);
      }
      const float sc[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
      const float sf[8] = {f0.x, f0.y, f0.z, f0.w, f1.x, f1.y, f1.z, f1.w};
      const float bb[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        rp.sc[e] = sc[e];
        rp.sf[e] = sf[e];
        rp.bb[e] = bb[e];
      }
    }
  } else {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int c = ech + e < a.K ? ech + e : a.K - 1;
      if constexpr (IS_I8) {
        rp.ib[e] = (a.flags & F_BIAS) ? a.qbias[c] : 0;
      } else {
        rp.sc[e] = (a.flags & F_BN) ? a.scale[c] : 1.f;
        rp.sf[e] = (a.flags & F_BN) ? a.shift[c] : 0.f;
        rp.bb[e] = (a.flags & F_BIAS) ? a.bias[c] : 0.f;
      }
    }
  }
}

template <bool IS_I8>
__device__ __forceinline__ void finish_lane_params(const RawLaneParams& rp, LaneParams& lp) {
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    if constexpr (IS_I8) {
      lp.ibias[e] = rp.ib[e];
    } else {
      lp.mul[e] = rp.sc[e];
      lp.add[e] = rp.bb[e] * rp.sc[e] + rp.sf[e];  // (acc + b)*sc + sf
    }
  }
}

template <bool IS_I8>
__device__ __forceinline__ void load_lane_params(const ConvArgs& a, int ech, LaneParams& lp) {
  RawLaneParams rp;
  fetch_lane_params<IS_I8>(a, ech, rp);
  finish_lane_params<IS_I8>(rp, lp);
}

// EXT: the instantiation that knows about output segments (the plain one ignores ol).
// Finish the 8 consecutive channels [ech, ech + 8) of output pixel m (its index in the NHWC output;
// residual and random draws are addressed in the plain [M][K] tensor, the store goes where ol says)
// from the raw accumulator bits and store them (bias, scale/shift, residual, relu, cast -- or the
// quantized epilogue, with STOCH the stochastic rounding).
// The 8 residual values of output element (m, ech..ech+7) as one vector load (fp16: 16 bytes; int8: 8 bytes
// in .x/.y); for epilogues that fetch all their residual operands ahead of the arithmetic, so that the
// loads are in flight together instead of one memory latency per stored vector.  K % 8 == 0 only.
template <bool IS_I8>
__device__ __forceinline__ uint4 load_residual8(const ConvArgs& a, int m, int ech) {
  const size_t o = (size_t)m * a.K + ech;
  if constexpr (IS_I8) {
    const uint2 v = *reinterpret_cast<const uint2*>(static_cast<const int8_t*>(a.res) + o);
    return make_uint4(v.x, v.y, 0u, 0u);
  } else {
    return *reinterpret_cast<const uint4*>(static_cast<const _Float16*>(a.res) + o);
  }
}

// have_pre: `pre` is the element's residual vector from load_residual8; else it is loaded here
template <bool IS_I8, bool STOCH, bool EXT = false>
__device__ __forceinline__ void finish_store8(const ConvArgs& a, const unsigned (&raw)[8], int m, int ech,
                                              const LaneParams& lp, const OutLoc& ol, bool vec_ok,
                                              bool have_pre = false, uint4 pre = uint4{0u, 0u, 0u, 0u}) {
  const float(&emul)[8] = lp.mul;
  const float(&eadd)[8] = lp.add;
  const int(&ebias)[8] = lp.ibias;
  const size_t o = (size_t)m * a.K + ech;
  const bool relu = (a.flags & F_RELU) && !(EXT && ol.norelu);
  if constexpr (!IS_I8) {
    // (as in the quantized tail every instruction counts: the residual enters through a mixed-precision
    // multiply-add -- 1.0 * r + t, the same sum as convert-then-add -- two results are narrowed by one packed
    // conversion, and relu is a packed maximum on the narrowed pair: rounding is monotone and keeps the
    // sign, so max(round(t), 0) == round(max(t, 0)), and the hardware's maximum of -0 and +0 is +0)
    typedef float float2v __attribute__((ext_vector_type(2)));
    typedef _Float16 half2v __attribute__((ext_vector_type(2)));
    float t[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) t[e] = __builtin_bit_cast(float, raw[e]) * emul[e] + eadd[e];
    if (a.flags & F_RES) {
      const _Float16* rp = static_cast<const _Float16*>(a.res) + o;
      if (vec_ok) {
        const uint4 rv = have_pre ? pre : *reinterpret_cast<const uint4*>(rp);
        const unsigned rw[4] = {rv.x, rv.y, rv.z, rv.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          asm("v_fma_mix_f32 %0, %1, 1.0, %0 op_sel:[0,0,0] op_sel_hi:[1,0,0]" : "+v"(t[2 * e]) : "v"(rw[e]));
          asm("v_fma_mix_f32 %0, %1, 1.0, %0 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "+v"(t[2 * e + 1]) : "v"(rw[e]));
        }
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (ech + e < a.K) t[e] += (float)rp[e];
      }
    }
    unsigned hw[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      asm("" : "+v"(t[2 * e]), "+v"(t[2 * e + 1]));   // (rounded to fp32 first, in every instantiation: never merged with the narrowing)
      const float2v f = {t[2 * e], t[2 * e + 1]};
      half2v h = __builtin_convertvector(f, half2v);
      if (relu) h = __builtin_elementwise_max(h, half2v{(_Float16)0, (_Float16)0});
      hw[e] = __builtin_bit_cast(unsigned, h);
    }
    _Float16* yp = static_cast<_Float16*>(a.y) + o;
    if constexpr (EXT)
      if (a.nseg) yp = static_cast<_Float16*>(ol.y) + ((size_t)m * ol.ldy + ol.cho);
    if (vec_ok) {
      *reinterpret_cast<uint4*>(yp) = make_uint4(hw[0], hw[1], hw[2], hw[3]);
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e)
        if (ech + e < a.K) yp[e] = __builtin_bit_cast(_Float16, (unsigned short)(hw[e >> 1] >> (16 * (e & 1))));
    }
  } else {
    int t[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) t[e] = (int)raw[e] + ebias[e];
    if (a.flags & F_RES) {
      const int8_t* rp = static_cast<const int8_t*>(a.res) + o;
      if (vec_ok) {
        const uint2 rv = have_pre ? make_uint2(pre.x, pre.y) : *reinterpret_cast<const uint2*>(rp);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          t[e] += (int)(int8_t)(rv.x >> (8 * e)) * (1 << a.lshift);
          t[4 + e] += (int)(int8_t)(rv.y >> (8 * e)) * (1 << a.lshift);
        }
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (ech + e < a.K) t[e] += (int)rp[e] * (1 << a.lshift);
      }
    }
    // Each scaling rule sits behind a uniform branch of its own, the default one first and at its
    // shortest.
    const ClipBounds cb = clip_bounds(a, relu);
    if constexpr (STOCH) {
      WordStream rng{a.seed_lo, a.seed_hi};
#pragma unroll
      for (int e = 0; e < 8; ++e)
        t[e] = clip_med3(requant_shift(t[e], a.rshift, ROUND_STOCHASTIC, rng, o + e), cb.lo, cb.hi);
    } else if (a.qmode == QMODE_SHIFT) {
      if (cb.sat_ok) {
#pragma unroll
        for (int e = 0; e < 8; ++e) t[e] = shift_round_clip<true>(t[e], a, cb);
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) t[e] = shift_round_clip<false>(t[e], a, cb);
      }
    } else if (a.qmode == QMODE_SCALED) {
      // the per-channel operands are fetched here, behind the main loop: nothing of this rule is
      // held in registers while the tile accumulates, and nothing of it runs under another rule
      int qm[8], qs[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        int c = ech + e < a.K ? ech + e : a.K - 1;
        asm volatile("" : "+v"(c));   // keeps the address arithmetic of this rule inside its branch
        qm[e] = a.qmult[c];
        qs[e] = a.qshift[c];
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) t[e] = clip_med3(scale_round(t[e], qm[e], qs[e]), cb.lo, cb.hi);
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) t[e] = shift_round_clip<false>(saturate16(t[e]), a, cb);
    }
    const unsigned pk[2] = {pack_low_bytes(t[0], t[1], t[2], t[3]), pack_low_bytes(t[4], t[5], t[6], t[7])};
    int8_t* yp = static_cast<int8_t*>(a.y) + o;
    if constexpr (EXT)
      if (a.nseg) yp = static_cast<int8_t*>(ol.y) + ((size_t)m * ol.ldy + ol.cho);
    if (vec_ok) {
      *reinterpret_cast<uint2*>(yp) = make_uint2(pk[0], pk[1]);
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e)
        if (ech + e < a.K) yp[e] = (int8_t)t[e];
    }
  }
}

}  // namespace relay
