// Pieces shared by the implicit-GEMM conv kernels: MFMA wrappers, the LDS slot swizzle and
// the fused epilogues (float: paper Section 4.1; quantized: Section 4.2, "Realize").
#pragma once
#include "kernels.hpp"
#include "lds_dma.hpp"
#include "rounding.hpp"

namespace relay {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef int intx16 __attribute__((ext_vector_type(16)));

constexpr int BKV = 4;  // 16-byte k-vectors per tile row per chunk: 64 bytes of reduction

// LDS slot (in 16-byte units) of k-vector kv of a tile row.  The XOR spreads the 32 rows that
// one MFMA operand read (ds_read_b128: lanes 0-31 one k-vector of 32 rows, lanes 32-63 the
// next) touches over all banks: measured 126 B/clk/CU of the 128 B/clk LDS read peak, against
// 61 B/clk unswizzled and 111 B/clk with the row pair (row >> 1) as the key.
__device__ __forceinline__ int lds_swizzle(int row) { return (row >> 2) & (BKV - 1); }
__device__ __forceinline__ int lds_slot(int row, int kv) { return row * BKV + (kv ^ lds_swizzle(row)); }

template <bool IS_I8>
struct Mma;
template <>
struct Mma<false> {
  typedef floatx16 acc_t;
  typedef float scalar_t;
  static __device__ __forceinline__ acc_t mma(const uint4& a, const uint4& b, acc_t c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8, a), __builtin_bit_cast(half8, b), c, 0,
                                                  0, 0);
  }
};
template <>
struct Mma<true> {
  typedef intx16 acc_t;
  typedef int scalar_t;
  static __device__ __forceinline__ acc_t mma(const uint4& a, const uint4& b, acc_t c) {
    return __builtin_amdgcn_mfma_i32_32x32x32_i8(__builtin_bit_cast(intx4, a), __builtin_bit_cast(intx4, b), c, 0, 0,
                                                 0);
  }
};

// Per-channel epilogue constants of 4 consecutive channels.
//   float:  y = acc*mul + add   with mul = scale (or 1), add = bias*scale + shift
//   int8 :  acc += ibias
struct EpiParams {
  float mul[4], add[4];
  int ibias[4];
};

template <bool IS_I8>
__device__ __forceinline__ EpiParams load_epi_params(const ConvArgs& a, int ch) {
  EpiParams p;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int c = (ch + e < a.K) ? ch + e : a.K - 1;
    if constexpr (IS_I8) {
      p.ibias[e] = (a.flags & F_BIAS) ? a.qbias[c] : 0;
    } else {
      const float sc = (a.flags & F_BN) ? a.scale[c] : 1.f;
      const float sf = (a.flags & F_BN) ? a.shift[c] : 0.f;
      const float b = (a.flags & F_BIAS) ? a.bias[c] : 0.f;
      p.mul[e] = sc;
      p.add[e] = b * sc + sf;
    }
  }
  return p;
}

// Finish and store 4 consecutive channels [ch, ch+4) of output pixel m.
template <bool IS_I8, typename S>
__device__ __forceinline__ void epilogue_store4(const ConvArgs& a, const S (&v)[4], int m, int ch,
                                                const EpiParams& p, bool vec_ok) {
  const size_t o = (size_t)m * a.K + ch;
  if constexpr (!IS_I8) {
    float rs[4] = {0.f, 0.f, 0.f, 0.f};
    if (a.flags & F_RES) {
      const _Float16* rp = static_cast<const _Float16*>(a.res) + o;
      if (vec_ok) {
        const half4 rv = *reinterpret_cast<const half4*>(rp);
#pragma unroll
        for (int e = 0; e < 4; ++e) rs[e] = (float)rv[e];
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (ch + e < a.K) rs[e] = (float)rp[e];
      }
    }
    half4 hv;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float t = v[e] * p.mul[e] + p.add[e];
      t += rs[e];
      if (a.flags & F_RELU) t = t > 0.f ? t : 0.f;
      hv[e] = (_Float16)t;
    }
    _Float16* yp = static_cast<_Float16*>(a.y) + o;
    if (vec_ok) {
      *reinterpret_cast<half4*>(yp) = hv;
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (ch + e < a.K) yp[e] = hv[e];
    }
  } else {
    int rs[4] = {0, 0, 0, 0};
    if (a.flags & F_RES) {
      const int8_t* rp = static_cast<const int8_t*>(a.res) + o;
      if (vec_ok) {
        const unsigned rv = *reinterpret_cast<const unsigned*>(rp);
#pragma unroll
        for (int e = 0; e < 4; ++e) rs[e] = (int)(int8_t)(rv >> (8 * e));
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (ch + e < a.K) rs[e] = rp[e];
      }
    }
    int q[4];
    WordStream rng{a.seed_lo, a.seed_hi};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      int t = v[e] + p.ibias[e] + rs[e] * (1 << a.lshift);
      if (a.qmode == QMODE_SCALED) {
        const int c = ch + e < a.K ? ch + e : a.K - 1;
        t = scale_round(t, a.qmult[c], a.qshift[c]);
      } else {
        t = requant_shift(a.qmode == QMODE_ACC16 ? saturate16(t) : t, a.rshift, a.round_mode, rng, o + e);
      }
      t = t < a.clip_lo ? a.clip_lo : (t > a.clip_hi ? a.clip_hi : t);
      if (a.flags & F_RELU) t = t > 0 ? t : 0;
      q[e] = t;
    }
    int8_t* yp = static_cast<int8_t*>(a.y) + o;
    if (vec_ok) {
      *reinterpret_cast<unsigned*>(yp) = (unsigned)(q[0] & 0xff) | ((unsigned)(q[1] & 0xff) << 8) |
                                         ((unsigned)(q[2] & 0xff) << 16) | ((unsigned)(q[3] & 0xff) << 24);
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (ch + e < a.K) yp[e] = (int8_t)q[e];
    }
  }
}

}  // namespace relay
