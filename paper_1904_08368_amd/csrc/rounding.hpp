// Rounding strategies of the quantization flow (paper Section 4.2: nearest, floor, ceiling,
// stochastic) and the counter-based generator behind the stochastic one.
#pragma once
#include "kernels.hpp"

namespace relay {

// Philox-4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11): ten rounds of two 32x32->64 multiplies
// and a key schedule of two Weyl sequences.
__device__ __forceinline__ void philox4x32_10(unsigned c0, unsigned c1, unsigned c2, unsigned c3, unsigned k0,
                                              unsigned k1, unsigned (&out)[4]) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const unsigned hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
    const unsigned hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
    const unsigned n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
    c0 = n0;
    c1 = lo1;
    c2 = n2;
    c3 = lo0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0;
  out[1] = c1;
  out[2] = c2;
  out[3] = c3;
}

// The random word of tensor element `index`: word index%4 of the block with counter
// (index/4, 0, 0, 0).  `cache` holds the last block computed, so that the consecutive elements a
// lane finishes cost one block per four.
struct WordStream {
  unsigned k0, k1;
  unsigned long long block = ~0ull;
  unsigned w[4];
  __device__ __forceinline__ unsigned word(unsigned long long index) {
    const unsigned long long b = index >> 2;
    if (b != block) {
      block = b;
      philox4x32_10((unsigned)b, (unsigned)(b >> 32), 0u, 0u, k0, k1, w);
    }
    const unsigned j = (unsigned)index & 3u;
    return j == 0 ? w[0] : j == 1 ? w[1] : j == 2 ? w[2] : w[3];
  }
};

// floor((acc + addend) / 2^s) for 0 <= addend < 2^s and 0 <= s <= 31, without forming acc + addend:
// that sum can leave int32 (s near 31) although the quotient never does.  With acc = (acc >> s) * 2^s +
// (acc & (2^s - 1)) the low part plus the addend stays below 2^32.
__device__ __forceinline__ int shift_round(int acc, unsigned addend, int s) {
  const unsigned mask = (1u << s) - 1u;
  return (acc >> s) + (int)((((unsigned)acc & mask) + addend) >> s);
}

// round(acc * mult / 2^(31 + s)), ties toward +infinity: the requantization by a general scale
// mult / 2^31 * 2^-s (0 < mult < 2^31, 0 <= s <= 31).  |acc * mult| < 2^62 and the rounding addend
// is at most 2^61, so the 64-bit sum cannot overflow.
__device__ __forceinline__ int scale_round(int acc, int mult, int s) {
  const long long p = (long long)acc * (long long)mult + (1ll << (30 + s));
  return (int)(p >> (31 + s));
}

// the exact sum as a 16-bit accumulator holds it: saturated
__device__ __forceinline__ int saturate16(int acc) { return acc < -32768 ? -32768 : (acc > 32767 ? 32767 : acc); }

// q clipped to [lo, hi], lo <= hi: the median of the three, one instruction
__device__ __forceinline__ int clip_med3(int q, int lo, int hi) {
  int r;
  asm("v_med3_i32 %0, %1, %2, %3" : "=v"(r) : "v"(q), "v"(lo), "v"(hi));
  return r;
}

// the low bytes of four words in one: two byte permutes and an or
__device__ __forceinline__ unsigned pack_low_bytes(int q0, int q1, int q2, int q3) {
  return __builtin_amdgcn_perm((unsigned)q1, (unsigned)q0, 0x0c0c0400u) |
         __builtin_amdgcn_perm((unsigned)q3, (unsigned)q2, 0x04000c0cu);
}

// The bounds of the quantized tail with relu folded in as a raised lower bound, and whether a
// saturating add may stand in for the exact rounding: acc + addend leaves int32 only where the
// quotient is 2^(31 - s), and the saturated sum gives 2^(31 - s) - 1; once that is no smaller than
// the upper bound, the clip sends both to the same value.
struct ClipBounds {
  int lo, hi;
  bool sat_ok;
};
__device__ __forceinline__ ClipBounds clip_bounds(const ConvArgs& a, bool relu) {
  ClipBounds b;
  b.lo = relu ? (a.clip_lo > 0 ? a.clip_lo : 0) : a.clip_lo;
  b.hi = relu ? (a.clip_hi > 0 ? a.clip_hi : 0) : a.clip_hi;
  b.sat_ok = (0x7fffffff >> a.rshift) >= a.clip_hi;
  return b;
}

// round((acc + addend) / 2^s) of the deterministic rules, clipped.  SAT: only under ClipBounds::sat_ok.
// Every instruction here costs a wave four clocks per result with all waves of a tile in the tail
// at once, so the common case is kept to three.
template <bool SAT>
__device__ __forceinline__ int shift_round_clip(int acc, const ConvArgs& a, const ClipBounds& b) {
  const int q = SAT ? (__builtin_elementwise_add_sat(acc, a.round_add) >> a.rshift)
                    : shift_round(acc, (unsigned)a.round_add, a.rshift);
  return clip_med3(q, b.lo, b.hi);
}

// acc / 2^s rounded by `mode` (arithmetic shift = floor division): what is added before the shift.
__device__ __forceinline__ int requant_shift(int acc, int s, int mode, WordStream& rng, unsigned long long index) {
  if (s == 0) return acc;
  unsigned addend;
  if (mode == ROUND_NEAREST) addend = 1u << (s - 1);  // ties toward +infinity
  else if (mode == ROUND_FLOOR) addend = 0u;
  else if (mode == ROUND_CEIL) addend = (1u << s) - 1u;
  else addend = rng.word(index) & ((1u << s) - 1u);  // up with probability frac(acc / 2^s)
  return shift_round(acc, addend, s);
}

}  // namespace relay
