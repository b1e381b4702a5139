// The multiply-add of the depthwise kernels: fp16 operands taken straight from the halves of 32-bit
// registers, fp32 accumulation (v_fma_mix_f32), no conversion instructions.
#pragma once
#include <hip/hip_runtime.h>

namespace relay {

// acc += x.lo*w.lo (fp16 halves of 32-bit registers), fp32 accumulate
__device__ __forceinline__ void fma_mix_lo(float& acc, unsigned x, unsigned w) {
  asm("v_fma_mix_f32 %0, %1, %2, %0 op_sel:[0,0,0] op_sel_hi:[1,1,0]" : "+v"(acc) : "v"(x), "v"(w));
}
__device__ __forceinline__ void fma_mix_hi(float& acc, unsigned x, unsigned w) {
  asm("v_fma_mix_f32 %0, %1, %2, %0 op_sel:[1,1,0] op_sel_hi:[1,1,0]" : "+v"(acc) : "v"(x), "v"(w));
}

// The fused tail of eight depthwise results: scale and shift in fp32, two results narrowed by one packed
// conversion, the lower bound (0 for relu, -infinity for none) applied to the narrowed pair by one packed
// maximum.  Rounding is monotone and keeps the sign, so this equals the bound applied before the
// narrowing; the hardware's maximum of -0 and +0 is +0.
__device__ __forceinline__ uint4 scale_shift_narrow8(const float (&acc)[8], const float (&mul)[8], const float (&add)[8],
                                                     float lo) {
  typedef float float2v __attribute__((ext_vector_type(2)));
  typedef _Float16 half2v __attribute__((ext_vector_type(2)));
  const half2v lo2 = {(_Float16)lo, (_Float16)lo};
  unsigned w[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    float f0 = acc[2 * e] * mul[2 * e] + add[2 * e], f1 = acc[2 * e + 1] * mul[2 * e + 1] + add[2 * e + 1];
    // (rounded to fp32 first in every kernel: left alone the compiler may merge a multiply-add and its narrowing
    // into one instruction that rounds once, in one kernel and not in another)
    asm("" : "+v"(f0), "+v"(f1));
    const float2v f = {f0, f1};
    w[e] = __builtin_bit_cast(unsigned, __builtin_elementwise_max(__builtin_convertvector(f, half2v), lo2));
  }
  return make_uint4(w[0], w[1], w[2], w[3]);
}

}  // namespace relay
