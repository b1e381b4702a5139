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

}  // namespace relay
