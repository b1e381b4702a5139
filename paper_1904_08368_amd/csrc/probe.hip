// Measured ceilings of the chip, for the roofline figures of the benchmark: a register-only loop of
// matrix instructions (what the matrix cores deliver when nothing feeds them from memory) and a
// streaming copy (what HBM delivers to a kernel with nothing else to do), and the cost of a barrier
// across all workgroups of a resident grid (what a kernel that runs several dependent layers in one
// launch would pay between them, to set beside the cost of a kernel boundary).  Not part of any fused
// primitive function; a profiler run of these gives the "measured peak" beside the nominal one.
#include "dma_common.hpp"

namespace relay {
namespace {

// Every wave runs `iters` rounds of four independent 32x32 matrix instructions on registers only.
template <bool IS_I8>
__global__ __launch_bounds__(256) void mfma_loop_kernel(int iters, unsigned* out) {
  typedef typename Mma<IS_I8>::acc_t acc_t;
  const unsigned seed = threadIdx.x * 2654435761u + blockIdx.x;
  uint4 a = make_uint4(seed, seed ^ 0x3c003c00u, 0x3c003c00u, 0x38003800u), b = make_uint4(0x3c003c00u, seed, 0x34003400u, 0x3c003c00u);
  if constexpr (!IS_I8) {   // keep the fp16 operands finite: exponent fields of small numbers
    a = make_uint4(0x2c002c00u | (seed & 0x03ff03ffu), 0x2c002c00u, 0x28002800u, 0x2c002c00u);
    b = make_uint4(0x2c002c00u, 0x28002800u | (seed & 0x03ff03ffu), 0x2c002c00u, 0x28002800u);
  }
  acc_t c0, c1, c2, c3;
#pragma unroll
  for (int v = 0; v < 16; ++v) c0[v] = c1[v] = c2[v] = c3[v] = 0;
  for (int i = 0; i < iters; ++i) {
    c0 = Mma<IS_I8>::mma(a, b, c0);
    c1 = Mma<IS_I8>::mma(b, a, c1);
    c2 = Mma<IS_I8>::mma(a, a, c2);
    c3 = Mma<IS_I8>::mma(b, b, c3);
  }
  unsigned s = 0;
#pragma unroll
  for (int v = 0; v < 16; ++v) s ^= as_u32(c0[v]) ^ as_u32(c1[v]) ^ as_u32(c2[v]) ^ as_u32(c3[v]);
  if (s == 0x12345678u) out[0] = s;   // (keeps the loop alive; practically never true)
}

__global__ __launch_bounds__(256) void stream_copy_kernel(const uint4* src, uint4* dst, long n16) {
  const long stride = (long)gridDim.x * 256;
  for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

// `rounds` barriers across the whole grid.  cells[0] counts arrivals (it only grows during a launch: round r
// is over once it reaches (r + 1) * workgroups), cells[1] is set when a wait ran out of its `spin_limit`
// polls, cells[2] counts workgroups that are done: the last one puts cells[0] and cells[2] back to zero for
// the next launch.  Arrival is a device-scope release (the L2s of the chip's dies are not coherent with each
// other) and an atomic add, the wait polls with device-scope loads and ends in an acquire -- what a layer
// boundary inside one launch needs.  data (or NULL): every thread adds to a word of its own before each
// barrier, so that the release has something to write back.  Every wait is bounded: a workgroup whose
// wait runs out raises the flag and leaves, and so, one after another, do the others.
__global__ __launch_bounds__(256) void grid_barrier_kernel(unsigned* cells, int rounds, unsigned spin_limit, float* data) {
  __shared__ int ok;
  const int tid = threadIdx.x;
  if (rounds == 0) return;   // an empty kernel: what a launch costs by itself (no counter is touched)
  for (int r = 0; r < rounds; ++r) {
    if (data) data[(size_t)blockIdx.x * 256 + tid] += 1.0f;
    __syncthreads();
    if (tid == 0) {
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
      atomicAdd(cells, 1u);
      const unsigned target = (unsigned)(r + 1) * gridDim.x;
      bool good = false;
      for (unsigned i = 0; i < spin_limit && !good; ++i) {
        good = __hip_atomic_load(cells, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= target;
        if (!good) __builtin_amdgcn_s_sleep(1);
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
      if (!good) atomicExch(cells + 1, 1u);
      ok = good;
    }
    __syncthreads();
    if (!ok) return;   // (the counters stay as they are: the caller clears them after a failed launch)
  }
  if (tid == 0 && atomicAdd(cells + 2, 1u) == gridDim.x - 1) {
    atomicExch(cells, 0u);
    atomicExch(cells + 2, 0u);
  }
}

}  // namespace

hipError_t launch_probe_grid_barrier(int workgroups, int rounds, unsigned spin_limit, unsigned* cells, float* data, hipStream_t st) {
  hipLaunchKernelGGL(grid_barrier_kernel, dim3(workgroups), dim3(256), 0, st, cells, rounds, spin_limit, data);
  return hipGetLastError();
}

hipError_t launch_probe_mfma(bool is_i8, int iters, int workgroups, unsigned* out, hipStream_t st) {
  if (is_i8) hipLaunchKernelGGL((mfma_loop_kernel<true>), dim3(workgroups), dim3(256), 0, st, iters, out);
  else hipLaunchKernelGGL((mfma_loop_kernel<false>), dim3(workgroups), dim3(256), 0, st, iters, out);
  return hipGetLastError();
}

hipError_t launch_probe_copy(const void* src, void* dst, long bytes, hipStream_t st) {
  hipLaunchKernelGGL(stream_copy_kernel, dim3(256 * 16), dim3(256), 0, st, static_cast<const uint4*>(src), static_cast<uint4*>(dst),
                     bytes / 16);
  return hipGetLastError();
}

}  // namespace relay
