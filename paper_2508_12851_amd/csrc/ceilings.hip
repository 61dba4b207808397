// Measured ceilings of the machine the library runs on, for measurement harnesses:
// the rate of a pure bf16 MFMA loop on caller-supplied operand values (the chip
// lowers its clock with the switching activity of the operands, so the ceiling
// for real data is below the one for constants) and the rate of a streaming read
// of a caller-supplied buffer.  Both only enqueue; the caller times them.
#include "prism_internal.h"

namespace prism {
namespace {

constexpr int kAcc = 8;   // independent accumulators per wavefront

__global__ __launch_bounds__(256) void mfma_loop_kernel(const bf16x8* __restrict__ operands,
                                                        float* __restrict__ out, int iters) {
  const size_t lane_id = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const bf16x8 a = operands[2 * lane_id], b = operands[2 * lane_id + 1];
  f32x16 acc[kAcc];
#pragma unroll
  for (int n = 0; n < kAcc; ++n)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[n][v] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int n = 0; n < kAcc; ++n)
      acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[n], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int n = 0; n < kAcc; ++n)
#pragma unroll
    for (int v = 0; v < 16; ++v) s += acc[n][v];
  out[lane_id] = s;
}

__global__ __launch_bounds__(256) void stream_read_kernel(const uint4* __restrict__ p, size_t n,
                                                          uint4* __restrict__ out) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  uint4 acc = {0, 0, 0, 0};
  for (; i + 3 * stride < n; i += 4 * stride) {
    const uint4 a = p[i], b = p[i + stride], c = p[i + 2 * stride], d = p[i + 3 * stride];
    acc.x ^= a.x ^ b.x ^ c.x ^ d.x; acc.y ^= a.y ^ b.y ^ c.y ^ d.y;
    acc.z ^= a.z ^ b.z ^ c.z ^ d.z; acc.w ^= a.w ^ b.w ^ c.w ^ d.w;
  }
  for (; i < n; i += stride) {
    const uint4 a = p[i];
    acc.x ^= a.x; acc.y ^= a.y; acc.z ^= a.z; acc.w ^= a.w;
  }
  // A data-dependent store keeps the loads alive without adding write traffic for the
  // usual all-zero source: a thread stores the xor of what it read only if that is not zero.
  if ((acc.x | acc.y | acc.z | acc.w) != 0) out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = acc;
}

}  // namespace
}  // namespace prism

using namespace prism;

extern "C" {
#pragma GCC visibility push(default)

prism_status prism_ceiling_mfma_bf16(const void* operands, float* out, int32_t n_workgroups,
                                     int32_t iters, double* flop, void* stream) {
  PRISM_ENTER();
  PRISM_RETURN_IF(operands == nullptr || out == nullptr || flop == nullptr, PRISM_ERR_INVALID_ARG);
  PRISM_RETURN_IF(n_workgroups < 1 || iters < 1, PRISM_ERR_INVALID_ARG);
  PRISM_RETURN_IF(((uintptr_t)operands & 15u) != 0, PRISM_ERR_INVALID_ARG);
  // 4 wavefronts per workgroup, kAcc MFMAs per iteration, 2 * 32 * 32 * 16 flop each
  *flop = (double)n_workgroups * 4.0 * (double)iters * kAcc * 32768.0;
  hipLaunchKernelGGL(mfma_loop_kernel, dim3(n_workgroups), dim3(256), 0, (hipStream_t)stream,
                     (const bf16x8*)operands, out, iters);
  PRISM_CHECK_LAUNCH();
  return PRISM_OK;
}

prism_status prism_ceiling_hbm_read(const void* src, size_t bytes, void* out, int32_t n_workgroups,
                                    void* stream) {
  PRISM_ENTER();
  PRISM_RETURN_IF(src == nullptr || out == nullptr, PRISM_ERR_INVALID_ARG);
  PRISM_RETURN_IF(n_workgroups < 1 || bytes < 16, PRISM_ERR_INVALID_ARG);
  PRISM_RETURN_IF(((uintptr_t)src & 15u) != 0 || ((uintptr_t)out & 15u) != 0, PRISM_ERR_INVALID_ARG);
  hipLaunchKernelGGL(stream_read_kernel, dim3(n_workgroups), dim3(256), 0, (hipStream_t)stream,
                     (const uint4*)src, bytes / 16, (uint4*)out);
  PRISM_CHECK_LAUNCH();
  return PRISM_OK;
}

#pragma GCC visibility pop
}  // extern "C"
