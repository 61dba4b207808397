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

// Streaming reads with the access pattern as parameters, to find what the memory system of the
// machine at hand serves fastest.  The source is cut into spans of span16 16-byte units; workgroup
// b takes spans b, b + gridDim.x, ... and walks each with its 256 threads, U loads of 16 bytes per
// thread in flight.  MODE 0: plain loads into registers; 1: direct-to-LDS loads (no register
// ever holds the data, as in the GEMM rings); 2: loads marked non-temporal; 3: direct-to-LDS
// loads marked non-temporal (kNonTemporal in the instruction's cache-policy operand).
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
template <int U, int MODE>
__global__ __launch_bounds__(256) void stream_pattern_kernel(const u32x4* __restrict__ p, size_t n_spans,
                                                             uint32_t span16, u32x4* __restrict__ out) {
#if defined(__HIP_DEVICE_COMPILE__)
  constexpr bool kLds = MODE == 1 || MODE == 3;
  __shared__ __align__(16) uint8_t s_sink[kLds ? 4 * U * 1024 : 16];
  u32x4 acc = {0, 0, 0, 0};
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  for (size_t sp = blockIdx.x; sp < n_spans; sp += gridDim.x) {
    const u32x4* q = p + sp * span16;
    if (kLds) {
      // a wavefront walks its quarter of the span, 1 KiB per load instruction, U in flight
      const uint32_t per_wave = span16 / 4;                 // 16-byte units, a multiple of 64 U
      const __amdgpu_buffer_rsrc_t r =
          __builtin_amdgcn_make_buffer_rsrc((void*)(q + (size_t)wave * per_wave), 0, (int)(per_wave * 16), kBufferFlags);
      uint8_t* base = s_sink + wave * (U * 1024);
      for (uint32_t i = 0; i < per_wave; i += 64 * U) {
#pragma unroll
        for (int u = 0; u < U; ++u)
          __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (lds_ptr_t)(base + u * 1024), 16, lane * 16,
                                                   (int)((i + u * 64) * 16), 0, MODE == 3 ? kNonTemporal : 0);
        wait_vmcnt<U / 2>();                                // the older half has landed: keep the rest in flight
      }
    } else {
      for (uint32_t i = threadIdx.x; i < span16; i += 256 * U) {
        u32x4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u)
          v[u] = MODE == 2 ? __builtin_nontemporal_load(q + i + u * 256) : q[i + u * 256];
#pragma unroll
        for (int u = 0; u < U; ++u) acc ^= v[u];
      }
    }
  }
  if (kLds) {
    wait_vmcnt<0>();
    __syncthreads();
    // what the wavefront's last trip left in its U slots (keeps the loads observable)
#pragma unroll
    for (int u = 0; u < U; ++u)
      acc ^= *reinterpret_cast<const u32x4*>(s_sink + wave * (U * 1024) + u * 1024 + lane * 16);
  }
  // data-dependent store: an all-zero source is read without any write traffic
  if ((acc.x | acc.y | acc.z | acc.w) != 0) out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = acc;
#endif
}

template <int U>
static bool launch_pattern(int mode, const u32x4* p, size_t n_spans, uint32_t span16, u32x4* out,
                           int n_workgroups, hipStream_t st) {
  const dim3 grid(n_workgroups), block(256);
  if (mode == 0) hipLaunchKernelGGL((stream_pattern_kernel<U, 0>), grid, block, 0, st, p, n_spans, span16, out);
  else if (mode == 1) hipLaunchKernelGGL((stream_pattern_kernel<U, 1>), grid, block, 0, st, p, n_spans, span16, out);
  else if (mode == 2) hipLaunchKernelGGL((stream_pattern_kernel<U, 2>), grid, block, 0, st, p, n_spans, span16, out);
  else if (mode == 3) hipLaunchKernelGGL((stream_pattern_kernel<U, 3>), grid, block, 0, st, p, n_spans, span16, out);
  else return false;
  return true;
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

prism_status prism_ceiling_hbm_read_pattern(const void* src, size_t bytes, void* out, int32_t n_workgroups,
                                            int32_t loads_in_flight, size_t span_bytes, int32_t mode,
                                            size_t* bytes_read, void* stream) {
  PRISM_ENTER();
  PRISM_RETURN_IF(src == nullptr || out == nullptr || bytes_read == nullptr, PRISM_ERR_INVALID_ARG);
  PRISM_RETURN_IF(((uintptr_t)src & 15u) != 0 || ((uintptr_t)out & 15u) != 0, PRISM_ERR_INVALID_ARG);
  PRISM_RETURN_IF(n_workgroups < 1 || mode < 0 || mode > 3, PRISM_ERR_INVALID_ARG);
  const int U = loads_in_flight;
  PRISM_RETURN_IF(U != 2 && U != 4 && U != 8 && U != 16, PRISM_ERR_UNSUPPORTED);
  // a span is walked in trips of 256 threads x U loads x 16 bytes; it must hold whole trips
  const size_t trip = (size_t)4096 * U;
  PRISM_RETURN_IF(span_bytes < trip || span_bytes % trip != 0 || span_bytes > ((size_t)1 << 31), PRISM_ERR_UNSUPPORTED);
  const size_t n_spans = bytes / span_bytes;
  PRISM_RETURN_IF(n_spans < 1, PRISM_ERR_INVALID_ARG);
  *bytes_read = n_spans * span_bytes;
  const u32x4* p = (const u32x4*)src;
  const uint32_t span16 = (uint32_t)(span_bytes / 16);
  const hipStream_t st = (hipStream_t)stream;
  bool ok = false;
  if (U == 2) ok = launch_pattern<2>(mode, p, n_spans, span16, (u32x4*)out, n_workgroups, st);
  else if (U == 4) ok = launch_pattern<4>(mode, p, n_spans, span16, (u32x4*)out, n_workgroups, st);
  else if (U == 8) ok = launch_pattern<8>(mode, p, n_spans, span16, (u32x4*)out, n_workgroups, st);
  else ok = launch_pattern<16>(mode, p, n_spans, span16, (u32x4*)out, n_workgroups, st);
  PRISM_RETURN_IF(!ok, PRISM_ERR_INVALID_ARG);
  PRISM_CHECK_LAUNCH();
  return PRISM_OK;
}

#pragma GCC visibility pop
}  // extern "C"
