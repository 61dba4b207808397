// Placement split and stable bucketing (paper Sec. III-B: an expert is remote
// for server n iff no GPU of n hosts it, i.e. local_mask[e] == 0).
//
// A stable counting sort of the T*k assignments by expert, in three launches:
//   hist     each workgroup histograms its chunk of assignments in LDS;
//   scan     one workgroup turns the per-chunk histograms into per-chunk start
//            positions inside every expert's bucket, and the per-expert totals
//            into the local / remote offset arrays, totals and byte counts;
//   scatter  each workgroup re-reads its chunk in order and places every
//            assignment: position = bucket start + chunk start + wavefront
//            start + rank among the equal-expert lanes below it (ballot).
// Bucket order is ascending assignment id by construction, so the result is a
// pure function of the input (no atomics decide an order).
#include "prism_internal.h"

namespace prism {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kPerWave = kDispatchChunk / kWaves;   // contiguous assignments per wavefront
constexpr int kSteps = kPerWave / kWave;

__global__ __launch_bounds__(kThreads) void dispatch_hist_kernel(const int32_t* __restrict__ idx,
                                                                 int A, int E,
                                                                 int32_t* __restrict__ block_hist) {
  __shared__ int s_hist[PRISM_MAX_EXPERTS];
  for (int e = threadIdx.x; e < E; e += kThreads) s_hist[e] = 0;
  __syncthreads();
  const int a0 = blockIdx.x * kDispatchChunk;
  for (int i = threadIdx.x; i < kDispatchChunk; i += kThreads) {
    const int a = a0 + i;
    if (a < A) {
      const int e = idx[a];
      if ((unsigned)e < (unsigned)E) atomicAdd(&s_hist[e], 1);
    }
  }
  __syncthreads();
  for (int e = threadIdx.x; e < E; e += kThreads) block_hist[(size_t)blockIdx.x * E + e] = s_hist[e];
}

__global__ __launch_bounds__(PRISM_MAX_EXPERTS) void dispatch_scan_kernel(
    int32_t* __restrict__ block_hist, int n_chunks, int E, const uint8_t* __restrict__ mask,
    int row_bytes, int32_t* __restrict__ local_offsets, int32_t* __restrict__ remote_offsets,
    int32_t* __restrict__ n_local_remote, int64_t* __restrict__ remote_bytes) {
  __shared__ int s_total[PRISM_MAX_EXPERTS];
  const int e = threadIdx.x;
  if (e < E) {
    int run = 0;
    for (int b = 0; b < n_chunks; ++b) {
      const int c = block_hist[(size_t)b * E + e];
      block_hist[(size_t)b * E + e] = run;
      run += c;
    }
    s_total[e] = run;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int nl = 0, nr = 0;
    for (int i = 0; i < E; ++i) {
      local_offsets[i] = nl;
      remote_offsets[i] = nr;
      if (mask[i]) nl += s_total[i]; else nr += s_total[i];
    }
    local_offsets[E] = nl;
    remote_offsets[E] = nr;
    n_local_remote[0] = nl;
    n_local_remote[1] = nr;
    const int64_t bytes = (int64_t)nr * row_bytes;
    remote_bytes[0] = bytes;   // activations shipped to the hosting servers
    remote_bytes[1] = bytes;   // expert outputs shipped back
  }
}

__global__ __launch_bounds__(kThreads) void dispatch_scatter_kernel(
    const int32_t* __restrict__ idx, int A, int E, const uint8_t* __restrict__ mask,
    const int32_t* __restrict__ block_base, const int32_t* __restrict__ local_offsets,
    const int32_t* __restrict__ remote_offsets, int32_t* __restrict__ local_src,
    int32_t* __restrict__ remote_src, int32_t* __restrict__ inv) {
  __shared__ int s_whist[kWaves][PRISM_MAX_EXPERTS];
  __shared__ int s_pos[kWaves][PRISM_MAX_EXPERTS];
  __shared__ uint8_t s_mask[PRISM_MAX_EXPERTS];
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  for (int i = threadIdx.x; i < kWaves * PRISM_MAX_EXPERTS; i += kThreads) (&s_whist[0][0])[i] = 0;
  for (int e = threadIdx.x; e < E; e += kThreads) s_mask[e] = mask[e];
  __syncthreads();

  const int wave0 = blockIdx.x * kDispatchChunk + wave * kPerWave;
  int my_e[kSteps];
#pragma unroll
  for (int s = 0; s < kSteps; ++s) {
    const int a = wave0 + s * kWave + lane;
    int e = -1;
    if (a < A) {
      e = idx[a];
      if ((unsigned)e >= (unsigned)E) e = -1;
    }
    my_e[s] = e;
    if (e >= 0) atomicAdd(&s_whist[wave][e], 1);
  }
  __syncthreads();
  for (int e = threadIdx.x; e < E; e += kThreads) {
    int run = block_base[(size_t)blockIdx.x * E + e] + (s_mask[e] ? local_offsets[e] : remote_offsets[e]);
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      s_pos[w][e] = run;
      run += s_whist[w][e];
    }
  }
  __syncthreads();

#pragma unroll
  for (int s = 0; s < kSteps; ++s) {
    const int a = wave0 + s * kWave + lane;
    const int e = my_e[s];
    const bool valid = e >= 0;
    // lanes holding the same expert as this lane
    unsigned long long todo = __ballot(valid);
    unsigned long long same = 0;
    while (todo) {
      const int leader = __ffsll((long long)todo) - 1;
      const int ev = __shfl(e, leader);
      const unsigned long long m = __ballot(valid && e == ev);
      if (valid && e == ev) same = m;
      todo &= ~m;
    }
    int pos = 0;
    if (valid) {
      const unsigned long long below = same & ((1ull << lane) - 1ull);
      pos = s_pos[wave][e] + __popcll(below);
      const bool local = s_mask[e] != 0;
      (local ? local_src : remote_src)[pos] = a;
      if (inv != nullptr) inv[a] = local ? pos : -1;
    }
    __syncthreads();
    if (valid && (same >> lane) == 1ull)   // highest lane of its group advances the cursor
      s_pos[wave][e] += __popcll(same);
    __syncthreads();
  }
}

}  // namespace

prism_status launch_dispatch(const prism_layer_desc& d, const int32_t* topk_idx,
                             const uint8_t* mask, int T, int32_t* local_src,
                             int32_t* local_offsets, int32_t* remote_src, int32_t* remote_offsets,
                             int32_t* n_local_remote, int64_t* remote_bytes, int32_t* inv,
                             int32_t* block_hist, hipStream_t st) {
  const int A = T * d.top_k;
  const int E = d.n_experts;
  const int n_chunks = A > 0 ? ceil_div(A, kDispatchChunk) : 0;
  if (n_chunks > 0) {
    hipLaunchKernelGGL(dispatch_hist_kernel, dim3(n_chunks), dim3(kThreads), 0, st, topk_idx, A, E,
                       block_hist);
    PRISM_CHECK_LAUNCH();
  }
  hipLaunchKernelGGL(dispatch_scan_kernel, dim3(1), dim3(PRISM_MAX_EXPERTS), 0, st, block_hist,
                     n_chunks, E, mask, d.hidden * elem_size(d.dtype), local_offsets,
                     remote_offsets, n_local_remote, remote_bytes);
  PRISM_CHECK_LAUNCH();
  if (n_chunks > 0) {
    hipLaunchKernelGGL(dispatch_scatter_kernel, dim3(n_chunks), dim3(kThreads), 0, st, topk_idx, A,
                       E, mask, block_hist, local_offsets, remote_offsets, local_src, remote_src,
                       inv);
    PRISM_CHECK_LAUNCH();
  }
  return PRISM_OK;
}

}  // namespace prism
