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
// A batch of at most one chunk (decode) runs all three steps in one workgroup.
// The per-expert totals are the activation counts f_n^l(e) of Sec. III-B, so the
// scan step can also publish them (the fused layer takes them from here instead
// of a second histogram in the router).
#include "dispatch_device.h"

namespace prism {
namespace {

using namespace dispatch_dev;

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
    const SplitOut o) {
  __shared__ int s_total[PRISM_MAX_EXPERTS];
  __shared__ int s_start[PRISM_MAX_EXPERTS];
  __shared__ uint8_t s_mask[PRISM_MAX_EXPERTS];
  const int e = threadIdx.x;
  if (e < E) {
    int run = 0;
    for (int b = 0; b < n_chunks; ++b) {
      const int c = block_hist[(size_t)b * E + e];
      block_hist[(size_t)b * E + e] = run;
      run += c;
    }
    s_total[e] = run;
    s_mask[e] = mask[e];
  }
  __syncthreads();
  if (threadIdx.x < kWave) split_offsets(s_total, s_mask, E, o, s_start);
}

template <bool FUSED>
__global__ __launch_bounds__(kThreads) void dispatch_scatter_kernel(
    const int32_t* __restrict__ idx, int A, int E, const uint8_t* __restrict__ mask,
    const int32_t* __restrict__ block_base, const SplitOut o, int32_t* __restrict__ local_src,
    int32_t* __restrict__ remote_src, int32_t* __restrict__ inv) {
  dispatch_scatter_block<FUSED>(idx, A, E, mask, block_base, blockIdx.x, o, local_src, remote_src, inv);
}

}  // namespace

prism_status launch_dispatch(const prism_layer_desc& d, const int32_t* topk_idx,
                             const uint8_t* mask, int T, int32_t* local_src,
                             int32_t* local_offsets, int32_t* remote_src, int32_t* remote_offsets,
                             int32_t* n_local_remote, int64_t* remote_bytes, int32_t* inv,
                             int32_t* block_hist, int32_t* counts, int64_t* counts_accum,
                             hipStream_t st) {
  const int A = T * d.top_k;
  const int E = d.n_experts;
  const int n_chunks = A > 0 ? ceil_div(A, kDispatchChunk) : 0;
  const SplitOut o{local_offsets, remote_offsets, n_local_remote, remote_bytes, counts,
                   (unsigned long long*)counts_accum, d.hidden * elem_size(d.dtype)};
  if (n_chunks == 1) {
    hipLaunchKernelGGL(dispatch_scatter_kernel<true>, dim3(1), dim3(kThreads), 0, st, topk_idx, A, E,
                       mask, (const int32_t*)nullptr, o, local_src, remote_src, inv);
    PRISM_CHECK_LAUNCH();
    return PRISM_OK;
  }
  if (n_chunks > 0) {
    hipLaunchKernelGGL(dispatch_hist_kernel, dim3(n_chunks), dim3(kThreads), 0, st, topk_idx, A, E,
                       block_hist);
    PRISM_CHECK_LAUNCH();
  }
  hipLaunchKernelGGL(dispatch_scan_kernel, dim3(1), dim3(PRISM_MAX_EXPERTS), 0, st, block_hist,
                     n_chunks, E, mask, o);
  PRISM_CHECK_LAUNCH();
  if (n_chunks > 0) {
    hipLaunchKernelGGL(dispatch_scatter_kernel<false>, dim3(n_chunks), dim3(kThreads), 0, st,
                       topk_idx, A, E, mask, block_hist, o, local_src, remote_src, inv);
    PRISM_CHECK_LAUNCH();
  }
  return PRISM_OK;
}

}  // namespace prism
