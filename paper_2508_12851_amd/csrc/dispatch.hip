// Placement split and stable bucketing (paper Sec. III-B: an expert is remote
// for server n iff no GPU of n hosts it, i.e. local_mask[e] == 0).
//
// A stable counting sort of the T*k assignments by expert, in two launches:
//   hist     each workgroup histograms its block of assignments in LDS;
//   place    each workgroup sums the histograms (all of them: the per-expert totals,
//            from which it derives the local / remote offset arrays itself; those of the
//            blocks before it: its start inside every expert's bucket), re-reads its
//            block in order and places every assignment: position = bucket start + block
//            start + wavefront start + rank among the equal-expert lanes below it
//            (ballots).  Block 0 also writes the offset arrays, totals and byte counts.
// Bucket order is ascending assignment id by construction, so the result is a
// pure function of the input (no atomics decide an order).
// A batch of at most one chunk runs both steps in one workgroup.
// The per-expert totals are the activation counts f_n^l(e) of Sec. III-B, so block 0 can
// also publish them (the fused layer takes them from here instead of a second histogram
// in the router).
// The work schedules of the two grouped GEMMs of the expert FFN depend on the local
// offsets only, which any workgroup can derive from the histograms; the place launch
// therefore carries a few more workgroups that build them while the others place.
#include "dispatch_device.h"
#include "schedule.h"

namespace prism {
namespace {

using namespace dispatch_dev;

__global__ __launch_bounds__(kThreads) void dispatch_hist_kernel(const int32_t* __restrict__ idx,
                                                                 int A, int E, int sub,
                                                                 int32_t* __restrict__ block_hist) {
  __shared__ int s_hist[PRISM_MAX_EXPERTS];
  for (int e = threadIdx.x; e < E; e += kThreads) s_hist[e] = 0;
  __syncthreads();
  const long long a0 = (long long)blockIdx.x * sub * kDispatchChunk;
  for (int i = threadIdx.x; i < sub * kDispatchChunk; i += kThreads) {
    const long long a = a0 + i;
    if (a < A) {
      const int e = idx[a];
      if ((unsigned)e < (unsigned)E) atomicAdd(&s_hist[e], 1);
    }
  }
  __syncthreads();
  for (int e = threadIdx.x; e < E; e += kThreads) block_hist[(size_t)blockIdx.x * E + e] = s_hist[e];
}

constexpr int kSchedParts = 4;   // workgroups that share the building of one schedule

// Workgroups [0, n_blocks) place their block; if n_sched > 0, workgroups n_blocks + 4 s + part
// build part `part` of schedule s (0: gate/up GEMM, 1: down GEMM) from the same histograms.
template <bool FROM_HIST>
__global__ __launch_bounds__(kThreads) void dispatch_place_kernel(
    const int32_t* __restrict__ idx, int A, int E, const uint8_t* __restrict__ mask,
    const int32_t* __restrict__ block_hist, int n_blocks, int sub, const SplitOut o,
    int32_t* __restrict__ local_src, int32_t* __restrict__ remote_src, int32_t* __restrict__ inv,
    int S, int T, const gg::SchedParams p0, const gg::SchedParams p1) {
  if ((int)blockIdx.x < n_blocks) {
    dispatch_place_block<FROM_HIST>(idx, A, E, mask, block_hist, n_blocks, sub, blockIdx.x, o,
                                    local_src, remote_src, inv);
    return;
  }
  if (FROM_HIST) {
    __shared__ int s_total[PRISM_MAX_EXPERTS];
    __shared__ int s_start[PRISM_MAX_EXPERTS];
    __shared__ int s_local_off[PRISM_MAX_EXPERTS + 1];
    __shared__ uint8_t s_mask[PRISM_MAX_EXPERTS];
    const int j = blockIdx.x - n_blocks;
    for (int e = threadIdx.x; e < E; e += kThreads) s_mask[e] = mask[e];
    const HistSums hs = sum_block_hists(block_hist, n_blocks, E, 0);
    if (threadIdx.x < E) s_total[threadIdx.x] = hs.total;
    lds_barrier();
    if (threadIdx.x < kWave) split_offsets(s_total, s_mask, E, o, s_start, false, s_local_off);
    lds_barrier();
    const gg::SchedParams p[1] = {j / kSchedParts == 0 ? p0 : p1};
    gg::build_schedules_block<1>(s_local_off, E, S, T, A, p, j % kSchedParts, kSchedParts);
  }
}

}  // namespace

prism_status launch_dispatch(const prism_layer_desc& d, const int32_t* topk_idx,
                             const uint8_t* mask, int T, int32_t* local_src,
                             int32_t* local_offsets, int32_t* remote_src, int32_t* remote_offsets,
                             int32_t* n_local_remote, int64_t* remote_bytes, int32_t* inv,
                             int32_t* block_hist, int32_t* counts, int64_t* counts_accum,
                             hipStream_t st, int32_t* tiles, bool* schedules_built) {
  const int A = T * d.top_k;
  const int E = d.n_experts;
  const SplitOut o{local_offsets, remote_offsets, n_local_remote, remote_bytes, counts,
                   (unsigned long long*)counts_accum, d.hidden * elem_size(d.dtype)};
  if (schedules_built != nullptr) *schedules_built = false;
  gg::SchedParams p0{}, p1{};
  if (A <= kDispatchChunk) {   // one workgroup histograms and places (T = 0: writes the empty split)
    hipLaunchKernelGGL(dispatch_place_kernel<false>, dim3(1), dim3(kThreads), 0, st, topk_idx, A, E,
                       mask, (const int32_t*)nullptr, 1, 1, o, local_src, remote_src, inv, 0, T, p0, p1);
    PRISM_CHECK_LAUNCH();
    return PRISM_OK;
  }
  const int sub = sub_chunks(A);
  const int n_blocks = ceil_div(A, sub * kDispatchChunk);
  int n_sched = 0;
  if (tiles != nullptr && d.dtype == PRISM_BF16) {
    gg::ffn_sched_params(d, T, tiles, &p0, &p1);
    n_sched = 2 * kSchedParts;
    if (schedules_built != nullptr) *schedules_built = true;
  }
  hipLaunchKernelGGL(dispatch_hist_kernel, dim3(n_blocks), dim3(kThreads), 0, st, topk_idx, A, E, sub,
                     block_hist);
  PRISM_CHECK_LAUNCH();
  hipLaunchKernelGGL(dispatch_place_kernel<true>, dim3(n_blocks + n_sched), dim3(kThreads), 0, st,
                     topk_idx, A, E, mask, block_hist, n_blocks, sub, o, local_src, remote_src, inv,
                     d.n_shared, T, p0, p1);
  PRISM_CHECK_LAUNCH();
  return PRISM_OK;
}

}  // namespace prism
