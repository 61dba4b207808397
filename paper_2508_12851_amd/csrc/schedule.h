// Work schedule of the grouped GEMMs: layout, the device-side builder and the
// host-side size bounds.
#ifndef PRISM_SCHEDULE_H_
#define PRISM_SCHEDULE_H_

#include "prism_internal.h"

namespace prism {
namespace gg {

constexpr int kMaxGroups = PRISM_MAX_EXPERTS + PRISM_MAX_SHARED;
constexpr int kXcds = 8;
constexpr int kSchedHeader = 16;     // ints
constexpr int kItemInts = 8;         // ints per work item

// Schedule memory (int32):
//   [0] n_mtiles  [1] capacity of one XCD list (items)  [4 + x] items in the list of XCD x
//   then, from int kSchedHeader on, 8 lists of `capacity` items of 8 ints:
//     [0] group id g (g < E: routed expert g; else shared expert g - E)
//     [1] first row of the row tile in h / y row space
//     [2] rows in the tile (1..BM)
//     [3] first token of the tile for shared experts, -1 for routed ones
//     [4] column tile
struct SchedParams {
  int BM;            // row tile
  int n_ntiles;      // column tiles
  int capacity;      // items one XCD list can hold
  int32_t* sched;
};

// Builds NS (1 or 2) schedules of the same row groups side by side; called by every
// thread of a workgroup (any size that is a multiple of 64).  Inside, only LDS data
// crosses between threads, so the barriers do not wait for the global stores.
// local_offsets may have been written earlier in the same kernel by this workgroup
// (with a __syncthreads() in between), hence no __restrict__ on it.
template <int NS>
__device__ __forceinline__ void build_schedules_block(const int32_t* local_offsets, int E, int S,
                                                      int T, int A_total,
                                                      const SchedParams (&p)[NS]) {
  __shared__ int s_rows[kMaxGroups], s_row0[kMaxGroups];
  __shared__ int s_start[NS][kMaxGroups + 1];            // first row tile of group g
  __shared__ int s_rank[NS][kMaxGroups];                 // index of g among the non-empty groups
  __shared__ int s_base[NS][kXcds][kMaxGroups + 1];      // items of XCD x before group g
  const int G = E + S;
  // p[s] for a thread-dependent s, without indexing the parameter array at run time
  // (that would put it in scratch memory)
  auto pick = [&](int s) { return NS == 1 || s == 0 ? p[0] : p[NS - 1]; };
  for (int g = threadIdx.x; g < G; g += blockDim.x) {
    int rows, row0;
    if (g < E) {
      row0 = local_offsets[g];
      rows = local_offsets[g + 1] - row0;
    } else {
      row0 = A_total + (g - E) * T;
      rows = T;
    }
    s_rows[g] = rows;
    s_row0[g] = row0;
  }
  lds_barrier();
  if (threadIdx.x < NS) {
    const int s = threadIdx.x;
    const SchedParams ps = pick(s);
    const int BM = ps.BM;
    int run = 0, rank = 0;
    for (int g = 0; g < G; ++g) {
      s_start[s][g] = run;
      s_rank[s][g] = rank;
      const int m = (s_rows[g] + BM - 1) / BM;
      run += m;
      rank += m > 0;
    }
    s_start[s][G] = run;
    ps.sched[0] = run;
    ps.sched[1] = ps.capacity;
  }
  lds_barrier();
  // Pair (g, nt) has index q = rank(g) * n_ntiles + nt and belongs to XCD q % 8.
  // XCD x owns the column tiles r, r + 8, ... of group g with r = (x - rank(g) n_ntiles) mod 8.
  auto first_nt = [&](int s, int n_ntiles, int g, int x) {
    const int r = (x - s_rank[s][g] * n_ntiles) % kXcds;
    return r < 0 ? r + kXcds : r;
  };
  if (threadIdx.x < NS * kXcds) {
    const int s = threadIdx.x / kXcds, x = threadIdx.x % kXcds;
    const SchedParams ps = pick(s);
    const int n_ntiles = ps.n_ntiles;
    int run = 0;
    for (int g = 0; g < G; ++g) {
      s_base[s][x][g] = run;
      const int m = s_start[s][g + 1] - s_start[s][g];
      const int r = first_nt(s, n_ntiles, g, x);
      const int c = r < n_ntiles ? (n_ntiles - 1 - r) / kXcds + 1 : 0;
      run += m * c;
    }
    s_base[s][x][G] = run;
    ps.sched[4 + x] = run;
  }
  lds_barrier();
#pragma unroll
  for (int s = 0; s < NS; ++s) {
    const int BM = p[s].BM, n_ntiles = p[s].n_ntiles, capacity = p[s].capacity;
    const int n_mtiles = s_start[s][G];
    auto group_of_tile = [&](int i) {   // largest g with s_start[g] <= i (skips empty groups)
      int lo = 0, hi = G;               // invariant: s_start[lo] <= i < s_start[hi]
      while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (s_start[s][mid] <= i) lo = mid; else hi = mid;
      }
      return lo;
    };
    const long long n_items = (long long)n_mtiles * n_ntiles;
    for (long long w = threadIdx.x; w < n_items; w += blockDim.x) {
      const int i = (int)(w % n_mtiles), nt = (int)(w / n_mtiles);
      const int g = group_of_tile(i);
      const int mi = i - s_start[s][g];
      const int m = s_start[s][g + 1] - s_start[s][g];
      const int x = (s_rank[s][g] * n_ntiles + nt) % kXcds;
      const int pos = s_base[s][x][g] + ((nt - first_nt(s, n_ntiles, g, x)) / kXcds) * m + mi;   // row tiles fastest
      int4* out = reinterpret_cast<int4*>(p[s].sched + kSchedHeader +
                                          ((size_t)x * capacity + pos) * kItemInts);
      out[0] = int4{g, s_row0[g] + mi * BM, min(BM, s_rows[g] - mi * BM), g < E ? -1 : mi * BM};
      out[1] = int4{nt, 0, 0, 0};
    }
  }
}

// Upper bound on the number of row tiles for T tokens (host side).
static inline int max_row_tiles(const prism_layer_desc& d, int T, int BM) {
  return T * d.top_k / BM + d.n_experts + d.n_shared * ceil_div(T, BM);
}

// Items one XCD list must be able to hold: every row tile times its share of the column tiles.
static inline int sched_capacity(const prism_layer_desc& d, int T, int BM, int n_ntiles) {
  return max_row_tiles(d, T, BM) * ceil_div(n_ntiles, kXcds);
}

}  // namespace gg
}  // namespace prism
#endif  // PRISM_SCHEDULE_H_
