// Device-side pieces of the placement split (paper Sec. III-B) that more than one
// kernel uses: the per-expert offset scan and the stable scatter of one chunk.
#ifndef PRISM_DISPATCH_DEVICE_H_
#define PRISM_DISPATCH_DEVICE_H_

#include "prism_internal.h"

namespace prism {
namespace dispatch_dev {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kPerWave = kDispatchChunk / kWaves;   // contiguous assignments per wavefront
constexpr int kSteps = kPerWave / kWave;

struct SplitOut {
  int32_t* local_offsets;    // [E+1]
  int32_t* remote_offsets;   // [E+1]
  int32_t* n_local_remote;   // [2]
  int64_t* remote_bytes;     // [2]
  int32_t* counts;           // [E] or NULL
  unsigned long long* counts_accum;   // [E] or NULL
  int row_bytes;
};

// Run by one whole wavefront: exclusive scans of the local and of the remote
// bucket sizes over the experts (4 per lane), all outputs of the split, and for
// every expert the start of its bucket in its own list (s_start).
__device__ __forceinline__ void split_offsets(const int* s_total, const uint8_t* s_mask, int E,
                                              const SplitOut& o, int* s_start) {
  const int lane = threadIdx.x & 63;
  int tot[4], loc = 0, rem = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int e = 4 * lane + j;
    tot[j] = e < E ? s_total[e] : 0;
    if (e < E && s_mask[e]) loc += tot[j]; else rem += tot[j];
  }
  int loc_incl = loc, rem_incl = rem;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int a = __shfl_up(loc_incl, off), b = __shfl_up(rem_incl, off);
    if (lane >= off) { loc_incl += a; rem_incl += b; }
  }
  int nl = loc_incl - loc, nr = rem_incl - rem;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int e = 4 * lane + j;
    if (e < E) {
      const bool local = s_mask[e] != 0;
      o.local_offsets[e] = nl;
      o.remote_offsets[e] = nr;
      s_start[e] = local ? nl : nr;
      if (o.counts != nullptr) o.counts[e] = tot[j];
      if (o.counts_accum != nullptr && tot[j] != 0)
        atomicAdd(&o.counts_accum[e], (unsigned long long)tot[j]);
      if (local) nl += tot[j]; else nr += tot[j];
    }
  }
  if (lane == 63) {   // nl, nr are now the grand totals
    o.local_offsets[E] = nl;
    o.remote_offsets[E] = nr;
    o.n_local_remote[0] = nl;
    o.n_local_remote[1] = nr;
    const int64_t bytes = (int64_t)nr * o.row_bytes;
    o.remote_bytes[0] = bytes;   // activations shipped to the hosting servers
    o.remote_bytes[1] = bytes;   // expert outputs shipped back
  }
}

// FUSED: the whole batch is this one chunk; the workgroup also does the scan step
// (block_base is not read, the offset arrays and totals in o are written here).
// Called by all kThreads threads of a workgroup for chunk `chunk` of the assignments.
// idx may have been written earlier in the same kernel by this workgroup (with a
// __syncthreads() in between), hence no __restrict__ on it.
template <bool FUSED>
__device__ __forceinline__ void dispatch_scatter_block(
    const int32_t* idx, int A, int E, const uint8_t* __restrict__ mask,
    const int32_t* __restrict__ block_base, int chunk, const SplitOut& o,
    int32_t* __restrict__ local_src, int32_t* __restrict__ remote_src, int32_t* __restrict__ inv) {
  // Only LDS data crosses between threads in here, so the barriers do not wait for
  // the global stores.
  __shared__ int s_whist[kWaves][PRISM_MAX_EXPERTS];
  __shared__ int s_total[FUSED ? PRISM_MAX_EXPERTS : 1];
  __shared__ int s_start[FUSED ? PRISM_MAX_EXPERTS : 1];
  __shared__ int s_pos[kWaves][PRISM_MAX_EXPERTS];
  __shared__ uint8_t s_mask[PRISM_MAX_EXPERTS];
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  for (int i = threadIdx.x; i < kWaves * PRISM_MAX_EXPERTS; i += kThreads) (&s_whist[0][0])[i] = 0;
  for (int e = threadIdx.x; e < E; e += kThreads) s_mask[e] = mask[e];
  lds_barrier();

  const int wave0 = chunk * kDispatchChunk + wave * kPerWave;
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
  lds_barrier();
  if (FUSED) {
    for (int e = threadIdx.x; e < E; e += kThreads) {
      int c = 0;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) c += s_whist[w][e];
      s_total[e] = c;
    }
    lds_barrier();
    if (threadIdx.x < kWave) split_offsets(s_total, s_mask, E, o, s_start);
    lds_barrier();
  }
  for (int e = threadIdx.x; e < E; e += kThreads) {
    int run;
    if (FUSED)
      run = s_start[e];
    else
      run = block_base[(size_t)chunk * E + e] +
            (s_mask[e] ? o.local_offsets[e] : o.remote_offsets[e]);
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      s_pos[w][e] = run;
      run += s_whist[w][e];
    }
  }
  lds_barrier();

#pragma unroll
  for (int s = 0; s < kSteps; ++s) {
    if (wave0 + s * kWave >= A) break;   // nothing left for this wavefront
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
    // s_pos[wave] belongs to this wavefront alone, whose LDS accesses execute in program
    // order: no barrier is needed between the read above and this update, nor before the
    // next step's read.
    if (valid && (same >> lane) == 1ull)   // highest lane of its group advances the cursor
      s_pos[wave][e] += __popcll(same);
  }
}

}  // namespace dispatch_dev
}  // namespace prism
#endif  // PRISM_DISPATCH_DEVICE_H_
