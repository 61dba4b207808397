// Device-side pieces of the placement split (paper Sec. III-B) that more than one
// kernel uses: the per-expert offset scan and the stable placement of a block of assignments.
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

// Assignments one workgroup places: `sub` consecutive chunks of kDispatchChunk, the fewest
// that keep the number of workgroups at or below kMaxBlocks (every workgroup sums the
// histograms of the workgroups before it).
constexpr int kMaxBlocks = 256;
static inline int sub_chunks(int A) {
  const int chunks = (A + kDispatchChunk - 1) / kDispatchChunk;
  return chunks > kMaxBlocks ? (chunks + kMaxBlocks - 1) / kMaxBlocks : 1;
}

// Run by one whole wavefront: exclusive scans of the local and of the remote
// bucket sizes over the experts (4 per lane); for every expert the start of its bucket
// in its own list (s_start); if s_local_off is given, the local offsets [E + 1] there;
// if write, all outputs of the split in o.
__device__ __forceinline__ void split_offsets(const int* s_total, const uint8_t* s_mask, int E,
                                              const SplitOut& o, int* s_start, bool write = true,
                                              int* s_local_off = nullptr) {
  const int lane = threadIdx.x & 63;
  int tot[4], loc = 0, rem = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int e = 4 * lane + j;
    tot[j] = e < E ? s_total[e] : 0;
    if (e < E && s_mask[e]) loc += tot[j]; else rem += tot[j];
  }
  const int loc_incl = wave_inclusive_scan(loc), rem_incl = wave_inclusive_scan(rem);
  int nl = loc_incl - loc, nr = rem_incl - rem;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int e = 4 * lane + j;
    if (e < E) {
      const bool local = s_mask[e] != 0;
      s_start[e] = local ? nl : nr;
      if (s_local_off != nullptr) s_local_off[e] = nl;
      if (write) {
        o.local_offsets[e] = nl;
        o.remote_offsets[e] = nr;
        if (o.counts != nullptr) o.counts[e] = tot[j];
        if (o.counts_accum != nullptr && tot[j] != 0)
          atomicAdd(&o.counts_accum[e], (unsigned long long)tot[j]);
      }
      if (local) nl += tot[j]; else nr += tot[j];
    }
  }
  if (lane == 63) {   // nl, nr are now the grand totals
    if (s_local_off != nullptr) s_local_off[E] = nl;
    if (write) {
      o.local_offsets[E] = nl;
      o.remote_offsets[E] = nr;
      o.n_local_remote[0] = nl;
      o.n_local_remote[1] = nr;
      const int64_t bytes = (int64_t)nr * o.row_bytes;
      o.remote_bytes[0] = bytes;   // activations shipped to the hosting servers
      o.remote_bytes[1] = bytes;   // expert outputs shipped back
    }
  }
}

// Per-expert totals of the whole batch and of the blocks before `block`, from the block
// histograms [n_blocks][E]: thread e < E returns its expert's pair.  (The loads do not depend
// on each other, so the loop runs at memory throughput, not latency.)
struct HistSums {
  int total, before;
};
__device__ __forceinline__ HistSums sum_block_hists(const int32_t* __restrict__ block_hist,
                                                    int n_blocks, int E, int block) {
  HistSums r{0, 0};
  const int e = threadIdx.x;
  if (e < E) {
    for (int b = 0; b < n_blocks; ++b) {
      const int c = block_hist[(size_t)b * E + e];
      r.total += c;
      if (b < block) r.before += c;
    }
  }
  return r;
}

// Places the assignments of block `block` (sub consecutive chunks of kDispatchChunk),
// called by all kThreads threads of a workgroup.
// FROM_HIST: block_hist [n_blocks][E] holds every block's histogram; the workgroup derives
// the bucket starts from it and, if it is block 0, writes the outputs in o.
// Otherwise the whole batch is one chunk: the workgroup histograms it itself (block_hist
// is not read) and writes the outputs.
// idx may have been written earlier in the same kernel by this workgroup (to memory with a
// __syncthreads() in between, or to LDS with a barrier), hence no __restrict__ on it.
// s_local_off (LDS, [E + 1], only without FROM_HIST): also receives the local offsets.
// my_mask >= 0: thread e < E already holds mask[e] (read before the steps that precede the call,
// so that its latency is not paid here).
template <bool FROM_HIST>
__device__ __forceinline__ void dispatch_place_block(
    const int32_t* idx, int A, int E, const uint8_t* __restrict__ mask,
    const int32_t* __restrict__ block_hist, int n_blocks, int sub, int block, const SplitOut& o,
    int32_t* __restrict__ local_src, int32_t* __restrict__ remote_src, int32_t* __restrict__ inv,
    int* s_local_off = nullptr, int my_mask = -1) {
  static_assert(PRISM_MAX_EXPERTS <= kThreads, "one thread per expert");
  // Only LDS data crosses between threads in here, so the barriers do not wait for
  // the global stores.
  __shared__ int s_whist[kWaves][PRISM_MAX_EXPERTS];
  __shared__ int s_total[PRISM_MAX_EXPERTS];
  __shared__ int s_run[PRISM_MAX_EXPERTS];      // next free position of every expert's bucket
  __shared__ int s_pos[kWaves][PRISM_MAX_EXPERTS];
  __shared__ uint8_t s_mask[PRISM_MAX_EXPERTS];
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  if (my_mask >= 0) {
    if (threadIdx.x < E) s_mask[threadIdx.x] = (uint8_t)my_mask;
  } else {
    for (int e = threadIdx.x; e < E; e += kThreads) s_mask[e] = mask[e];
  }
  if (FROM_HIST) {
    const HistSums hs = sum_block_hists(block_hist, n_blocks, E, block);
    if (threadIdx.x < E) s_total[threadIdx.x] = hs.total;
    lds_barrier();
    if (threadIdx.x < kWave) split_offsets(s_total, s_mask, E, o, s_run, block == 0);
    lds_barrier();
    if (threadIdx.x < E) s_run[threadIdx.x] += hs.before;   // thread e alone touches s_run[e] from here on
  }
  // bits that tell the expert ids apart
  const int id_bits = 32 - __clz(max(E - 1, 1));

  for (int c = 0; c < sub; ++c) {
    for (int i = threadIdx.x; i < kWaves * PRISM_MAX_EXPERTS; i += kThreads) (&s_whist[0][0])[i] = 0;
    lds_barrier();
    const int wave0 = (block * sub + c) * kDispatchChunk + wave * kPerWave;
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
    if (!FROM_HIST) {
      for (int e = threadIdx.x; e < E; e += kThreads) {
        int t = 0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) t += s_whist[w][e];
        s_total[e] = t;
      }
      lds_barrier();
      if (threadIdx.x < kWave) split_offsets(s_total, s_mask, E, o, s_run, true, s_local_off);
      lds_barrier();
    }
    if (threadIdx.x < E) {
      const int e = threadIdx.x;
      int run = s_run[e];
#pragma unroll
      for (int w = 0; w < kWaves; ++w) {
        s_pos[w][e] = run;
        run += s_whist[w][e];
      }
      s_run[e] = run;
    }
    lds_barrier();

#pragma unroll
    for (int s = 0; s < kSteps; ++s) {
      if (wave0 + s * kWave >= A) break;   // nothing left for this wavefront
      const int a = wave0 + s * kWave + lane;
      const int e = my_e[s];
      const bool valid = e >= 0;
      // lanes holding the same expert as this lane: one ballot per id bit
      unsigned long long same = __ballot(valid);
      for (int b = 0; b < id_bits; ++b) {
        const bool bit = (e >> b) & 1;
        const unsigned long long set = __ballot(valid && bit);
        same &= bit ? set : ~set;
      }
      if (valid) {
        const unsigned long long below = same & ((1ull << lane) - 1ull);
        const int pos = s_pos[wave][e] + __popcll(below);
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
    // the next chunk's clearing of s_whist needs no barrier here: s_whist is not read after
    // the barrier above, and its next use follows the barrier after the clearing
  }
}

}  // namespace dispatch_dev
}  // namespace prism
#endif  // PRISM_DISPATCH_DEVICE_H_
