// Gating network of one edge server (paper Sec. III-A) and the activation
// statistic f_n^l(e) (Sec. III-B): router GEMM, top-k, softmax gates, counts.
//
// Router logits must agree bit for bit with an independent implementation, so
// the dot products are accumulated in fp64 (every bf16*bf16 and fp32*fp32
// product is exact in fp64) on the fp64 matrix cores and rounded once to fp32.
//
// Work split: a workgroup takes 16 tokens; its 8 wavefronts split the hidden
// dimension (so even a 32-token decode batch has 16 wavefronts in flight) and
// their partial 16-token x E logit tiles, held as v_mfma_f64_16x16x4 blocks, are
// summed pairwise through LDS in a fixed order.  Operands are loaded straight
// from global memory with 16-byte (bf16) or 2x16-byte (fp32) loads per lane:
// lane (r = lane % 16, q = lane / 16) fetches elements h0 + 8q .. h0 + 8q + 7 of
// row r, and MFMA step j consumes element j of every lane, so both operands see
// the same permutation of the contraction index.
// The accumulator layout leaves each token's logits spread over one 16-lane
// group, so the k best experts are picked right there with xor-shuffle
// arg-max reductions over (logit, index) pairs, four tokens at a time.
//
// Decode batches (at most 64 tokens, bf16) have only 1..4 token tiles, which would
// leave the router on 1..4 compute units.  There the hidden dimension is also
// split over workgroups: route_kernel<PARTIAL> writes each workgroup's fp64 tile
// to memory, and a single-workgroup kernel sums those in a fixed order, finishes
// the routing and, being alone on the critical path anyway, goes on to do the
// placement split and to build the work schedules of the two grouped GEMMs.
#include "dispatch_device.h"
#include "prism_internal.h"
#include "schedule.h"

namespace prism {
namespace {

constexpr int kTokPerBlock = 16;
constexpr int kWavesPerBlock = 8;      // split the hidden dimension

__device__ __forceinline__ void load8(const float* p, float (&v)[8]) {
  const f32x4 a = *reinterpret_cast<const f32x4*>(p);
  const f32x4 b = *reinterpret_cast<const f32x4*>(p + 4);
  v[0] = a[0]; v[1] = a[1]; v[2] = a[2]; v[3] = a[3];
  v[4] = b[0]; v[5] = b[1]; v[6] = b[2]; v[7] = b[3];
}
__device__ __forceinline__ void load8(const uint16_t* p, float (&v)[8]) {
  const uint4 a = *reinterpret_cast<const uint4*>(p);
  v[0] = bf16_lo(a.x); v[1] = bf16_hi(a.x); v[2] = bf16_lo(a.y); v[3] = bf16_hi(a.y);
  v[4] = bf16_lo(a.z); v[5] = bf16_hi(a.z); v[6] = bf16_lo(a.w); v[7] = bf16_hi(a.w);
}

// Router-bias entries of token t for the experts 16 n + r this lane holds (0 where there is
// none: no bias, expert past E, token past T).
template <int NT>
__device__ __forceinline__ void load_bias_group(const float* __restrict__ bias, int t, int T, int E,
                                                int bias_group_tokens, float (&b)[NT]) {
  const int r = threadIdx.x & 15;
  const int row = bias_group_tokens > 0 ? t / bias_group_tokens : 0;
#pragma unroll
  for (int n = 0; n < NT; ++n) {
    const int e = n * 16 + r;
    b[n] = bias != nullptr && e < E && t < T ? bias[(size_t)row * E + e] : 0.f;
  }
}

// From the complete fp64 logits of U tokens per 16-lane group (lane r of the group holds
// experts 16 n + r of tokens t[0..U)) to those tokens' top-k indices and gates.  Run by a whole
// wavefront.  The routing of a token is one long dependent chain (arg-max rounds, an fp64
// exponential, a division); the U chains run side by side in one instruction stream.
// has_bias: add b (from load_bias_group) after the one rounding to fp32.
// s_counts (LDS, may be NULL) receives +1 per selected expert; s_idx (LDS, may be NULL) a copy
// of topk_idx for what follows in the same kernel.
template <int NT, int U>
__device__ __forceinline__ void finish_groups(const double (&s)[U][NT], const float (&b)[U][NT],
                                              bool has_bias, const int (&t)[U], int T, int E, int k,
                                              int gate_mode, float* __restrict__ logits,
                                              int32_t* topk_idx, float* __restrict__ topk_gate,
                                              int* s_counts, int32_t* s_idx) {
  const int r = threadIdx.x & 15;
  // ---- one rounding to fp32, then the fp32 bias add --------------------------
  float lg[U][NT];
#pragma unroll
  for (int u = 0; u < U; ++u)
#pragma unroll
    for (int n = 0; n < NT; ++n) {
      const int e = n * 16 + r;
      float val = (float)s[u][n];
      if (e < E && t[u] < T) {
        if (has_bias) val = val + b[u][n];
        if (logits != nullptr) logits[(size_t)t[u] * E + e] = val;
      } else if (e >= E) {
        val = -INFINITY;
      }
      lg[u][n] = val;
    }

  // ---- top-k: k rounds of arg-max over (logit, expert index) with xor-exchanges inside the
  // group; equal logits resolve to the lower expert index.
  float vals[U][NT];
  float sel0[U], mysel[U];
  int myidx[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
#pragma unroll
    for (int n = 0; n < NT; ++n) vals[u][n] = lg[u][n];
    sel0[u] = 0.f; mysel[u] = 0.f; myidx[u] = 0;
  }
  for (int j = 0; j < k; ++j) {
    float best[U];
    int bidx[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      best[u] = vals[u][0];
      bidx[u] = r;
#pragma unroll
      for (int n = 1; n < NT; ++n)
        if (vals[u][n] > best[u]) { best[u] = vals[u][n]; bidx[u] = n * 16 + r; }
    }
    auto meet = [&](int u, float ov, int oi) {
      if (ov > best[u] || (ov == best[u] && oi < bidx[u])) { best[u] = ov; bidx[u] = oi; }
    };
#pragma unroll
    for (int u = 0; u < U; ++u) meet(u, row_xor<8>(best[u]), row_xor<8>(bidx[u]));
#pragma unroll
    for (int u = 0; u < U; ++u) meet(u, row_xor<4>(best[u]), row_xor<4>(bidx[u]));
#pragma unroll
    for (int u = 0; u < U; ++u) meet(u, row_xor<2>(best[u]), row_xor<2>(bidx[u]));
#pragma unroll
    for (int u = 0; u < U; ++u) meet(u, row_xor<1>(best[u]), row_xor<1>(bidx[u]));
    // every lane of the group holds the winner; its owner retires it
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int n = 0; n < NT; ++n)
        if (bidx[u] == n * 16 + r) vals[u][n] = -INFINITY;
      if (j == 0) sel0[u] = best[u];
      if (r == j) { mysel[u] = best[u]; myidx[u] = bidx[u]; }
    }
  }
  // gates: softmax over the k picked logits, or the picked entries of the softmax over
  // all experts; lane r < k owns slot r, sel0 is the token's largest logit
  double w[U], sum[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    w[u] = r < k ? exp((double)mysel[u] - (double)sel0[u]) : 0.0;
    sum[u] = w[u];
  }
  if (gate_mode == PRISM_GATES_SOFTMAX_ALL) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      sum[u] = 0.0;
#pragma unroll
      for (int n = 0; n < NT; ++n) sum[u] += exp((double)lg[u][n] - (double)sel0[u]);   // exp(-inf) = 0 past E
    }
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    sum[u] += row_xor<8>(sum[u]);
    sum[u] += row_xor<4>(sum[u]);
    sum[u] += row_xor<2>(sum[u]);
    sum[u] += row_xor<1>(sum[u]);
  }
#pragma unroll
  for (int u = 0; u < U; ++u)
    if (r < k && t[u] < T) {
      topk_idx[(size_t)t[u] * k + r] = myidx[u];
      if (s_idx != nullptr) s_idx[t[u] * k + r] = myidx[u];
      topk_gate[(size_t)t[u] * k + r] = (float)(w[u] / sum[u]);
      if (s_counts != nullptr) atomicAdd(&s_counts[myidx[u]], 1);
    }
}

template <int NT>
__device__ __forceinline__ void finish_group(const double (&s)[NT], const float (&b)[NT],
                                             bool has_bias, int t, int T, int E, int k, int gate_mode,
                                             float* __restrict__ logits, int32_t* topk_idx,
                                             float* __restrict__ topk_gate, int* s_counts,
                                             int32_t* s_idx = nullptr) {
  double s1[1][NT];
  float b1[1][NT];
#pragma unroll
  for (int n = 0; n < NT; ++n) { s1[0][n] = s[n]; b1[0][n] = b[n]; }
  const int t1[1] = {t};
  finish_groups<NT, 1>(s1, b1, has_bias, t1, T, E, k, gate_mode, logits, topk_idx, topk_gate, s_counts,
                       s_idx);
}

// The same for a tile of 16 tokens held by one wavefront in the accumulator layout of
// v_mfma_f64_16x16x4: register v of lane (r, q) is token 4 v + q, expert 16 n + r.
// v_mask (wave-uniform): bit v set = handle the four tokens 4v + q of the tile, so
// several wavefronts can share one tile's work.
template <int NT>
__device__ __forceinline__ void finish_tile(const f64x4 (&acc)[NT], int tok0, int v_mask,
                                            const float* __restrict__ bias, int T, int E, int k,
                                            int bias_group_tokens, int gate_mode,
                                            float* __restrict__ logits, int32_t* topk_idx,
                                            float* __restrict__ topk_gate, int* s_counts,
                                            int32_t* s_idx = nullptr) {
  const int q = (threadIdx.x & 63) >> 4;
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    if (!((v_mask >> v) & 1)) continue;
    const int t = tok0 + 4 * v + q;
    double s[NT];
    float b[NT];
#pragma unroll
    for (int n = 0; n < NT; ++n) s[n] = acc[n][v];
    load_bias_group<NT>(bias, t, T, E, bias_group_tokens, b);
    finish_group<NT>(s, b, bias != nullptr, t, T, E, k, gate_mode, logits, topk_idx, topk_gate,
                     s_counts, s_idx);
  }
}

// NT = number of 16-expert column tiles (E <= 16 * NT).
// PARTIAL: workgroup (tile, y) covers hidden elements [y h_span, (y + 1) h_span) only and
// stores its fp64 tile to partial[tile][y][NT][64 lanes][4]; nothing else is written.
template <typename TIn, int NT, bool PARTIAL>
__global__ __launch_bounds__(kWavesPerBlock* kWave) void route_kernel(
    const TIn* __restrict__ x, const TIn* __restrict__ w_router, const float* __restrict__ bias,
    int T, int H, int E, int k, int bias_group_tokens, int gate_mode, float* __restrict__ logits,
    int32_t* __restrict__ topk_idx, float* __restrict__ topk_gate, int32_t* __restrict__ counts,
    unsigned long long* __restrict__ counts_accum, int h_span, double* __restrict__ partial) {
  constexpr int EP = NT * 16;             // padded expert count
  __shared__ int s_counts[EP];
  extern __shared__ __align__(16) double s_part[];   // [kWavesPerBlock / 2][NT * 4][64]

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int r = lane & 15;
  const int q = lane >> 4;
  const int tok0 = blockIdx.x * kTokPerBlock;

  for (int e = threadIdx.x; e < EP; e += blockDim.x) s_counts[e] = 0;
  __syncthreads();

  // ---- router GEMM on the fp64 matrix cores --------------------------------
  f64x4 acc[NT];
#pragma unroll
  for (int n = 0; n < NT; ++n) acc[n] = f64x4{0.0, 0.0, 0.0, 0.0};

  const int t_load = min(tok0 + r, T - 1);
  const TIn* xrow = x + (size_t)t_load * H;
  const TIn* wrow[NT];
#pragma unroll
  for (int n = 0; n < NT; ++n) wrow[n] = w_router + (size_t)min(n * 16 + r, E - 1) * H;

  // Wavefront w takes the 32-element slices w, w + 8, w + 16, ... of the hidden dimension,
  // U slices per trip so that their loads are all in flight before the first MFMA waits.
  // H % 8 == 0, so a lane's 8-element chunk is entirely inside or outside; lanes past the
  // end feed zeros (the MFMA itself is wave-wide).
  constexpr int U = PARTIAL ? 1 : NT <= 1 ? 8 : NT <= 2 ? 4 : NT <= 4 ? 2 : 1;
  constexpr int kSliceStride = 32 * kWavesPerBlock;
  const int h_begin = PARTIAL ? (int)blockIdx.y * h_span : 0;
  const int h_end = PARTIAL ? min(H, h_begin + h_span) : H;
  for (int h0 = h_begin + wave * 32; h0 < h_end; h0 += kSliceStride * U) {
    float xa[U][8];
    float wb[U][NT][8];
    bool inside[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int h = h0 + u * kSliceStride + q * 8;
      inside[u] = h < h_end;
      const int hl = inside[u] ? h : 0;
      load8(xrow + hl, xa[u]);
#pragma unroll
      for (int n = 0; n < NT; ++n) load8(wrow[n] + hl, wb[u][n]);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const double a = inside[u] ? (double)xa[u][j] : 0.0;
#pragma unroll
        for (int n = 0; n < NT; ++n)
          acc[n] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, (double)wb[u][n][j], acc[n], 0, 0, 0);
      }
    }
  }

  // ---- sum the partial tiles: (1,3,5,7) -> (0,2,4,6), (2,6) -> (0,4), 4 -> 0 ----
#pragma unroll
  for (int step = 1; step < kWavesPerBlock; step <<= 1) {
    const bool sender = (wave & (2 * step - 1)) == step;
    const bool receiver = (wave & (2 * step - 1)) == 0;
    double* slot = s_part + (size_t)(wave / (2 * step)) * (NT * 4 * 64);
    if (sender) {
#pragma unroll
      for (int n = 0; n < NT; ++n)
#pragma unroll
        for (int v = 0; v < 4; ++v) slot[(n * 4 + v) * 64 + lane] = acc[n][v];
    }
    __syncthreads();
    if (receiver) {
#pragma unroll
      for (int n = 0; n < NT; ++n)
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[n][v] += slot[(n * 4 + v) * 64 + lane];
    }
    __syncthreads();
  }
  if (wave != 0) return;   // wavefront 0 holds the full sums (no barrier follows)

  if (PARTIAL) {
    double* out = partial + ((size_t)blockIdx.x * gridDim.y + blockIdx.y) * (NT * 256);
#pragma unroll
    for (int n = 0; n < NT; ++n) *reinterpret_cast<f64x4*>(out + n * 256 + lane * 4) = acc[n];
    return;
  }

  finish_tile<NT>(acc, tok0, 0xF, bias, T, E, k, bias_group_tokens, gate_mode, logits, topk_idx,
                  topk_gate, counts != nullptr ? s_counts : nullptr);
  if (counts == nullptr) return;   // the caller derives the counts from the dispatch histogram
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");   // this wavefront's LDS atomics, then its reads

  // ---- per-expert activation counts -----------------------------------------
  for (int e = lane; e < E; e += 64) {
    const int c = s_counts[e];
    if (c != 0) {
      atomicAdd(&counts[e], c);
      if (counts_accum != nullptr) atomicAdd(&counts_accum[e], (unsigned long long)c);
    }
  }
}

// Router for bf16 batches of more than 64 tokens and at most 64 experts: operands staged
// through LDS.
//
// Loading operands from global memory straight in the MFMA layout (route_kernel) makes every
// quarter of a load instruction touch 16 rows, 16 bytes of each, and the vector cache then
// bounds the kernel (64 cache-line lookups per instruction; the fp64 matrix cores were busy
// 42 % of the time at 8192 tokens x 60 experts).  Here a wavefront brings its 32-element
// slice of 16 rows with one buffer_load_dwordx4 ... lds whose lanes cover each row's 64 bytes
// contiguously (lane l: row l / 4, 16 lookups per instruction), into LDS that is private to
// the wavefront, and reads it back in the MFMA layout (lane (r, q): row r, chunk q).  A
// 1 KiB block holds 16 rows x 4 chunks of 16 bytes; chunk c of row r sits in slot
// (c + r / 4) % 4 of the row, which the global side provides by fetching chunk
// (l % 4 - l / 16) % 4 into lane l, so that the 16 rows a quarter-wavefront reads fall into
// 16 different 16-byte slots of the 256-byte bank window.
// A workgroup takes TMB tiles of 16 tokens (two when there are more tiles than compute
// units, which halves the router-weight traffic); its 8 wavefronts split the hidden
// dimension into eighths, each with kDepth slices in flight (no workgroup barrier in the
// loop).  The partial tiles are then summed in wavefront order, each
// finishing wavefront taking four tokens of one tile.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// N consecutive 1 KiB blocks of LDS, 16 bytes per lane at byte address addr + 1024 b, then
// the wait for them.  One assembly statement up to the wait: the compiler takes an output for
// valid as soon as its statement ends (and may copy it elsewhere right away).  From assembly
// because for LDS reads it sees, the compiler first waits for every direct-to-LDS load in
// flight, the prefetched slices included.
template <int N>
__device__ __forceinline__ void read_blocks(u32x4 (&o)[N], uint32_t addr) {
  static_assert(N >= 2 && N <= 6, "TMB + NT blocks");
  if constexpr (N == 2)
    asm volatile("ds_read_b128 %0, %2\n\tds_read_b128 %1, %2 offset:1024\n\ts_waitcnt lgkmcnt(0)"
                 : "=&v"(o[0]), "=&v"(o[1]) : "v"(addr) : "memory");
  else if constexpr (N == 3)
    asm volatile("ds_read_b128 %0, %3\n\tds_read_b128 %1, %3 offset:1024\n\t"
                 "ds_read_b128 %2, %3 offset:2048\n\ts_waitcnt lgkmcnt(0)"
                 : "=&v"(o[0]), "=&v"(o[1]), "=&v"(o[2]) : "v"(addr) : "memory");
  else if constexpr (N == 4)
    asm volatile("ds_read_b128 %0, %4\n\tds_read_b128 %1, %4 offset:1024\n\t"
                 "ds_read_b128 %2, %4 offset:2048\n\tds_read_b128 %3, %4 offset:3072\n\t"
                 "s_waitcnt lgkmcnt(0)"
                 : "=&v"(o[0]), "=&v"(o[1]), "=&v"(o[2]), "=&v"(o[3]) : "v"(addr) : "memory");
  else if constexpr (N == 5)
    asm volatile("ds_read_b128 %0, %5\n\tds_read_b128 %1, %5 offset:1024\n\t"
                 "ds_read_b128 %2, %5 offset:2048\n\tds_read_b128 %3, %5 offset:3072\n\t"
                 "ds_read_b128 %4, %5 offset:4096\n\ts_waitcnt lgkmcnt(0)"
                 : "=&v"(o[0]), "=&v"(o[1]), "=&v"(o[2]), "=&v"(o[3]), "=&v"(o[4]) : "v"(addr) : "memory");
  else
    asm volatile("ds_read_b128 %0, %6\n\tds_read_b128 %1, %6 offset:1024\n\t"
                 "ds_read_b128 %2, %6 offset:2048\n\tds_read_b128 %3, %6 offset:3072\n\t"
                 "ds_read_b128 %4, %6 offset:4096\n\tds_read_b128 %5, %6 offset:5120\n\t"
                 "s_waitcnt lgkmcnt(0)"
                 : "=&v"(o[0]), "=&v"(o[1]), "=&v"(o[2]), "=&v"(o[3]), "=&v"(o[4]), "=&v"(o[5])
                 : "v"(addr) : "memory");
}

template <int NT, int TMB>
struct StagedCfg {
  static constexpr int kBlocks = TMB + NT;                       // 1 KiB blocks per slice
  static constexpr int kFit = (96 * 1024) / (kWavesPerBlock * kBlocks * 1024);
  static constexpr int kDepth = kFit < 4 ? kFit : 4;             // slices in flight per wavefront
  static constexpr int kStageBytes = kWavesPerBlock * kDepth * kBlocks * 1024;
  static constexpr int kReduceBytes = kWavesPerBlock * TMB * NT * 4 * 64 * 8;
  static constexpr int kLdsBytes = kStageBytes > kReduceBytes ? kStageBytes : kReduceBytes;
  static_assert(kDepth >= 2, "the next slice must be in flight during the MFMAs of this one");
};

template <int NT, int TMB>
__global__ __launch_bounds__(kWavesPerBlock* kWave) void route_staged_kernel(
    const uint16_t* __restrict__ x, const uint16_t* __restrict__ w_router,
    const float* __restrict__ bias, int T, int H, int E, int k, int bias_group_tokens, int gate_mode,
    float* __restrict__ logits, int32_t* __restrict__ topk_idx, float* __restrict__ topk_gate,
    int32_t* __restrict__ counts, unsigned long long* __restrict__ counts_accum) {
#if defined(__HIP_DEVICE_COMPILE__)   // buffer resources exist in device code only
  using C = StagedCfg<NT, TMB>;
  constexpr int EP = NT * 16;
  constexpr int kBlocks = C::kBlocks, kDepth = C::kDepth;
  __shared__ int s_counts[EP];
  extern __shared__ __align__(16) uint8_t smem[];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int r = lane & 15;
  const int q = lane >> 4;
  const int tok0 = blockIdx.x * (kTokPerBlock * TMB);

  for (int e = threadIdx.x; e < EP; e += blockDim.x) s_counts[e] = 0;
  __syncthreads();

  // ---- global side: lane l fetches row l / 4 of each block, chunk (l % 4 - l / 16) % 4 ----
  const int lrow = lane >> 2;
  const int chunk = ((lane & 3) - (lane >> 4)) & 3;
  uint32_t voff[kBlocks];
#pragma unroll
  for (int b = 0; b < TMB; ++b) {
    const int t = tok0 + b * kTokPerBlock + lrow;
    voff[b] = t < T ? ((uint32_t)t * (uint32_t)H + chunk * 8) * 2u : kOutOfRange;
  }
#pragma unroll
  for (int n = 0; n < NT; ++n) {
    const int e = n * 16 + lrow;
    voff[TMB + n] = e < E ? ((uint32_t)e * (uint32_t)H + chunk * 8) * 2u : kOutOfRange;
  }
  const __amdgpu_buffer_rsrc_t x_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      (void*)x, 0, (int)((uint32_t)T * (uint32_t)H * 2u), kBufferFlags);
  const __amdgpu_buffer_rsrc_t w_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      (void*)w_router, 0, (int)((uint32_t)E * (uint32_t)H * 2u), kBufferFlags);
  uint8_t* const wave_base = smem + wave * (kDepth * kBlocks * 1024);
  const int n_slices = (H + 31) / 32;
  // Fills ring position `buf` with slice s (hidden elements 32 s ..): rows or chunks past
  // the end, and whole slices past the last one, arrive as zeros.  Always kBlocks loads, so
  // the vector-memory counter can be awaited with a constant.
  auto issue = [&](int s, int buf) {
    const bool live = s < n_slices;                       // wavefront-uniform
    const int h0 = live ? s * 32 : 0;
    const bool inside = live && h0 + chunk * 8 < H;
#pragma unroll
    for (int b = 0; b < kBlocks; ++b)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(b < TMB ? x_rsrc : w_rsrc,
                                               (lds_ptr_t)(wave_base + (buf * kBlocks + b) * 1024), 16,
                                               inside ? voff[b] : kOutOfRange, h0 * 2, 0, 0);
  };

  // After the GEMM this wavefront finishes token 4 v + q of tile b; its bias entries are
  // fetched now, so that their latency is not paid at the end.
  const int b_fin = wave >> 2, v_fin = wave & 3;
  const int t_fin = tok0 + b_fin * kTokPerBlock + 4 * v_fin + q;
  float bias_fin[NT];
  load_bias_group<NT>(bias, b_fin < TMB ? t_fin : T, T, E, bias_group_tokens, bias_fin);

  // ---- router GEMM on the fp64 matrix cores -----------------------------------------
  f64x4 acc[TMB][NT];
#pragma unroll
  for (int b = 0; b < TMB; ++b)
#pragma unroll
    for (int n = 0; n < NT; ++n) acc[b][n] = f64x4{0.0, 0.0, 0.0, 0.0};

  // Wavefront w owns the w-th eighth of the slices and walks it cyclically from a phase that
  // keeps the 8 wavefronts 512 bytes (or, where an eighth is a multiple of 4 KiB, 256 bytes)
  // apart modulo 4 KiB: every row of x and of the router weights starts a multiple of 2 H
  // bytes from the base, so all rows at one hidden offset sit in the same memory channels,
  // and all workgroups run in step.  (With each wavefront taking every eighth slice, the
  // whole chip read a 512-byte column window at any time, and the L2 channels holding it
  // bounded the kernel.)  The order is the same for every workgroup, so a token's logits do
  // not depend on where in the batch it sits.
  const int seg = (n_slices + kWavesPerBlock - 1) / kWavesPerBlock;
  const int first = wave * seg;
  const int n_mine = max(0, min(seg, n_slices - first));
  const int phase = n_mine > 0 ? (4 * ((wave * seg) >> 6)) % n_mine : 0;
  auto slice_of = [&](int i) {   // i-th slice this wavefront multiplies; past its last: none
    if (i >= n_mine) return n_slices;
    const int j = i + phase;
    return first + (j >= n_mine ? j - n_mine : j);
  };
#pragma unroll
  for (int d = 0; d < kDepth; ++d) issue(slice_of(d), d);
  // LDS byte address of row r, chunk q of this wavefront's first block
  const uint32_t lds_base = (uint32_t)(uintptr_t)(lds_ptr_t)wave_base +
                            (uint32_t)((r * 4 + ((q + (r >> 2)) & 3)) * 16);
  int buf = 0;
  for (int i = 0; i < n_mine; ++i) {
    wait_vmcnt<(kDepth - 1) * kBlocks>();                 // slice i has landed
    const uint32_t sb = lds_base + buf * (kBlocks * 1024);
    u32x4 blk[kBlocks];
    read_blocks(blk, sb);                                  // waits: read before the refill may overwrite it
    issue(slice_of(i + kDepth), buf);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      auto element = [&](const u32x4& v) {
        const unsigned w = v[j >> 1];
        return (double)((j & 1) ? bf16_hi(w) : bf16_lo(w));
      };
      double a[TMB];
#pragma unroll
      for (int b = 0; b < TMB; ++b) a[b] = element(blk[b]);
#pragma unroll
      for (int n = 0; n < NT; ++n) {
        const double bw = element(blk[TMB + n]);
#pragma unroll
        for (int b = 0; b < TMB; ++b)
          acc[b][n] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[b], bw, acc[b][n], 0, 0, 0);
      }
    }
    buf = buf + 1 == kDepth ? 0 : buf + 1;
  }
  wait_vmcnt<0>();   // the zero-filled refills past the end must land before the LDS is reused
  __syncthreads();

  // ---- partial tiles -> LDS as [wavefront][tile][n][v][lane]; summed in wavefront order ----
  double* part = reinterpret_cast<double*>(smem);
#pragma unroll
  for (int b = 0; b < TMB; ++b)
#pragma unroll
    for (int n = 0; n < NT; ++n)
#pragma unroll
      for (int v = 0; v < 4; ++v)
        part[((((size_t)wave * TMB + b) * NT + n) * 4 + v) * 64 + lane] = acc[b][n][v];
  __syncthreads();
  if (b_fin < TMB) {
    double sum[NT];
#pragma unroll
    for (int n = 0; n < NT; ++n) {
      double s = 0.0;
#pragma unroll
      for (int w = 0; w < kWavesPerBlock; ++w)
        s += part[((((size_t)w * TMB + b_fin) * NT + n) * 4 + v_fin) * 64 + lane];
      sum[n] = s;
    }
    finish_group<NT>(sum, bias_fin, bias != nullptr, t_fin, T, E, k, gate_mode, logits, topk_idx,
                     topk_gate, counts != nullptr ? s_counts : nullptr);
  }
  if (counts == nullptr) return;   // the caller derives the counts from the dispatch histogram

  // ---- per-expert activation counts -----------------------------------------
  __syncthreads();
  for (int e = threadIdx.x; e < E; e += blockDim.x) {
    const int c = s_counts[e];
    if (c != 0) {
      atomicAdd(&counts[e], c);
      if (counts_accum != nullptr) atomicAdd(&counts_accum[e], (unsigned long long)c);
    }
  }
#endif
}

__global__ void fill_i32_kernel(int32_t* p, int n, int32_t v) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// Decode front end, second launch (one workgroup): sums the hidden-dimension slices of
// every token tile in slice order and finishes the routing (each wavefront four tokens of
// every tile), then splits the T*k assignments by placement and builds the schedules of the
// two grouped GEMMs.  The kernel is a chain of short dependent steps on the critical path of
// the layer, so the steps hand their results to each other in LDS (expert indices, local
// offsets): no step waits for a store to memory or re-reads what the step before wrote there.
constexpr int kFrontThreads = dispatch_dev::kThreads;
template <int NT>
__global__ __launch_bounds__(kFrontThreads) void decode_front_end_kernel(
    const double* __restrict__ partial, int n_hsplit, const float* __restrict__ bias, int T, int E,
    int k, int S, int bias_group_tokens, int gate_mode, int32_t* topk_idx,
    float* __restrict__ topk_gate,
    const uint8_t* __restrict__ mask, const dispatch_dev::SplitOut o,
    int32_t* __restrict__ local_src, int32_t* __restrict__ remote_src, int32_t* __restrict__ inv,
    const gg::SchedParams p0, const gg::SchedParams p1) {
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int n_tiles = (T + kTokPerBlock - 1) / kTokPerBlock;
  // asked for now, used by the split: the load's latency passes during the routing
  const int my_mask = (int)threadIdx.x < E ? (int)mask[threadIdx.x] : 0;
  __shared__ int32_t s_idx[kDispatchChunk];                 // topk_idx, for the split
  __shared__ int s_local_off[PRISM_MAX_EXPERTS + 1];        // local_offsets, for the schedules
  // A tile's routing is four units of four tokens (accumulator register v holds tokens
  // 4v + q); wavefront w takes unit v = w of every tile, so even a 16-token batch keeps all
  // four wavefronts busy.  The logits are the sums over the router's slices, in slice order.
  static_assert(kFrontThreads / kWave == 4, "one wavefront per accumulator register index");
  constexpr int kMaxTiles = kDecodeMaxTokens / kTokPerBlock;
  if constexpr (NT <= 4) {
    // All threads share the slice sums -- element j of tile t is a 4-double vector of the
    // NT * 64 that make a tile, its 16 slice loads issued together -- and leave them in LDS.
    __shared__ __align__(32) double s_sum[kMaxTiles * NT * 256];
    for (int item = threadIdx.x; item < n_tiles * NT * 64; item += kFrontThreads) {
      const int tile = item / (NT * 64), j = item % (NT * 64);
      const double* base = partial + (size_t)tile * n_hsplit * (NT * 256) + j * 4;
      f64x4 part[kRouteMaxHSplit];
#pragma unroll
      for (int y = 0; y < kRouteMaxHSplit; ++y)   // slices past the end re-read the last one (unused)
        part[y] = *reinterpret_cast<const f64x4*>(base + (size_t)min(y, n_hsplit - 1) * (NT * 256));
      f64x4 sum = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
      for (int y = 0; y < kRouteMaxHSplit; ++y) {
        const bool on = y < n_hsplit;
#pragma unroll
        for (int v = 0; v < 4; ++v) sum[v] += on ? part[y][v] : 0.0;
      }
      *reinterpret_cast<f64x4*>(s_sum + (size_t)tile * (NT * 256) + j * 4) = sum;
    }
    lds_barrier();
    // Wavefront w routes tokens 4w + q of every tile, two tiles per pass side by side.  The
    // second tile of the last pass may not exist: its tokens are past T, so nothing is stored.
    static_assert(kMaxTiles % 2 == 0, "tile pairs stay inside s_sum");
    const int q = lane >> 4;
    for (int tile = 0; tile < n_tiles; tile += 2) {
      double s2[2][NT];
      float b2[2][NT];
      int t2[2];
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        t2[u] = (tile + u) * kTokPerBlock + 4 * wave + q;
#pragma unroll
        for (int n = 0; n < NT; ++n)   // register v = wave of lane `lane` of the accumulator tile
          s2[u][n] = s_sum[(size_t)(tile + u) * (NT * 256) + n * 256 + lane * 4 + wave];
        load_bias_group<NT>(bias, t2[u], T, E, bias_group_tokens, b2[u]);
      }
      finish_groups<NT, 2>(s2, b2, bias != nullptr, t2, T, E, k, gate_mode, nullptr, topk_idx, topk_gate,
                           nullptr, s_idx);
    }
  } else {
    // Too many expert columns for LDS: every wavefront sums the component it needs itself.
    for (int tile = 0; tile < n_tiles; ++tile) {
      const double* base = partial + (size_t)tile * n_hsplit * (NT * 256) + lane * 4 + wave;
      f64x4 acc[NT];
#pragma unroll
      for (int n = 0; n < NT; ++n) {
        double part[kRouteMaxHSplit];
#pragma unroll
        for (int y = 0; y < kRouteMaxHSplit; ++y)
          part[y] = base[(size_t)min(y, n_hsplit - 1) * (NT * 256) + n * 256];
        double sum = 0.0;
#pragma unroll
        for (int y = 0; y < kRouteMaxHSplit; ++y) sum += y < n_hsplit ? part[y] : 0.0;
        acc[n] = f64x4{sum, sum, sum, sum};         // finish_tile reads component `wave` only
      }
      finish_tile<NT>(acc, tile * kTokPerBlock, 1 << wave, bias, T, E, k, bias_group_tokens, gate_mode,
                      nullptr, topk_idx, topk_gate, nullptr, s_idx);
    }
  }
  lds_barrier();   // s_idx is complete (the copy in memory is for the caller)
  dispatch_dev::dispatch_place_block<false>(s_idx, T * k, E, mask, nullptr, 1, 1, 0, o, local_src,
                                            remote_src, inv, s_local_off, my_mask);
  lds_barrier();   // s_local_off, written by the split
  const gg::SchedParams p[2] = {p0, p1};
  gg::build_schedules_block<2>(s_local_off, E, S, T, T * k, p);
}

// Hidden elements per workgroup of the split router: a multiple of the 256 elements one
// trip of the 8 wavefronts covers, at most kRouteMaxHSplit slices.
inline int route_h_span(int H) { return 256 * ceil_div(H, 256 * kRouteMaxHSplit); }

// Whether route_staged_kernel serves this call (else route_kernel does).
inline bool staged_router_applies(const prism_layer_desc& d, int T) {
  return d.dtype == PRISM_BF16 && T > kDecodeMaxTokens && route_col_tiles(d.n_experts) <= 4 &&
         (uint64_t)T * d.hidden * 2 < 0xFFFF0000ull;
}

template <int NT, int TMB>
prism_status launch_staged_one(const prism_layer_desc& d, const void* x, const void* w,
                               const float* bias, int T, float* logits, int32_t* idx, float* gate,
                               int32_t* counts, int64_t* accum, hipStream_t st) {
  using C = StagedCfg<NT, TMB>;
  static LdsLimitOnce lds_limit;   // more than 64 KiB of dynamic LDS; one per instantiation
  if (!raise_lds_limit(lds_limit, (const void*)route_staged_kernel<NT, TMB>, C::kLdsBytes))
    return PRISM_ERR_LAUNCH;
  hipLaunchKernelGGL((route_staged_kernel<NT, TMB>), dim3(ceil_div(T, kTokPerBlock * TMB)),
                     dim3(kWavesPerBlock * kWave), (size_t)C::kLdsBytes, st, (const uint16_t*)x,
                     (const uint16_t*)w, bias, T, d.hidden, d.n_experts, d.top_k,
                     d.bias_group_tokens, d.gate_mode, logits, idx, gate, counts,
                     (unsigned long long*)accum);
  PRISM_CHECK_LAUNCH();
  return PRISM_OK;
}

prism_status launch_staged(const prism_layer_desc& d, const void* x, const void* w, const float* bias,
                           int T, float* logits, int32_t* idx, float* gate, int32_t* counts,
                           int64_t* accum, hipStream_t st) {
  const int nt = route_col_tiles(d.n_experts);
  const bool two = ceil_div(T, kTokPerBlock) > 256;   // more token tiles than compute units
#define PRISM_STAGED_CASE(NT)                                                                     \
  return two ? launch_staged_one<NT, 2>(d, x, w, bias, T, logits, idx, gate, counts, accum, st)   \
             : launch_staged_one<NT, 1>(d, x, w, bias, T, logits, idx, gate, counts, accum, st)
  if (nt <= 1) PRISM_STAGED_CASE(1);
  if (nt <= 2) PRISM_STAGED_CASE(2);
  PRISM_STAGED_CASE(4);
#undef PRISM_STAGED_CASE
}

template <typename TIn>
prism_status launch_typed(const prism_layer_desc& d, const void* x, const void* w, const float* bias,
                          int T, float* logits, int32_t* idx, float* gate, int32_t* counts,
                          int64_t* accum, double* partial, hipStream_t st) {
  const int E = d.n_experts;
  const int nt = route_col_tiles(E);
  const int h_span = route_h_span(d.hidden);
  const dim3 grid(ceil_div(T, kTokPerBlock), partial != nullptr ? ceil_div(d.hidden, h_span) : 1);
  const dim3 block(kWavesPerBlock * kWave);
  // the 256-expert tile needs 128 KiB of LDS for the partial sums
  if (nt > 8) {
    static LdsLimitOnce lds_full, lds_partial;
    const int bytes = (kWavesPerBlock / 2) * 16 * 4 * 64 * 8;
    if (!raise_lds_limit(lds_full, (const void*)route_kernel<TIn, 16, false>, bytes) ||
        !raise_lds_limit(lds_partial, (const void*)route_kernel<TIn, 16, true>, bytes))
      return PRISM_ERR_LAUNCH;
  }
#define PRISM_ROUTE_LAUNCH(NT, PARTIAL)                                                          \
  hipLaunchKernelGGL((route_kernel<TIn, NT, PARTIAL>), grid, block,                              \
                     (size_t)(kWavesPerBlock / 2) * NT * 4 * 64 * 8, st, (const TIn*)x, (const TIn*)w,  \
                     bias, T, d.hidden, E, d.top_k, d.bias_group_tokens, d.gate_mode, logits,    \
                     idx, gate,                                                                  \
                     counts, (unsigned long long*)accum, h_span, partial)
#define PRISM_ROUTE_CASE(NT)                                                                     \
  do {                                                                                           \
    if (partial != nullptr) PRISM_ROUTE_LAUNCH(NT, true);                                        \
    else PRISM_ROUTE_LAUNCH(NT, false);                                                          \
  } while (0)
  if (nt <= 1) PRISM_ROUTE_CASE(1);
  else if (nt <= 2) PRISM_ROUTE_CASE(2);
  else if (nt <= 4) PRISM_ROUTE_CASE(4);
  else if (nt <= 8) PRISM_ROUTE_CASE(8);
  else PRISM_ROUTE_CASE(16);
#undef PRISM_ROUTE_CASE
#undef PRISM_ROUTE_LAUNCH
  PRISM_CHECK_LAUNCH();
  return PRISM_OK;
}

}  // namespace

prism_status launch_fill_i32(int32_t* p, int n, int32_t v, hipStream_t st) {
  if (n <= 0) return PRISM_OK;
  hipLaunchKernelGGL(fill_i32_kernel, dim3(ceil_div(n, 256)), dim3(256), 0, st, p, n, v);
  PRISM_CHECK_LAUNCH();
  return PRISM_OK;
}

prism_status launch_route(const prism_layer_desc& d, const void* x, const void* w_router,
                          const float* bias, int T, float* logits, int32_t* topk_idx,
                          float* topk_gate, int32_t* counts, int64_t* counts_accum,
                          hipStream_t st) {
  if (counts != nullptr) PRISM_TRY(launch_fill_i32(counts, d.n_experts, 0, st));
  if (T == 0) return PRISM_OK;
  if (d.dtype == PRISM_F32)
    return launch_typed<float>(d, x, w_router, bias, T, logits, topk_idx, topk_gate, counts,
                               counts_accum, nullptr, st);
  if (staged_router_applies(d, T))
    return launch_staged(d, x, w_router, bias, T, logits, topk_idx, topk_gate, counts, counts_accum,
                         st);
  return launch_typed<uint16_t>(d, x, w_router, bias, T, logits, topk_idx, topk_gate, counts,
                                counts_accum, nullptr, st);
}

bool decode_front_end_applies(const prism_layer_desc& d, int T) {
  return d.dtype == PRISM_BF16 && T > 0 && T <= kDecodeMaxTokens;
}

prism_status launch_decode_front_end(const prism_layer_desc& d, const void* x, const void* w_router,
                                     const float* bias, const uint8_t* mask, int T,
                                     int32_t* topk_idx, float* topk_gate, int32_t* counts,
                                     int64_t* counts_accum, int32_t* local_src,
                                     int32_t* local_offsets, int32_t* remote_src,
                                     int32_t* remote_offsets, int32_t* n_local_remote,
                                     int64_t* remote_bytes, int32_t* inv, double* route_part,
                                     int32_t* tiles, hipStream_t st, void* const* stage_events) {
  if (!decode_front_end_applies(d, T) || T * d.top_k > kDispatchChunk) return PRISM_ERR_INVALID_ARG;
  trace(stage_events, PRISM_STAGE_ROUTE, 0, st);
  PRISM_TRY(launch_typed<uint16_t>(d, x, w_router, bias, T, nullptr, nullptr, nullptr, nullptr,
                                   nullptr, route_part, st));
  trace(stage_events, PRISM_STAGE_ROUTE, 1, st);

  const int E = d.n_experts;
  const int n_hsplit = ceil_div(d.hidden, route_h_span(d.hidden));
  const dispatch_dev::SplitOut o{local_offsets, remote_offsets, n_local_remote, remote_bytes, counts,
                                 (unsigned long long*)counts_accum, d.hidden * elem_size(d.dtype)};
  gg::SchedParams p0, p1;
  gg::ffn_sched_params(d, T, tiles, &p0, &p1);
  trace(stage_events, PRISM_STAGE_DISPATCH, 0, st);
#define PRISM_FRONT_CASE(NT)                                                                     \
  hipLaunchKernelGGL((decode_front_end_kernel<NT>), dim3(1), dim3(kFrontThreads), 0, st,        \
                     route_part, n_hsplit, bias, T, E, d.top_k, d.n_shared,                     \
                     d.bias_group_tokens, d.gate_mode, topk_idx, topk_gate, mask, o, local_src,  \
                     remote_src,                                                                 \
                     inv, p0, p1)
  const int nt = route_col_tiles(E);
  if (nt <= 1) PRISM_FRONT_CASE(1);
  else if (nt <= 2) PRISM_FRONT_CASE(2);
  else if (nt <= 4) PRISM_FRONT_CASE(4);
  else if (nt <= 8) PRISM_FRONT_CASE(8);
  else PRISM_FRONT_CASE(16);
#undef PRISM_FRONT_CASE
  PRISM_CHECK_LAUNCH();
  trace(stage_events, PRISM_STAGE_DISPATCH, 1, st);
  return PRISM_OK;
}

}  // namespace prism
