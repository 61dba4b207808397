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
#include "prism_internal.h"

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

// NT = number of 16-expert column tiles (E <= 16 * NT).
template <typename TIn, int NT>
__global__ __launch_bounds__(kWavesPerBlock* kWave) void route_kernel(
    const TIn* __restrict__ x, const TIn* __restrict__ w_router, const float* __restrict__ bias,
    int T, int H, int E, int k, int bias_group_tokens, float* __restrict__ logits,
    int32_t* __restrict__ topk_idx, float* __restrict__ topk_gate, int32_t* __restrict__ counts,
    unsigned long long* __restrict__ counts_accum) {
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

  // wavefront w takes the 32-element slices w, w + 8, w + 16, ... of the hidden dimension
  for (int h0 = wave * 32; h0 < H; h0 += 32 * kWavesPerBlock) {
    // H % 8 == 0, so a lane's 8-element chunk is entirely inside or outside;
    // lanes past the end feed zeros (the MFMA itself is wave-wide).
    const int h = h0 + q * 8;
    const bool inside = h < H;
    const int hl = inside ? h : 0;
    float xa[8];
    load8(xrow + hl, xa);
    float wb[NT][8];
#pragma unroll
    for (int n = 0; n < NT; ++n) load8(wrow[n] + hl, wb[n]);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const double a = inside ? (double)xa[j] : 0.0;
#pragma unroll
      for (int n = 0; n < NT; ++n)
        acc[n] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, (double)wb[n][j], acc[n], 0, 0, 0);
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

  // ---- one rounding to fp32, then the fp32 bias add --------------------------
  // Accumulator register v of lane (r, q) is token 4v + q, expert 16n + r.
  float lg[NT][4];
#pragma unroll
  for (int n = 0; n < NT; ++n) {
    const int e = n * 16 + r;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int t = tok0 + 4 * v + q;
      float val = (float)acc[n][v];
      if (e < E && t < T) {
        if (bias != nullptr) {
          const int row = bias_group_tokens > 0 ? t / bias_group_tokens : 0;
          val = val + bias[(size_t)row * E + e];
        }
        if (logits != nullptr) logits[(size_t)t * E + e] = val;
      } else if (e >= E) {
        val = -INFINITY;
      }
      lg[n][v] = val;
    }
  }

  // ---- top-k: each 16-lane group owns one token per register index v ---------
  // k rounds of arg-max over (logit, expert index) with xor-shuffles inside the
  // group; equal logits resolve to the lower expert index.
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    const int t = tok0 + 4 * v + q;
    float vals[NT];
#pragma unroll
    for (int n = 0; n < NT; ++n) vals[n] = lg[n][v];
    float sel0 = 0.f, mysel = 0.f;
    int myidx = 0;
    for (int j = 0; j < k; ++j) {
      float best = vals[0];
      int bidx = r;
#pragma unroll
      for (int n = 1; n < NT; ++n)
        if (vals[n] > best) { best = vals[n]; bidx = n * 16 + r; }
#pragma unroll
      for (int off = 8; off >= 1; off >>= 1) {
        const float ov = __shfl_xor(best, off);
        const int oi = __shfl_xor(bidx, off);
        if (ov > best || (ov == best && oi < bidx)) { best = ov; bidx = oi; }
      }
      // every lane of the group holds the winner; its owner retires it
#pragma unroll
      for (int n = 0; n < NT; ++n)
        if (bidx == n * 16 + r) vals[n] = -INFINITY;
      if (j == 0) sel0 = best;
      if (r == j) { mysel = best; myidx = bidx; }
    }
    // gates: softmax over the k picked logits; lane r < k owns slot r
    double w = r < k ? exp((double)mysel - (double)sel0) : 0.0;
    double sum = w;
#pragma unroll
    for (int off = 8; off >= 1; off >>= 1) sum += __shfl_xor(sum, off);
    if (r < k && t < T) {
      topk_idx[(size_t)t * k + r] = myidx;
      topk_gate[(size_t)t * k + r] = (float)(w / sum);
      atomicAdd(&s_counts[myidx], 1);
    }
  }
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

__global__ void fill_i32_kernel(int32_t* p, int n, int32_t v) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

template <typename TIn>
prism_status launch_typed(const prism_layer_desc& d, const void* x, const void* w, const float* bias,
                          int T, float* logits, int32_t* idx, float* gate, int32_t* counts,
                          int64_t* accum, hipStream_t st) {
  const int E = d.n_experts;
  const int nt = ceil_div(E, 16);
  const dim3 grid(ceil_div(T, kTokPerBlock)), block(kWavesPerBlock * kWave);
  static bool attr_set = false;
  if (!attr_set) {   // the 256-expert tile needs 128 KiB of LDS for the partial sums
    if (hipFuncSetAttribute((const void*)route_kernel<TIn, 16>,
                            hipFuncAttributeMaxDynamicSharedMemorySize,
                            (kWavesPerBlock / 2) * 16 * 4 * 64 * 8) != hipSuccess)
      return PRISM_ERR_LAUNCH;
    attr_set = true;
  }
#define PRISM_ROUTE_CASE(NT)                                                                     \
  hipLaunchKernelGGL((route_kernel<TIn, NT>), grid, block,                                      \
                     (size_t)(kWavesPerBlock / 2) * NT * 4 * 64 * 8, st, (const TIn*)x, (const TIn*)w,  \
                     bias, T, d.hidden, E, d.top_k, d.bias_group_tokens, logits, idx, gate,     \
                     counts, (unsigned long long*)accum)
  if (nt <= 1) PRISM_ROUTE_CASE(1);
  else if (nt <= 2) PRISM_ROUTE_CASE(2);
  else if (nt <= 4) PRISM_ROUTE_CASE(4);
  else if (nt <= 8) PRISM_ROUTE_CASE(8);
  else PRISM_ROUTE_CASE(16);
#undef PRISM_ROUTE_CASE
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
  PRISM_TRY(launch_fill_i32(counts, d.n_experts, 0, st));
  if (T == 0) return PRISM_OK;
  if (d.dtype == PRISM_F32)
    return launch_typed<float>(d, x, w_router, bias, T, logits, topk_idx, topk_gate, counts,
                               counts_accum, st);
  return launch_typed<uint16_t>(d, x, w_router, bias, T, logits, topk_idx, topk_gate, counts,
                                counts_accum, st);
}

}  // namespace prism
