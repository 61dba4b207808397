// Grouped SwiGLU expert FFN over the locally hosted and the shared experts
// (paper Sec. III-A: the local expert execution of a server).
//
//   GEMM1  h[r, f] = silu( x[tok(r)] . W_gate^e[f] ) * ( x[tok(r)] . W_up^e[f] )
//   GEMM2  y[r, n] = h[r] . W_down^e[n]
//
// Both are "NT" contractions (activation rows and weight rows are contiguous
// along the contraction index), grouped by expert: device-built work schedules
// list the (row tile, column tile) items of every hosted expert, so the host
// never needs the routing-dependent segment sizes.
//
// bf16 path: the persistent grouped GEMM of grouped_gemm.h
// (v_mfma_f32_32x32x16_bf16, 4 wavefronts per workgroup, operand k-tiles in an
// LDS ring filled by direct-to-LDS loads), in the tile shapes chosen at the end
// of this file.  GEMM1 loads the gate rows and the up rows of the same f range
// into one tile, so silu(gate)*up is a register epilogue and only h is written.
// Activation rows of GEMM1 are gathered through local_src (no permuted copy of
// x is materialised).
#include "grouped_gemm.h"
#include "prism_internal.h"

namespace prism {
static bool stream_tiles_apply(const prism_layer_desc& d, int T);
namespace {

// ---------------------------------------------------------------------------
// fp32 path (small layers only): one wavefront per output element, the
// contraction split over lanes and reduced with shuffles.
// ---------------------------------------------------------------------------
struct F32Args {
  const float* x;
  const void* const* wg; const void* const* wu; const void* const* wd;
  const void* const* swg; const void* const* swu; const void* const* swd;
  const int32_t* local_src; const int32_t* local_offsets;
  float* h; float* y;
  int T, H, F, E, S, top_k;
};

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
  return v;
}

// Resolves output row r to (group, token); returns false for rows that hold nothing.
__device__ __forceinline__ bool resolve_row(const F32Args& p, int r, int& g, int& tok) {
  const int A = p.T * p.top_k;
  if (r >= A) {
    const int s = (r - A) / p.T;
    g = p.E + s;
    tok = (r - A) - s * p.T;
    return true;
  }
  if (r >= p.local_offsets[p.E]) return false;
  int e = 0;
  while (p.local_offsets[e + 1] <= r) ++e;
  g = e;
  tok = p.local_src[r] / p.top_k;
  return true;
}

constexpr int kF32ColsPerBlock = 64;

__global__ __launch_bounds__(256) void ffn1_f32_kernel(const F32Args p) {
  extern __shared__ float s_x[];
  __shared__ int s_g, s_tok, s_ok;
  const int r = blockIdx.x;
  if (threadIdx.x == 0) {
    int g = 0, tok = 0;
    s_ok = resolve_row(p, r, g, tok) ? 1 : 0;
    s_g = g; s_tok = tok;
  }
  __syncthreads();
  if (!s_ok) return;
  const int g = s_g;
  for (int i = threadIdx.x; i < p.H; i += blockDim.x) s_x[i] = p.x[(size_t)s_tok * p.H + i];
  __syncthreads();
  const float* wg = (const float*)(g < p.E ? p.wg[g] : p.swg[g - p.E]);
  const float* wu = (const float*)(g < p.E ? p.wu[g] : p.swu[g - p.E]);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int i = wave; i < kF32ColsPerBlock; i += 4) {
    const int f = blockIdx.y * kF32ColsPerBlock + i;
    if (f >= p.F) break;
    float ag = 0.f, au = 0.f;
    for (int hh = lane; hh < p.H; hh += 64) {
      const float xv = s_x[hh];
      ag = fmaf(xv, wg[(size_t)f * p.H + hh], ag);
      au = fmaf(xv, wu[(size_t)f * p.H + hh], au);
    }
    ag = wave_sum(ag);
    au = wave_sum(au);
    if (lane == 0) p.h[(size_t)r * p.F + f] = (ag / (1.0f + expf(-ag))) * au;
  }
}

__global__ __launch_bounds__(256) void ffn2_f32_kernel(const F32Args p) {
  extern __shared__ float s_h[];
  __shared__ int s_g, s_ok;
  const int r = blockIdx.x;
  if (threadIdx.x == 0) {
    int g = 0, tok = 0;
    s_ok = resolve_row(p, r, g, tok) ? 1 : 0;
    s_g = g;
  }
  __syncthreads();
  if (!s_ok) return;
  const int g = s_g;
  for (int i = threadIdx.x; i < p.F; i += blockDim.x) s_h[i] = p.h[(size_t)r * p.F + i];
  __syncthreads();
  const float* wd = (const float*)(g < p.E ? p.wd[g] : p.swd[g - p.E]);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int i = wave; i < kF32ColsPerBlock; i += 4) {
    const int n = blockIdx.y * kF32ColsPerBlock + i;
    if (n >= p.H) break;
    float acc = 0.f;
    for (int f = lane; f < p.F; f += 64) acc = fmaf(s_h[f], wd[(size_t)n * p.F + f], acc);
    acc = wave_sum(acc);
    if (lane == 0) p.y[(size_t)r * p.H + n] = acc;
  }
}

// ---------------------------------------------------------------------------
// bf16 path: two grouped GEMMs on the matrix cores
// ---------------------------------------------------------------------------
template <int BM_, int BN_, int BK_, int STAGES_> struct TileCfg {
  static constexpr int BM = BM_, BN = BN_, BK = BK_, STAGES = STAGES_;
};

// Fixed cost of one round of items of a split down projection, as weight bytes a workgroup
// could have streamed meanwhile (first loads of the ring, epilogue, partial-tile stores): fitted
// to the times of a 32-token batch of the 4096 x 14336 layer run with 2 to 8 splits.
constexpr float kSplitRoundBytes = 14 * 8192.f;

// What the schedule builders need to know about a path's two GEMMs (C1: gate/up, C2: down).
template <typename C1, typename C2, bool SPLIT_DOWN>
FfnShapes shapes_of(const prism_layer_desc& d, int T) {
  FfnShapes f{};
  f.bm1 = C1::BM;
  f.nt1 = ceil_div(d.ffn, C1::BN / 2);     // GEMM1 tile: BN/2 gate rows + BN/2 up rows
  f.bm2 = C2::BM;
  f.nt2 = ceil_div(d.hidden, C2::BN);
  f.interleave = SPLIT_DOWN;               // the paths that stream the weights once
  // prefill tiles: the down projection's last round may be cut along its contraction
  f.slice_kt2 = !SPLIT_DOWN && C2::BM == 256 && down_slicing_applies(d, T) ? d.ffn / C2::BK : 0;
  if (SPLIT_DOWN) {
    f.split_kt2 = d.ffn / C2::BK;
    f.split_min_kt2 = C2::STAGES - 1;      // a slice must be at least as long as the k-tile ring
    f.split_wgs2 = gg::gemm_wgs_per_xcd<C2::BM, C2::BN, 2, C2::BK, C2::STAGES, false, true>();
    const float kt_bytes = (float)(C2::BN * C2::BK * 2);   // weight bytes of one k-tile
    f.split_round_kt2 = kSplitRoundBytes / kt_bytes;
    // one more split: every row written once more as fp32 and read once more, shared by all workgroups
    f.split_row_kt2 = (float)d.hidden * 8.f / (float)(gg::kXcds * f.split_wgs2) / kt_bytes;
  }
  return f;
}

// Sums the contraction slices of the split down projection: y = bf16(sum_s part[s]).
__global__ __launch_bounds__(256) void reduce_splits_kernel(const float* __restrict__ part,
                                                            const int32_t* __restrict__ local_offsets,
                                                            int E, int A, int rows, int H,
                                                            const int32_t* __restrict__ n_splits_ptr,
                                                            uint16_t* __restrict__ y) {
  const int n_splits = min(*n_splits_ptr, kDecodeSplits);   // what the schedule builder chose
  const int vec_per_row = H / 4;
  const long long gid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= (long long)rows * vec_per_row) return;
  const int row = (int)(gid / vec_per_row);
  if (row >= local_offsets[E] && row < A) return;   // rows that hold no assignment
  const int col = (int)(gid - (long long)row * vec_per_row) * 4;
  f32x4 v[kDecodeSplits];   // all slices asked for before the first is added
#pragma unroll
  for (int s = 0; s < kDecodeSplits; ++s)
    if (s < n_splits) v[s] = *reinterpret_cast<const f32x4*>(part + ((size_t)s * rows + row) * H + col);
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int s = 0; s < kDecodeSplits; ++s)
    if (s < n_splits) acc += v[s];
  bf16x4 o;
#pragma unroll
  for (int e = 0; e < 4; ++e) o[e] = (bf16_t)acc[e];
  *reinterpret_cast<bf16x4*>(y + (size_t)row * H + col) = o;
}

// Adds up the slices of the down-projection tiles whose contraction the schedule cut (its last
// round of work items): y tile = bf16(sum of the tile's fp32 partial tiles, in slice order).
// One workgroup per (line of the schedule's list of sliced items, 16 rows of the tile) -- few
// lines are in use at a time, so the rows of a tile are spread over many workgroups; lines that
// are not in use end at once.
constexpr int kSliceTile = 256;    // the partial tiles are 256 x 256 (the prefill tile)
constexpr int kSumRows = 16;       // rows of a tile per workgroup of sum_slices_kernel
constexpr int kSumChunks = kSliceTile / kSumRows;
__global__ __launch_bounds__(256) void sum_slices_kernel(const int32_t* __restrict__ sched, int capacity,
                                                         const float* __restrict__ part, int N,
                                                         uint16_t* __restrict__ y) {
  const int line = blockIdx.x / kSumChunks, chunk = blockIdx.x % kSumChunks;
  const int4* red = reinterpret_cast<const int4*>(sched + gg::sched_reduce_offset(capacity)) +
                    (size_t)line * (gg::kReduceInts / 4);
  const int n_slices = red[1].x;
  if (n_slices <= 0) return;
  const int4 a = red[0];
  const int row_start = a.x, row_count = a.y, first = a.w;
  const int row_end = min(row_count, chunk * kSumRows + kSumRows);
  const int col0 = a.z * kSliceTile;
  const int col = (threadIdx.x & 63) * 4;
  if (col0 + col >= N) return;
  // Two rows per wavefront and pass; all slices of both rows are asked for before the first is
  // added (the partial tiles are read once: non-temporal); the sums themselves run in slice order.
  for (int r0 = chunk * kSumRows + (threadIdx.x >> 6); r0 < row_end; r0 += 8) {
    f32x4 v[2][gg::kMaxSlices];
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int c = 0; c < gg::kMaxSlices; ++c)
        if (c < n_slices && r0 + 4 * u < row_end)
          v[u][c] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(
              part + ((size_t)(first + c) * kSliceTile + r0 + 4 * u) * kSliceTile + col));
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      if (r0 + 4 * u >= row_end) break;
      f32x4 sum = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int c = 0; c < gg::kMaxSlices; ++c)
        if (c < n_slices) sum += v[u][c];
      bf16x4 o;
#pragma unroll
      for (int e = 0; e < 4; ++e) o[e] = (bf16_t)sum[e];
      *reinterpret_cast<bf16x4*>(y + (size_t)(row_start + r0 + 4 * u) * N + col0 + col) = o;
    }
  }
}

template <typename C1, typename C2, bool SPLIT_DOWN, bool STREAM_B = false>
prism_status run_bf16_ffn(const prism_layer_desc& d, const void* x, const prism_expert_weights& w,
                          const int32_t* local_src, const int32_t* local_offsets, int T, void* y,
                          void* h, int32_t* tiles, float* part, float* slice_part, hipStream_t st,
                          void* const* stage_events, const int32_t** deferred_splits,
                          bool schedules_built) {
  using gg::GemmArgs;
  constexpr bool kRotate = SPLIT_DOWN;   // the decode path: no weight tile is shared between items
  const int A = T * d.top_k;
  const int rows = A + d.n_shared * T;
  // the k-tile ring of a workgroup must not be longer than its contraction slice
  if (d.hidden / C1::BK < C1::STAGES - 1 || d.ffn / C2::BK < C2::STAGES - 1) return PRISM_ERR_UNSUPPORTED;
  int32_t* sched1 = tiles;
  int32_t* sched2 = tiles + tile_table_ints(d, T);
  // The schedules (built here, or by the caller's dispatch) follow ffn_schedule_shapes(), which
  // must describe the kernels this instantiation launches.
  const FfnShapes f = shapes_of<C1, C2, SPLIT_DOWN>(d, T);
  const FfnShapes told = ffn_schedule_shapes(d, T);
  if (f.bm1 != told.bm1 || f.nt1 != told.nt1 || f.bm2 != told.bm2 || f.nt2 != told.nt2 ||
      f.interleave != told.interleave || f.slice_kt2 != told.slice_kt2 || f.split_kt2 != told.split_kt2 ||
      f.split_wgs2 != told.split_wgs2)
    return PRISM_ERR_LAUNCH;
  const int nt1 = f.nt1, nt2 = f.nt2;
  // the down projection's last round of items may be cut along the contraction (prefill only)
  const int slice_kt = slice_part != nullptr ? f.slice_kt2 : 0;
  if (slice_kt != f.slice_kt2) return PRISM_ERR_INVALID_ARG;   // the schedule would hold slice entries
  static_assert(SPLIT_DOWN || (C2::BM == kSliceTile && C2::BN == kSliceTile && C2::BK == 32),
                "sum_slices_kernel assumes the prefill tile");
  if (!schedules_built) PRISM_TRY(gg::launch_build_schedules(d, local_offsets, T, tiles, st));

  GemmArgs g1{};
  g1.A = (const uint16_t*)x;
  g1.B0 = w.w_gate; g1.B1 = w.w_up; g1.SB0 = w.shared_w_gate; g1.SB1 = w.shared_w_up;
  g1.C = (uint16_t*)h;
  g1.sched = sched1; g1.local_src = local_src;
  g1.src_bytes = (uint32_t)A * 4;
  g1.a_bytes = (uint32_t)((size_t)T * d.hidden * 2);
  g1.b_bytes = (uint32_t)((size_t)d.ffn * d.hidden * 2);
  g1.K = d.hidden; g1.N = d.ffn; g1.top_k = d.top_k; g1.E = d.n_experts;
  g1.b_tiled = d.weight_layout == PRISM_WEIGHTS_TILED;
  trace(stage_events, PRISM_STAGE_FFN_UP, 0, st);
  PRISM_TRY((gg::launch_gemm<C1::BM, C1::BN, 2, 2, C1::BK, C1::STAGES, true, false, kRotate, STREAM_B>(
      g1, gg::sched_capacity(d, T, C1::BM, nt1), st)));
  trace(stage_events, PRISM_STAGE_FFN_UP, 1, st);

  GemmArgs g2{};
  g2.A = (const uint16_t*)h;
  g2.B0 = w.w_down; g2.B1 = nullptr; g2.SB0 = w.shared_w_down; g2.SB1 = nullptr;
  g2.C = (uint16_t*)y;
  g2.Cpart = SPLIT_DOWN ? part : slice_part; g2.c_rows = rows;
  g2.sched = sched2; g2.local_src = local_src;
  g2.a_bytes = (uint32_t)((size_t)rows * d.ffn * 2);
  g2.b_bytes = (uint32_t)((size_t)d.ffn * d.hidden * 2);
  g2.K = d.ffn; g2.N = d.hidden; g2.top_k = d.top_k; g2.E = d.n_experts;
  g2.b_tiled = d.weight_layout == PRISM_WEIGHTS_TILED;
  // SPLIT_DOWN: the number of contraction slices is in the schedule's header (schedule.h, "Splits")
  const int32_t* n_splits = sched2 + 2;
  trace(stage_events, PRISM_STAGE_FFN_DOWN, 0, st);
  PRISM_TRY((gg::launch_gemm<C2::BM, C2::BN, 2, 2, C2::BK, C2::STAGES, false, SPLIT_DOWN, kRotate, STREAM_B>(
      g2, gg::sched_capacity(d, T, C2::BM, nt2), st)));
  if constexpr (!SPLIT_DOWN) {
    if (slice_kt > 0)   // the cut last round: one slice entry per workgroup, fp32 partial tiles
      PRISM_TRY((gg::launch_gemm<C2::BM, C2::BN, 2, 2, C2::BK, C2::STAGES, false, false, false, false, true>(
          g2, gg::sched_capacity(d, T, C2::BM, nt2), st)));
  }
  if (slice_kt > 0) {
    hipLaunchKernelGGL(sum_slices_kernel, dim3(gg::kXcds * (gg::kSliceSlots / 2) * kSumChunks), dim3(256), 0, st, sched2,
                       gg::sched_capacity(d, T, C2::BM, nt2), slice_part, d.hidden, (uint16_t*)y);
    PRISM_CHECK_LAUNCH();
  }
  if (SPLIT_DOWN && deferred_splits != nullptr) {
    *deferred_splits = n_splits;   // the caller's combine sums the slices itself
  } else if (SPLIT_DOWN) {
    const long long threads = (long long)rows * (d.hidden / 4);
    hipLaunchKernelGGL(reduce_splits_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st,
                       part, local_offsets, d.n_experts, A, rows, d.hidden, n_splits, (uint16_t*)y);
    PRISM_CHECK_LAUNCH();
  }
  trace(stage_events, PRISM_STAGE_FFN_DOWN, 1, st);
  return PRISM_OK;
}

// One tile path of the bf16 FFN: tile shapes of the two GEMMs, whether the down projection is
// split along its contraction, whether the weight loads are marked non-temporal.
template <typename C1_, typename C2_, bool SPLIT_DOWN_, bool STREAM_B_> struct Path {
  using C1 = C1_;
  using C2 = C2_;
  static constexpr bool kSplitDown = SPLIT_DOWN_, kStreamB = STREAM_B_;
};

// Calls fn(Path<...>{}) with the path that serves a bf16 batch of T tokens of layer d.
template <typename Fn>
auto select_path(const prism_layer_desc& d, int T, Fn&& fn) {
  if (T <= kDecodeMaxTokens) {
    // Decode batch: every expert has at most 64 rows, the layer is bound by streaming
    // the weights once.  Small tiles make ~1000 work items; the down projection also
    // splits its contraction (the slices are summed by a last kernel or by the combine).
    // No weight tile is shared between workgroups here, so every item starts its
    // contraction at a different k-tile: at any moment the workgroups then read
    // different column ranges of the weight rows, whose power-of-two pitch would
    // otherwise send them all to the same few memory channels.
    // Tiled weights: 32-wide k-tiles, so that one load instruction takes one whole 1 KiB
    // tile (with 64-wide k-tiles it would take halves of two), and twice the stages.
    // An expert has one row tile here, so every weight element is read by exactly one
    // workgroup, once: the weight loads are marked non-temporal (see STREAM_B).
    if (d.weight_layout == PRISM_WEIGHTS_TILED && d.hidden >= 256 && d.ffn >= 1024)
      return fn(Path<TileCfg<64, 128, 32, 8>, TileCfg<64, 128, 32, 8>, true, true>{});
    if (d.hidden >= 192 && d.ffn >= 192)
      return fn(Path<TileCfg<64, 128, 64, 4>, TileCfg<64, 128, 64, 4>, true, true>{});
    return fn(Path<TileCfg<64, 128, 32, 3>, TileCfg<64, 128, 32, 3>, true, true>{});
  }
  // Batches of a few hundred tokens of a wide layer are still bound by streaming the weights
  // once, but an expert now has up to a few hundred rows; the down projection splits its
  // contraction as for decode batches.
  // Up to 256 tokens: 128 x 128 tiles with 64-wide k-tiles, weight loads non-temporal.  Up to
  // 128 tokens an expert has a single row tile (a token picks an expert at most once), so the
  // weights are read once and stream; between 129 and 256 the few experts with more than 128
  // rows read theirs twice, which still beats the wider tiles of the next case (4096 x 14336
  // layer, 5 of 8 experts hosted: 0.386 against 0.418 ms at 128 tokens, 0.381 against 0.413 at
  // 129, 0.450 against 0.470 at 192, 0.470 against 0.480 at 256; at 320 they lose, 0.555 against
  // 0.536).
  if (stream_tiles_apply(d, T) && T <= kMidMaxTokens)
    return fn(Path<TileCfg<128, 128, 64, 4>, TileCfg<128, 128, 64, 4>, true, true>{});
  // Beyond, most experts have several row tiles, which share weight tiles through the L2 (the
  // non-temporal hint costs 8-13 % there).  Tiles twice as wide in weight rows (256) as in
  // activation rows (128) bring twice the HBM bytes per k-tile for the same waits and barriers,
  // and the padding rows of a half-empty 256-row tile would cost their loads and MFMAs like
  // real ones (256 x 128 tiles: 0.590 against 0.546 ms at 352 tokens; the 256 x 256 prefill
  // tiles: their down projection has too few items to fill the machine).
  if (stream_tiles_apply(d, T))
    return fn(Path<TileCfg<128, 256, 32, 6>, TileCfg<128, 256, 32, 6>, true, false>{});
  // Prefill batch: 256 x 256 tiles (GEMM1: 128 gate + 128 up weight rows).  Very short
  // contractions (H or F of 64) get the shallowest ring.
  if (d.hidden >= 128 && d.ffn >= 128)
    return fn(Path<TileCfg<256, 256, 32, 4>, TileCfg<256, 256, 32, 4>, false, false>{});
  return fn(Path<TileCfg<256, 256, 32, 3>, TileCfg<256, 256, 32, 3>, false, false>{});
}

}  // namespace

prism_status launch_expert_ffn(const prism_layer_desc& d, const void* x,
                               const prism_expert_weights& w, const int32_t* local_src,
                               const int32_t* local_offsets, int T, void* y, void* h,
                               int32_t* tiles, float* part, float* slice_part, hipStream_t st,
                               void* const* stage_events, const int32_t** deferred_splits,
                               bool schedules_built) {
  if (deferred_splits != nullptr) *deferred_splits = nullptr;
  if (T == 0) return PRISM_OK;
  const int A = T * d.top_k;
  const int rows = A + d.n_shared * T;
  if (d.dtype == PRISM_F32) {
    if (d.weight_layout != PRISM_WEIGHTS_ROW_MAJOR) return PRISM_ERR_UNSUPPORTED;
    F32Args a{(const float*)x, w.w_gate, w.w_up, w.w_down, w.shared_w_gate, w.shared_w_up,
              w.shared_w_down, local_src, local_offsets, (float*)h, (float*)y,
              T, d.hidden, d.ffn, d.n_experts, d.n_shared, d.top_k};
    if ((size_t)d.hidden * 4 > 64 * 1024 || (size_t)d.ffn * 4 > 64 * 1024) return PRISM_ERR_UNSUPPORTED;
    trace(stage_events, PRISM_STAGE_FFN_UP, 0, st);
    hipLaunchKernelGGL(ffn1_f32_kernel, dim3(rows, ceil_div(d.ffn, kF32ColsPerBlock)), dim3(256),
                       (size_t)d.hidden * 4, st, a);
    PRISM_CHECK_LAUNCH();
    trace(stage_events, PRISM_STAGE_FFN_UP, 1, st);
    trace(stage_events, PRISM_STAGE_FFN_DOWN, 0, st);
    hipLaunchKernelGGL(ffn2_f32_kernel, dim3(rows, ceil_div(d.hidden, kF32ColsPerBlock)), dim3(256),
                       (size_t)d.ffn * 4, st, a);
    PRISM_CHECK_LAUNCH();
    trace(stage_events, PRISM_STAGE_FFN_DOWN, 1, st);
    return PRISM_OK;
  }

  // bf16: schedules for the two GEMMs, then the GEMMs.  Buffer addressing uses
  // 32-bit byte offsets, so every operand matrix must stay below 4 GiB.
  constexpr size_t kMaxOperandBytes = 0xFFFF0000ull;
  if ((size_t)T * d.hidden * 2 >= kMaxOperandBytes || (size_t)rows * d.ffn * 2 >= kMaxOperandBytes ||
      (size_t)d.ffn * d.hidden * 2 >= kMaxOperandBytes)
    return PRISM_ERR_UNSUPPORTED;
  return select_path(d, T, [&](auto path) {
    using P = decltype(path);
    return run_bf16_ffn<typename P::C1, typename P::C2, P::kSplitDown, P::kStreamB>(
        d, x, w, local_src, local_offsets, T, y, h, tiles, part, slice_part, st, stage_events, deferred_splits,
        schedules_built);
  });
}

// Batches between the decode and the prefill sizes of layers wide enough for the 6-stage ring,
// if the down projection in prefill tiles would have too few items for the machine: column
// tiles x row tiles, the latter estimated from what the host knows (half of the experts
// hosted, rows spread evenly).  Layers of many small experts have enough items at any batch
// size and run as fast or faster in prefill tiles (measured at E = 60 / 64 with 4 / 2 shared
// experts: within 3 % up to 256 tokens, 5-18 % faster from 384).
static bool stream_tiles_apply(const prism_layer_desc& d, int T) {
  const int t_max = slicing_shape(d) ? kStreamMaxTokensSliced : kStreamMaxTokens;
  if (T <= kDecodeMaxTokens || T > t_max || d.hidden < 256 || d.ffn < 1024) return false;
  const int row_tiles = ceil_div(T * d.top_k, 256) + d.n_experts / 2 + d.n_shared * ceil_div(T, 256);
  return row_tiles * ceil_div(d.hidden, 256) <= 128;
}

FfnShapes ffn_schedule_shapes(const prism_layer_desc& d, int T) {
  return select_path(d, T, [&](auto path) {
    using P = decltype(path);
    return shapes_of<typename P::C1, typename P::C2, P::kSplitDown>(d, T);
  });
}

}  // namespace prism
