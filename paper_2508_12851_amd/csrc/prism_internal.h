// Internal declarations shared by the HIP translation units of libprism.
#ifndef PRISM_INTERNAL_H_
#define PRISM_INTERNAL_H_

#include <hip/hip_runtime.h>
#include <algorithm>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

#include "prism.h"

namespace prism {

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef double f64x4 __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
static inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// ---------------------------------------------------------------------------
// Workspace layout.  One layout serves every entry point, so a buffer sized by
// prism_workspace_bytes() fits all of them.
// ---------------------------------------------------------------------------
constexpr int kDispatchChunk = 2048;   // assignments per dispatch block
constexpr int kDecodeMaxTokens = 64;    // batches up to this size take the weight-streaming path
constexpr int kDecodeSplits = 8;        // most contraction slices of its down projection (the schedule builder picks how many) ...
constexpr int kStreamSplits = 4;        // ... and of batches with more than kManySplitsRows rows that still split it
constexpr int kManySplitsRows = 256;    // (every slice is one more fp32 copy of all rows)
constexpr int kStreamMaxTokens = 512;   // wide bf16 layers: batches up to this size also split the down projection (expert_ffn.hip)
constexpr int kMidMaxTokens = 256;      // ... and up to this size they run in 128 x 128 tiles (expert_ffn.hip)
constexpr int kMinTileM = 64;           // smallest row tile of the grouped GEMM (bounds table sizes)
constexpr int kRouteTokTile = 16;       // tokens per router tile
constexpr int kRouteMaxHSplit = 16;     // hidden-dimension slices of the decode router

struct Workspace {
  int32_t* local_src;      // [A]
  int32_t* local_offsets;  // [E+1]
  int32_t* inv;            // [A]  row of assignment a in y, or -1 when remote
  int32_t* block_hist;     // [n_chunks * E]
  int32_t* tiles;          // 2 x [tile_table_ints]: schedules of the two grouped GEMMs
  void* h;                 // [(A + S*T) * F] layer dtype: silu(gate)*up
  void* y;                 // [(A + S*T) * H] layer dtype: expert outputs
  float* part;             // batches up to kStreamMaxTokens: [max_splits(T)][A + S*T][H] fp32 partial sums
  float* slice_part;       // larger batches of wide layers: 256 partial tiles of 256 x 256 fp32 (cut last round of the down projection)
  double* route_part;      // decode batches: [token tiles][kRouteMaxHSplit][route_col_tiles][64][4] fp64
  size_t total;
};

static inline int elem_size(int dtype) { return dtype == PRISM_F32 ? 4 : 2; }

// 16-expert column tiles of the router kernels: ceil(E / 16) rounded up to a power of two
// (the kernels are instantiated for 1, 2, 4, 8 and 16 tiles).
static inline int route_col_tiles(int n_experts) {
  int nt = 1;
  while (nt * 16 < n_experts) nt *= 2;
  return nt;
}

// ints in one GEMM schedule (schedule.h): a 32-int header, 8 per-XCD lists of 8-int entries -- a
// list holds at most (row tiles) x ceil(column tiles / 8) items (bounds for the smallest tiles
// used) plus 32 entries for a last round cut into slices -- and the list of sliced items
// (8 x 16 lines of 8 ints)
static inline size_t tile_table_ints(const prism_layer_desc& d, int T) {
  const size_t A = (size_t)T * d.top_k;
  const size_t mt = A / kMinTileM + d.n_experts + (size_t)d.n_shared * ceil_div(T > 0 ? T : 1, kMinTileM) + 1;
  const int wide = d.ffn > d.hidden ? d.ffn : d.hidden;
  const size_t nj8 = ceil_div(ceil_div(wide > 0 ? wide : 1, 64), 8);
  return align_up(32 + 8 * 8 * (mt * nj8 + 32) + 8 * 16 * 8, 64);
}

// Partial tiles of a down projection whose last round of work items is cut along the contraction:
// one tile per workgroup.  Prefill batches of layers whose contraction is long enough for the cut
// to pay: an item of K / 32 k-tiles takes about 0.74 us per k-tile, the cut saves at least half of
// one item per launch and costs two short launches plus up to 64 MB of fp32 tiles written and read
// (about 40 us); with fewer than 128 k-tiles (the gate/up GEMM of the same layers included, whose
// contraction is H) it was measured to lose.
constexpr int kSliceMinFfn = 4096;
// With the cut available, prefill tiles beat the 128 x 256 streaming tiles of the mid-size batches
// earlier (4096 x 14336 layer, 5 of 8 experts hosted: 0.503 against 0.492 ms at 320 tokens, 0.537
// against 0.556 at 384, 0.564 against 0.629 at 512).
constexpr int kStreamMaxTokensSliced = 352;
static inline bool slicing_shape(const prism_layer_desc& d) {
  return d.dtype == PRISM_BF16 && d.ffn >= kSliceMinFfn && d.hidden >= 128;
}
static inline bool down_slicing_applies(const prism_layer_desc& d, int T) {
  return slicing_shape(d) && T > kStreamMaxTokensSliced;
}
static inline size_t slice_part_bytes(const prism_layer_desc& d, int T) {
  return down_slicing_applies(d, T) ? (size_t)256 * 256 * 256 * 4 : 0;
}

// Most contraction slices the down projection of a batch of T tokens may be split into.
static inline int max_splits(const prism_layer_desc& d, int T) {
  return (long long)T * (d.top_k + d.n_shared) <= kManySplitsRows ? kDecodeSplits : kStreamSplits;
}

static inline Workspace carve(const prism_layer_desc& d, int T, void* base) {
  Workspace w;
  const size_t A = (size_t)T * d.top_k;
  const size_t rows = A + (size_t)d.n_shared * T;
  const size_t es = elem_size(d.dtype);
  const int n_chunks = ceil_div((int)(A > 0 ? A : 1), kDispatchChunk);
  char* p = (char*)base;
  size_t off = 0;
  auto take = [&](size_t bytes) { char* q = p ? p + off : nullptr; off += align_up(bytes ? bytes : 1, 256); return (void*)q; };
  w.local_src = (int32_t*)take(A * 4);
  w.local_offsets = (int32_t*)take((size_t)(d.n_experts + 1) * 4);
  w.inv = (int32_t*)take(A * 4);
  w.block_hist = (int32_t*)take((size_t)n_chunks * d.n_experts * 4);
  w.tiles = (int32_t*)take(2 * tile_table_ints(d, T) * 4);
  w.h = take(rows * d.ffn * es);
  w.y = take(rows * d.hidden * es);
  // The regions of the small-batch paths are reserved for every T (sized for min(T, limit of
  // the path) tokens), so that the total never shrinks as T grows: a workspace sized for
  // max_tokens serves every smaller batch.
  const size_t t_dec = (size_t)(T < kDecodeMaxTokens ? T : kDecodeMaxTokens);
  const size_t t_str = (size_t)(T < kStreamMaxTokens ? T : kStreamMaxTokens);
  const size_t rows_str = t_str * (size_t)(d.top_k + d.n_shared);
  const bool bf16 = d.dtype == PRISM_BF16;
  // up to kManySplitsRows rows the down projection may be split into kDecodeSplits slices,
  // beyond into kStreamSplits: the larger of the two needs (max_splits)
  const size_t planes_rows = std::max((size_t)kDecodeSplits * std::min(rows_str, (size_t)kManySplitsRows),
                                      (size_t)kStreamSplits * rows_str);
  w.part = (float*)take(bf16 ? planes_rows * d.hidden * 4 : 0);
  w.slice_part = (float*)take(slice_part_bytes(d, T));
  w.route_part = (double*)take(bf16 ? (size_t)ceil_div((int)t_dec, kRouteTokTile) * kRouteMaxHSplit *
                                          route_col_tiles(d.n_experts) * 64 * 4 * 8 : 0);
  w.total = off;
  return w;
}

// ---------------------------------------------------------------------------
// Validation and launch helpers.
// ---------------------------------------------------------------------------
prism_status validate_desc(const prism_layer_desc* d, int32_t T, bool need_ffn_shapes);

#define PRISM_RETURN_IF(cond, code) do { if (cond) return (code); } while (0)
// A launch reports its failure through the thread's last-error slot only, and that slot also
// keeps whatever an earlier, unrelated HIP call of this thread left there.  Every entry point
// of the ABI therefore empties the slot first (PRISM_ENTER), so that PRISM_CHECK_LAUNCH sees
// the errors of this call's launches alone.
#define PRISM_ENTER() do { (void)hipGetLastError(); } while (0)
#define PRISM_CHECK_LAUNCH() do { if (hipGetLastError() != hipSuccess) return PRISM_ERR_LAUNCH; } while (0)

// Raises a kernel's dynamic-LDS limit once per device (bit d of `done`: raised on device d);
// an attempt that fails is repeated by the next call instead of being remembered.
struct LdsLimitOnce {
  std::atomic<uint32_t> done{0};
};
static inline bool raise_lds_limit(LdsLimitOnce& once, const void* kernel, int bytes) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return false;
  const uint32_t bit = 1u << (dev & 31);
  if (once.done.load(std::memory_order_acquire) & bit) return true;
  if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess) {
    (void)hipGetLastError();
    return false;
  }
  once.done.fetch_or(bit, std::memory_order_release);
  return true;
}
#define PRISM_TRY(expr) do { prism_status s__ = (expr); if (s__ != PRISM_OK) return s__; } while (0)

// ---------------------------------------------------------------------------
// Stage entry points used by the public API (all enqueue only).
// ---------------------------------------------------------------------------
prism_status launch_route(const prism_layer_desc& d, const void* x, const void* w_router,
                          const float* bias, int T, float* logits, int32_t* topk_idx,
                          float* topk_gate, int32_t* counts, int64_t* counts_accum,
                          hipStream_t st);

// counts NULL: no activation counts from the router (launch_dispatch can supply them).
// inv, counts, counts_accum of launch_dispatch may be NULL.  tiles given (bf16 layers): the
// launch that places the assignments may also build the two GEMM schedules of
// launch_expert_ffn there; *schedules_built says whether it did.
prism_status launch_dispatch(const prism_layer_desc& d, const int32_t* topk_idx,
                             const uint8_t* mask, int T, int32_t* local_src,
                             int32_t* local_offsets, int32_t* remote_src, int32_t* remote_offsets,
                             int32_t* n_local_remote, int64_t* remote_bytes, int32_t* inv,
                             int32_t* block_hist, int32_t* counts, int64_t* counts_accum,
                             hipStream_t st, int32_t* tiles = nullptr,
                             bool* schedules_built = nullptr);

// schedules_built: the two schedules in tiles already exist (decode front end).
// slice_part: scratch for a cut last round of the down projection (slice_part_bytes).
// deferred_splits NULL: y holds the finished expert outputs.  Otherwise the paths that split the
// down projection's contraction leave it as fp32 slices in part, y unwritten, for launch_combine
// to sum, and *deferred_splits points at their number in device memory (the schedule builder
// chose it); *deferred_splits == NULL means y is finished.
prism_status launch_expert_ffn(const prism_layer_desc& d, const void* x,
                               const prism_expert_weights& w, const int32_t* local_src,
                               const int32_t* local_offsets, int T, void* y, void* h,
                               int32_t* tiles, float* part, float* slice_part, hipStream_t st,
                               void* const* stage_events, const int32_t** deferred_splits,
                               bool schedules_built = false);

// True when launch_decode_front_end serves this layer shape and batch.
bool decode_front_end_applies(const prism_layer_desc& d, int T);

// Decode batches: router, placement split and both GEMM schedules in two launches.
// Outputs as launch_route + launch_dispatch (+ the schedules in tiles); route_part is
// scratch.  stage_events: ROUTE brackets the first launch, DISPATCH the second.
prism_status launch_decode_front_end(const prism_layer_desc& d, const void* x, const void* w_router,
                                     const float* bias, const uint8_t* mask, int T,
                                     int32_t* topk_idx, float* topk_gate, int32_t* counts,
                                     int64_t* counts_accum, int32_t* local_src,
                                     int32_t* local_offsets, int32_t* remote_src,
                                     int32_t* remote_offsets, int32_t* n_local_remote,
                                     int64_t* remote_bytes, int32_t* inv, double* route_part,
                                     int32_t* tiles, hipStream_t st, void* const* stage_events);

// What whoever builds the schedules of launch_expert_ffn's two grouped GEMMs for a bf16 batch of
// T tokens needs to know about them.
struct FfnShapes {
  int bm1, nt1, bm2, nt2;   // row tile and number of column tiles of the gate/up and of the down GEMM
  bool interleave;          // the items are dealt to the XCDs one by one (batches that stream the weights)
  int slice_kt2;            // k-tiles of the down projection's contraction if its last round may be cut
                            // along it; else 0
  // Down projection whose items are split along the contraction by a count the schedule builder
  // chooses (schedule.h, "Splits"); split_kt2 == 0: not split.
  int split_kt2;            // k-tiles of the contraction
  int split_min_kt2;        // fewest k-tiles of a split
  int split_wgs2;           // workgroups per XCD of the launch
  float split_round_kt2;    // fixed cost of a round of items, in k-tiles of one workgroup
  float split_row_kt2;      // cost of one more fp32 copy of a row, in k-tiles of one workgroup
};
FfnShapes ffn_schedule_shapes(const prism_layer_desc& d, int T);

// Records stage_events[2 * stage + end] on st when tracing is on and the pair is set.
static inline void trace(void* const* ev, int stage, int end, hipStream_t st) {
  if (ev != nullptr && ev[2 * stage] != nullptr && ev[2 * stage + 1] != nullptr)
    (void)hipEventRecord((hipEvent_t)ev[2 * stage + end], st);
}

prism_status launch_fill_i32(int32_t* p, int n, int32_t v, hipStream_t st);

// Builds inv from local_src/local_offsets (fill -1, then scatter).
prism_status launch_build_inverse(const prism_layer_desc& d, const int32_t* local_src,
                                  const int32_t* local_offsets, int T, int32_t* inv,
                                  hipStream_t st);

// add_to_out: the gate-weighted rows are added to what out holds (no shared rows, no slices).
// n_splits (device memory) not NULL: expert outputs are taken from *n_splits fp32 slices in part
// (bf16 layers only), each element summed over the slices in slice order and rounded to bf16 as
// the finished y would hold it.
prism_status launch_combine(const prism_layer_desc& d, const void* y, const int32_t* inv,
                            const float* topk_gate, int T, void* out, hipStream_t st,
                            const float* part = nullptr, const int32_t* n_splits = nullptr,
                            bool add_to_out = false);

// Row-major bf16 [rows, cols] -> 16 x 32 tiles (rows a multiple of 16, cols of 32).
prism_status launch_pack_weights(const void* src, int rows, int cols, void* dst, hipStream_t st);

// packed[r] = x[src[r] / k] for the rows r < offsets[E] of an assignment list.
prism_status launch_pack_rows(const prism_layer_desc& d, const void* x, const int32_t* src,
                              const int32_t* offsets, int T, void* packed, hipStream_t st);

// ---------------------------------------------------------------------------
// Device helpers.
// ---------------------------------------------------------------------------
// Workgroup barrier for data handed over in LDS only: waits for this wavefront's LDS
// traffic but, unlike __syncthreads(), not for its outstanding global loads and stores.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// Cross-lane moves inside the vector ALU (data-parallel primitives: no trip through the LDS
// crossbar, which a __shfl costs).  The single-workgroup kernels on the critical path of a
// decode layer are chains of short dependent steps, and their reductions and scans are a large
// part of those chains.
//   row_xor<OFF>(v): the value of lane (lane ^ OFF), OFF in {1, 2, 4, 8} (lanes of one
//   16-lane row exchange: quad permutes for 1 and 2, a shift left / right by 4 chosen per
//   bank of 4 lanes, a rotation by 8).
//   wave_inclusive_scan(v): sum of v over lanes 0..lane of the wavefront.
template <int CTRL, int ROW_MASK = 0xF, int BANK_MASK = 0xF>
__device__ __forceinline__ int dpp_move(int old, int src) {
  return __builtin_amdgcn_update_dpp(old, src, CTRL, ROW_MASK, BANK_MASK, false);
}
template <int OFF> __device__ __forceinline__ int row_xor(int v) {
  static_assert(OFF == 1 || OFF == 2 || OFF == 4 || OFF == 8, "inside a row of 16 lanes");
  if constexpr (OFF == 1) return dpp_move<0xB1>(v, v);                 // quad_perm [1,0,3,2]
  else if constexpr (OFF == 2) return dpp_move<0x4E>(v, v);            // quad_perm [2,3,0,1]
  else if constexpr (OFF == 4)                                         // banks 0, 2: lane + 4; banks 1, 3: lane - 4
    return dpp_move<0x114, 0xF, 0xA>(dpp_move<0x104, 0xF, 0x5>(v, v), v);
  else return dpp_move<0x128>(v, v);                                   // row_ror:8
}
template <int OFF> __device__ __forceinline__ float row_xor(float v) {
  return __int_as_float(row_xor<OFF>(__float_as_int(v)));
}
template <int OFF> __device__ __forceinline__ double row_xor(double v) {
  const long long b = __double_as_longlong(v);
  const int lo = row_xor<OFF>((int)(unsigned)b), hi = row_xor<OFF>((int)(unsigned)((unsigned long long)b >> 32));
  return __longlong_as_double((long long)(((unsigned long long)(unsigned)hi << 32) | (unsigned)lo));
}
__device__ __forceinline__ int wave_inclusive_scan(int v) {
  v += dpp_move<0x111>(0, v);          // row_shr:1 (lanes without a source add 0)
  v += dpp_move<0x112>(0, v);          // row_shr:2
  v += dpp_move<0x114>(0, v);          // row_shr:4
  v += dpp_move<0x118>(0, v);          // row_shr:8 -> inclusive scan of every row of 16
  v += dpp_move<0x142, 0xA>(0, v);     // row_bcast:15 -> rows 1 and 3 add the total of rows 0 and 2
  v += dpp_move<0x143, 0xC>(0, v);     // row_bcast:31 -> rows 2 and 3 add the total of rows 0..1
  return v;
}

// Direct global -> LDS loads (buffer_load_dwordx4 ... lds): raw buffer resources whose size
// makes a lane offset at or above it read zeros (the scalar offset of a load is not part of
// that check), and the vector-memory counter the loads are awaited with.
typedef __attribute__((address_space(3))) void* lds_ptr_t;
constexpr int kBufferFlags = 0x00020000;        // raw buffer, 32-bit data format (gfx9 family)
constexpr int kNonTemporal = 2;                 // cache-policy operand of a buffer load: the "nt" bit (data read once)
constexpr uint32_t kOutOfRange = 0xFFFFFF00u;   // above every operand size (those stay below 0xFFFF0000)
template <int N> __device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) {
  return __uint_as_float((uint32_t)b << 16);
}
__device__ __forceinline__ float bf16_lo(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) { return __uint_as_float(packed & 0xffff0000u); }

}  // namespace prism
#endif  // PRISM_INTERNAL_H_
