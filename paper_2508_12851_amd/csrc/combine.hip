// Gate-weighted aggregation of the local expert outputs (paper Sec. III-A: the
// results of the experts are aggregated before the next block).  Remote slots
// contribute nothing here; their rows arrive later in the real system.
//
//   out[t] = sum_{j local, ascending} gate[t,j] * y[inv[t*k+j]] + sum_s y[A + s*T + t]
//
// fp32 accumulation, one rounding to the layer dtype.  HBM-bound: every thread
// moves 16 bytes per y row it touches.
//
// Decode batches leave the down projection as fp32 contraction slices; the
// fused layer then reads y from them: every element is the slice sum in slice
// order, rounded to bf16 exactly as the finished y row would have stored it.
#include "prism_internal.h"

namespace prism {
namespace {

__global__ void scatter_inverse_kernel(const int32_t* __restrict__ local_src,
                                       const int32_t* __restrict__ local_offsets, int E, int A,
                                       int32_t* __restrict__ inv) {
  const int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r < A && r < local_offsets[E]) inv[local_src[r]] = r;
}

template <typename T> struct Vec;
template <> struct Vec<float> {
  static constexpr int N = 4;
  typedef f32x4 raw;
  __device__ static void load(const float* p, float (&v)[N]) {
    const f32x4 a = *reinterpret_cast<const f32x4*>(p);
    v[0] = a[0]; v[1] = a[1]; v[2] = a[2]; v[3] = a[3];
  }
  __device__ static void store(float* p, const float (&v)[N]) {
    *reinterpret_cast<f32x4*>(p) = f32x4{v[0], v[1], v[2], v[3]};
  }
};
template <> struct Vec<uint16_t> {
  static constexpr int N = 8;
  typedef uint4 raw;
  // Non-temporal: every expert output row is read exactly once, by this kernel (combine of the
  // 60-expert layer with 4 shared experts: 57.8 -> 51.3 us for 245 MB of rows).
  __device__ static void load(const uint16_t* p, float (&v)[N]) {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 a = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
    v[0] = bf16_lo(a.x); v[1] = bf16_hi(a.x); v[2] = bf16_lo(a.y); v[3] = bf16_hi(a.y);
    v[4] = bf16_lo(a.z); v[5] = bf16_hi(a.z); v[6] = bf16_lo(a.w); v[7] = bf16_hi(a.w);
  }
  __device__ static void store(uint16_t* p, const float (&v)[N]) {
    bf16x8 o;
#pragma unroll
    for (int i = 0; i < N; ++i) o[i] = (bf16_t)v[i];
    *reinterpret_cast<bf16x8*>(p) = o;
  }
};

// ADD: the sum starts from the value out already holds (returned remote rows are added to
// the local partial sum) instead of zero.
template <typename TIO, bool ADD>
__global__ __launch_bounds__(256) void combine_kernel(const TIO* __restrict__ y,
                                                      const int32_t* __restrict__ inv,
                                                      const float* __restrict__ gate, int T, int H,
                                                      int k, int S, TIO* out) {
  constexpr int N = Vec<TIO>::N;
  const int vec_per_row = H / N;
  const long long gid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= (long long)T * vec_per_row) return;
  const int t = (int)(gid / vec_per_row);
  const int col = (int)(gid - (long long)t * vec_per_row) * N;
  float acc[N];
  if (ADD) {
    Vec<TIO>::load(out + (size_t)t * H + col, acc);
  } else {
#pragma unroll
    for (int i = 0; i < N; ++i) acc[i] = 0.f;
  }
  for (int j = 0; j < k; ++j) {
    const int row = inv[t * k + j];
    if (row >= 0) {
      const float gt = gate[t * k + j];
      float v[N];
      Vec<TIO>::load(y + (size_t)row * H + col, v);
#pragma unroll
      for (int i = 0; i < N; ++i) acc[i] = fmaf(gt, v[i], acc[i]);
    }
  }
  const size_t A = (size_t)T * k;
  for (int s = 0; s < S; ++s) {
    float v[N];
    Vec<TIO>::load(y + (A + (size_t)s * T + t) * H + col, v);
#pragma unroll
    for (int i = 0; i < N; ++i) acc[i] += v[i];
  }
  Vec<TIO>::store(out + (size_t)t * H + col, acc);
}

// Shipped activation rows of the remote list: packed[r] = x[src[r] / k] for r < offsets[E].
template <typename TIO>
__global__ __launch_bounds__(256) void pack_rows_kernel(const TIO* __restrict__ x,
                                                        const int32_t* __restrict__ src,
                                                        const int32_t* __restrict__ offsets, int E,
                                                        int k, int H, int max_rows,
                                                        TIO* __restrict__ packed) {
  constexpr int N = Vec<TIO>::N;
  const int vec_per_row = H / N;
  const long long gid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= (long long)max_rows * vec_per_row) return;
  const int r = (int)(gid / vec_per_row);
  if (r >= offsets[E]) return;
  const int col = (int)(gid - (long long)r * vec_per_row) * N;
  const int t = src[r] / k;
  typedef typename Vec<TIO>::raw raw_t;
  *reinterpret_cast<raw_t*>(packed + (size_t)r * H + col) =
      *reinterpret_cast<const raw_t*>(x + (size_t)t * H + col);
}

// One 16-byte chunk (8 bf16) per thread from the row-major matrix to its place in the
// layout of 16 x 32 tiles.
__global__ __launch_bounds__(256) void pack_weights_kernel(const uint4* __restrict__ src, int rows,
                                                           int cols, uint4* __restrict__ dst) {
  const int chunks_per_row = cols / 8;
  const long long gid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= (long long)rows * chunks_per_row) return;
  const unsigned r = (unsigned)(gid / chunks_per_row);
  const unsigned c = (unsigned)(gid - (long long)r * chunks_per_row) * 8;   // first column
  const size_t byte = ((size_t)(r >> 4) * (cols >> 5) + (c >> 5)) * 1024 + (r & 15u) * 64 + (c & 31u) * 2;
  dst[byte / 16] = src[gid];
}

// Same aggregation with y taken from the contraction slices (bf16 layers).  Four
// columns per thread: a decode batch has few tokens, and the narrower vectors put
// twice as many workgroups on the machine.  The kernel is a chain of dependent
// memory round trips (slot table, then rows), so the slot table of a token is read
// in one go and the slice loads of two rows are issued together.
struct SliceRow {
  f32x4 v[kDecodeSplits];
};
__device__ __forceinline__ void load_slices(const float* __restrict__ part, int n_splits,
                                            size_t rows, int H, size_t row, int col, bool on,
                                            SliceRow& r) {
#pragma unroll
  for (int s = 0; s < kDecodeSplits; ++s)
    if (on && s < n_splits)
      r.v[s] = *reinterpret_cast<const f32x4*>(part + ((size_t)s * rows + row) * H + col);
}
// Slice sum in slice order, rounded to bf16: what the finished y row would hold.
__device__ __forceinline__ f32x4 sum_slices(const SliceRow& r, int n_splits) {
  f32x4 sum = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int s = 0; s < kDecodeSplits; ++s)
    if (s < n_splits) sum += r.v[s];
#pragma unroll
  for (int i = 0; i < 4; ++i) sum[i] = (float)(bf16_t)sum[i];
  return sum;
}

__global__ __launch_bounds__(256) void combine_slices_kernel(const float* __restrict__ part,
                                                             const int32_t* __restrict__ n_splits_ptr,
                                                             const int32_t* __restrict__ inv,
                                                             const float* __restrict__ gate, int T,
                                                             int H, int k, int S,
                                                             uint16_t* __restrict__ out) {
  const int vec_per_row = H / 4;
  const long long gid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= (long long)T * vec_per_row) return;
  const int t = (int)(gid / vec_per_row);
  const int col = (int)(gid - (long long)t * vec_per_row) * 4;
  const size_t A = (size_t)T * k;
  const size_t rows = A + (size_t)S * T;
  const int n_splits = min(*n_splits_ptr, kDecodeSplits);   // what the schedule builder chose
  int row_of[PRISM_MAX_TOPK];
  float gate_of[PRISM_MAX_TOPK];
#pragma unroll
  for (int j = 0; j < PRISM_MAX_TOPK; ++j) {
    row_of[j] = j < k ? inv[t * k + j] : -1;
    gate_of[j] = j < k ? gate[t * k + j] : 0.f;
  }
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int j = 0; j < PRISM_MAX_TOPK; j += 2) {
    if (j >= k) break;
    SliceRow r0, r1;
    const bool on0 = row_of[j] >= 0, on1 = row_of[j + 1] >= 0;
    load_slices(part, n_splits, rows, H, (size_t)(on0 ? row_of[j] : 0), col, on0, r0);
    load_slices(part, n_splits, rows, H, (size_t)(on1 ? row_of[j + 1] : 0), col, on1, r1);
    if (on0) {
      const f32x4 v = sum_slices(r0, n_splits);
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[i] = fmaf(gate_of[j], v[i], acc[i]);
    }
    if (on1) {
      const f32x4 v = sum_slices(r1, n_splits);
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[i] = fmaf(gate_of[j + 1], v[i], acc[i]);
    }
  }
  for (int s = 0; s < S; ++s) {
    SliceRow r;
    load_slices(part, n_splits, rows, H, A + (size_t)s * T + t, col, true, r);
    acc += sum_slices(r, n_splits);
  }
  bf16x4 o;
#pragma unroll
  for (int i = 0; i < 4; ++i) o[i] = (bf16_t)acc[i];
  *reinterpret_cast<bf16x4*>(out + (size_t)t * H + col) = o;
}

}  // namespace

prism_status launch_build_inverse(const prism_layer_desc& d, const int32_t* local_src,
                                  const int32_t* local_offsets, int T, int32_t* inv,
                                  hipStream_t st) {
  const int A = T * d.top_k;
  if (A == 0) return PRISM_OK;
  PRISM_TRY(launch_fill_i32(inv, A, -1, st));
  hipLaunchKernelGGL(scatter_inverse_kernel, dim3(ceil_div(A, 256)), dim3(256), 0, st, local_src,
                     local_offsets, d.n_experts, A, inv);
  PRISM_CHECK_LAUNCH();
  return PRISM_OK;
}

prism_status launch_pack_weights(const void* src, int rows, int cols, void* dst, hipStream_t st) {
  const long long threads = (long long)rows * (cols / 8);
  hipLaunchKernelGGL(pack_weights_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st,
                     (const uint4*)src, rows, cols, (uint4*)dst);
  PRISM_CHECK_LAUNCH();
  return PRISM_OK;
}

prism_status launch_pack_rows(const prism_layer_desc& d, const void* x, const int32_t* src,
                              const int32_t* offsets, int T, void* packed, hipStream_t st) {
  const int A = T * d.top_k;
  if (A == 0) return PRISM_OK;
  const int n = d.dtype == PRISM_F32 ? 4 : 8;
  const long long threads = (long long)A * (d.hidden / n);
  const unsigned blocks = (unsigned)((threads + 255) / 256);
  if (d.dtype == PRISM_F32)
    hipLaunchKernelGGL(pack_rows_kernel<float>, dim3(blocks), dim3(256), 0, st, (const float*)x, src,
                       offsets, d.n_experts, d.top_k, d.hidden, A, (float*)packed);
  else
    hipLaunchKernelGGL(pack_rows_kernel<uint16_t>, dim3(blocks), dim3(256), 0, st,
                       (const uint16_t*)x, src, offsets, d.n_experts, d.top_k, d.hidden, A,
                       (uint16_t*)packed);
  PRISM_CHECK_LAUNCH();
  return PRISM_OK;
}

prism_status launch_combine(const prism_layer_desc& d, const void* y, const int32_t* inv,
                            const float* topk_gate, int T, void* out, hipStream_t st,
                            const float* part, const int32_t* n_splits, bool add_to_out) {
  if (T == 0) return PRISM_OK;
  if (add_to_out) {   // returned remote rows: no shared experts, no slices
    if (n_splits != nullptr) return PRISM_ERR_INVALID_ARG;
    const int nv = d.dtype == PRISM_F32 ? 4 : 8;
    const long long th = (long long)T * (d.hidden / nv);
    const unsigned bl = (unsigned)((th + 255) / 256);
    if (d.dtype == PRISM_F32)
      hipLaunchKernelGGL((combine_kernel<float, true>), dim3(bl), dim3(256), 0, st, (const float*)y,
                         inv, topk_gate, T, d.hidden, d.top_k, 0, (float*)out);
    else
      hipLaunchKernelGGL((combine_kernel<uint16_t, true>), dim3(bl), dim3(256), 0, st,
                         (const uint16_t*)y, inv, topk_gate, T, d.hidden, d.top_k, 0, (uint16_t*)out);
    PRISM_CHECK_LAUNCH();
    return PRISM_OK;
  }
  if (n_splits != nullptr && (d.dtype != PRISM_BF16 || part == nullptr)) return PRISM_ERR_INVALID_ARG;
  if (n_splits != nullptr) {
    const long long threads = (long long)T * (d.hidden / 4);
    hipLaunchKernelGGL(combine_slices_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0,
                       st, part, n_splits, inv, topk_gate, T, d.hidden, d.top_k, d.n_shared,
                       (uint16_t*)out);
    PRISM_CHECK_LAUNCH();
    return PRISM_OK;
  }
  const int n = d.dtype == PRISM_F32 ? 4 : 8;
  const long long threads = (long long)T * (d.hidden / n);
  const unsigned blocks = (unsigned)((threads + 255) / 256);
  if (d.dtype == PRISM_F32)
    hipLaunchKernelGGL((combine_kernel<float, false>), dim3(blocks), dim3(256), 0, st, (const float*)y, inv,
                       topk_gate, T, d.hidden, d.top_k, d.n_shared, (float*)out);
  else
    hipLaunchKernelGGL((combine_kernel<uint16_t, false>), dim3(blocks), dim3(256), 0, st, (const uint16_t*)y,
                       inv, topk_gate, T, d.hidden, d.top_k, d.n_shared, (uint16_t*)out);
  PRISM_CHECK_LAUNCH();
  return PRISM_OK;
}

}  // namespace prism
