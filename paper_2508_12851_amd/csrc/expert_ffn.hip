// Grouped SwiGLU expert FFN over the locally hosted and the shared experts
// (paper Sec. III-A: "experts resident on the server compute on routed tokens").
//
//   GEMM1  h[r, f] = silu( x[tok(r)] . W_gate^e[f] ) * ( x[tok(r)] . W_up^e[f] )
//   GEMM2  y[r, n] = h[r] . W_down^e[n]
//
// Both are "NT" contractions (activation rows and weight rows are contiguous
// along the contraction index), grouped by expert: a device-built tile table
// lists (expert, first row, row count) for every row tile, so the host never
// needs the routing-dependent segment sizes.
//
// bf16 path: v_mfma_f32_32x32x16_bf16, 4 wavefronts per workgroup, operand
// tiles of 64 contraction elements staged in LDS (double buffered, 16-byte
// chunks XOR-swizzled by row so the 16-byte MFMA operand reads spread over all
// banks).  GEMM1 loads the gate rows and the up rows of the same f range into
// one tile, so silu(gate)*up is a register epilogue and only h is written.
// Activation rows of GEMM1 are gathered through local_src (no permuted copy of
// x is materialised).
#include "prism_internal.h"

namespace prism {
namespace {

// ---------------------------------------------------------------------------
// Tile table: tiles[0] = number of row tiles; entry i at tiles + 4 + 4 i:
//   [0] group id g (g < E: routed expert g; else shared expert g - E)
//   [1] first row of the tile in h / y row space
//   [2] rows in the tile (1..BM)
//   [3] first token of the tile for shared experts, -1 for routed ones
// ---------------------------------------------------------------------------
constexpr int kMaxGroups = PRISM_MAX_EXPERTS + PRISM_MAX_SHARED;

__global__ __launch_bounds__(512) void build_tiles_kernel(const int32_t* __restrict__ local_offsets,
                                                          int E, int S, int T, int A_total, int BM,
                                                          int32_t* __restrict__ tiles) {
  __shared__ int s_start[kMaxGroups + 1];
  const int g = threadIdx.x;
  int rows = 0, row_start = 0;
  if (g < E) {
    row_start = local_offsets[g];
    rows = local_offsets[g + 1] - row_start;
  } else if (g < E + S) {
    row_start = A_total + (g - E) * T;
    rows = T;
  }
  const int nt = (rows + BM - 1) / BM;
  if (g < kMaxGroups) s_start[g] = nt;
  __syncthreads();
  if (threadIdx.x == 0) {
    int run = 0;
    for (int i = 0; i < E + S; ++i) {
      const int c = s_start[i];
      s_start[i] = run;
      run += c;
    }
    tiles[0] = run;
  }
  __syncthreads();
  if (g < E + S) {
    int32_t* out = tiles + 4 + 4 * s_start[g];
    for (int i = 0; i < nt; ++i) {
      out[4 * i + 0] = g;
      out[4 * i + 1] = row_start + i * BM;
      out[4 * i + 2] = min(BM, rows - i * BM);
      out[4 * i + 3] = g < E ? -1 : i * BM;
    }
  }
}

// ---------------------------------------------------------------------------
// bf16 grouped GEMM on the matrix cores
// ---------------------------------------------------------------------------
struct GemmArgs {
  const uint16_t* A;        // GATED: x [T, K]; else h [rows, K]
  const void* const* B0;    // routed: W_gate (GATED) or W_down tables
  const void* const* B1;    // routed: W_up table (GATED only)
  const void* const* SB0;   // shared experts, same roles
  const void* const* SB1;
  uint16_t* C;              // GATED: h [rows, N]; else y [rows, N]
  const int32_t* tiles;
  const int32_t* local_src;
  int K;                    // contraction length (H for GEMM1, F for GEMM2)
  int N;                    // output columns (F for GEMM1, H for GEMM2)
  int top_k;
  int E;
  int n_ntiles;
};

constexpr int BK = 64;                       // contraction elements per LDS tile
constexpr int kRowBytes = BK * 2;            // 128 bytes = 8 chunks of 16 bytes
constexpr int kGemmThreads = 256;

__device__ __forceinline__ float silu(float z) { return z / (1.0f + __expf(-z)); }

// BM x BN output tile per workgroup; BN counts weight rows in the tile (for
// GATED: BN/2 gate rows and BN/2 up rows).  Wavefronts form a WGM x WGN grid.
template <int BM, int BN, int WGM, int WGN, bool GATED>
__global__ __launch_bounds__(kGemmThreads) void grouped_gemm_kernel(const GemmArgs p) {
  static_assert(WGM * WGN == 4, "four wavefronts per workgroup");
  constexpr int WM = BM / WGM, WN = BN / WGN;
  constexpr int MI = WM / 32, NJ = WN / 32;
  static_assert(MI >= 1 && NJ >= 1 && (!GATED || NJ % 2 == 0), "tile shape");
  constexpr int A_CH = BM * 8 / kGemmThreads;     // 16-byte chunks per thread per tile
  constexpr int B_CH = BN * 8 / kGemmThreads;
  static_assert(A_CH >= 1 && B_CH >= 1, "tile too small for 256 threads");
  constexpr int kStageBytes = (BM + BN) * kRowBytes;

  extern __shared__ __align__(16) uint8_t smem[];

  const int n_mtiles = p.tiles[0];
  if (n_mtiles <= 0) return;
  const int nt = blockIdx.x / n_mtiles;
  if (nt >= p.n_ntiles) return;
  const int mt = blockIdx.x - nt * n_mtiles;
  const int4 tile = *reinterpret_cast<const int4*>(p.tiles + 4 + 4 * mt);
  const int g = tile.x, row_start = tile.y, row_count = tile.z, tok_base = tile.w;

  const uint16_t* b0 = (const uint16_t*)(g < p.E ? p.B0[g] : p.SB0[g - p.E]);
  const uint16_t* b1 = nullptr;
  if (GATED) b1 = (const uint16_t*)(g < p.E ? p.B1[g] : p.SB1[g - p.E]);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  const int r32 = lane & 31, q = lane >> 5;

  // ---- global -> LDS assignment: thread owns chunk c of rows tid/8 + 32 i -----
  const int c = tid & 7;
  const int lrow = tid >> 3;
  const int pc = c ^ (lrow & 7);                 // swizzled chunk slot (row + 32 i keeps row & 7)
  const uint16_t* a_ptr[A_CH];
#pragma unroll
  for (int i = 0; i < A_CH; ++i) {
    const int rr = min(lrow + 32 * i, row_count - 1);
    size_t src;
    if (GATED) src = tok_base >= 0 ? (size_t)(tok_base + rr) : (size_t)(p.local_src[row_start + rr] / p.top_k);
    else src = (size_t)(row_start + rr);
    a_ptr[i] = p.A + src * p.K + c * 8;
  }
  const uint16_t* b_ptr[B_CH];
#pragma unroll
  for (int i = 0; i < B_CH; ++i) {
    const int rr = lrow + 32 * i;
    if (GATED) {
      const int w = rr / WN, within = rr % WN;
      const bool up = within >= WN / 2;
      const int f = min(nt * (BN / 2) + w * (WN / 2) + (within % (WN / 2)), p.N - 1);
      b_ptr[i] = (up ? b1 : b0) + (size_t)f * p.K + c * 8;
    } else {
      const int n = min(nt * BN + rr, p.N - 1);
      b_ptr[i] = b0 + (size_t)n * p.K + c * 8;
    }
  }
  const int a_lds = lrow * kRowBytes + pc * 16;              // + i * 32 rows
  const int b_lds = BM * kRowBytes + lrow * kRowBytes + pc * 16;

  uint4 a_reg[A_CH], b_reg[B_CH];
  auto load_global = [&](int kt) {
#pragma unroll
    for (int i = 0; i < A_CH; ++i) a_reg[i] = *reinterpret_cast<const uint4*>(a_ptr[i] + kt * BK);
#pragma unroll
    for (int i = 0; i < B_CH; ++i) b_reg[i] = *reinterpret_cast<const uint4*>(b_ptr[i] + kt * BK);
  };
  auto store_lds = [&](int stage) {
    uint8_t* base = smem + stage * kStageBytes;
#pragma unroll
    for (int i = 0; i < A_CH; ++i) *reinterpret_cast<uint4*>(base + a_lds + i * 32 * kRowBytes) = a_reg[i];
#pragma unroll
    for (int i = 0; i < B_CH; ++i) *reinterpret_cast<uint4*>(base + b_lds + i * 32 * kRowBytes) = b_reg[i];
  };

  f32x16 acc[MI][NJ];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const int KT = p.K / BK;
  load_global(0);
  store_lds(0);
  __syncthreads();

  // operand rows of this lane inside the LDS tile
  const int a_row0 = wm * WM + r32;                 // + 32 i
  const int b_row0 = BM + wn * WN + r32;            // + 32 j
  const int sw = r32 & 7;

  for (int kt = 0; kt < KT; ++kt) {
    if (kt + 1 < KT) load_global(kt + 1);
    const uint8_t* base = smem + (kt & 1) * kStageBytes;
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      const int slot = ((kk * 2 + q) ^ sw) * 16;
      bf16x8 af[MI], bfr[NJ];
#pragma unroll
      for (int i = 0; i < MI; ++i)
        af[i] = *reinterpret_cast<const bf16x8*>(base + (a_row0 + 32 * i) * kRowBytes + slot);
#pragma unroll
      for (int j = 0; j < NJ; ++j)
        bfr[j] = *reinterpret_cast<const bf16x8*>(base + (b_row0 + 32 * j) * kRowBytes + slot);
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < KT) store_lds((kt + 1) & 1);
    __syncthreads();
  }

  // ---- epilogue ---------------------------------------------------------------
  // Accumulator register v of lane (r32, q) is row 8 (v / 4) + 4 q + v % 4, column r32.
  if (GATED) {
    constexpr int NH = NJ / 2;
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int j = 0; j < NH; ++j) {
        const int f = nt * (BN / 2) + wn * (WN / 2) + j * 32 + r32;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = wm * WM + i * 32 + (v >> 2) * 8 + q * 4 + (v & 3);
          if (row < row_count && f < p.N) {
            const float hval = silu(acc[i][j][v]) * acc[i][j + NH][v];
            const bf16_t hb = (bf16_t)hval;
            p.C[(size_t)(row_start + row) * p.N + f] = *reinterpret_cast<const uint16_t*>(&hb);
          }
        }
      }
  } else {
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        const int n = nt * BN + wn * WN + j * 32 + r32;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = wm * WM + i * 32 + (v >> 2) * 8 + q * 4 + (v & 3);
          if (row < row_count && n < p.N) {
            const bf16_t yb = (bf16_t)acc[i][j][v];
            p.C[(size_t)(row_start + row) * p.N + n] = *reinterpret_cast<const uint16_t*>(&yb);
          }
        }
      }
  }
}

template <int BM, int BN, int WGM, int WGN, bool GATED>
prism_status launch_gemm(const GemmArgs& args, int max_mtiles, hipStream_t st) {
  constexpr int smem = 2 * (BM + BN) * kRowBytes;
  auto kernel = grouped_gemm_kernel<BM, BN, WGM, WGN, GATED>;
  static bool attr_set = false;
  if (!attr_set) {
    if (hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, smem) != hipSuccess)
      return PRISM_ERR_LAUNCH;
    attr_set = true;
  }
  const long long blocks = (long long)max_mtiles * args.n_ntiles;
  if (blocks <= 0) return PRISM_OK;
  if (blocks > 0x7fffffffLL) return PRISM_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(kGemmThreads), smem, st, args);
  PRISM_CHECK_LAUNCH();
  return PRISM_OK;
}

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

}  // namespace

prism_status launch_expert_ffn(const prism_layer_desc& d, const void* x,
                               const prism_expert_weights& w, const int32_t* local_src,
                               const int32_t* local_offsets, int T, void* y, void* h,
                               int32_t* tiles, hipStream_t st, void* const* stage_events) {
  if (T == 0) return PRISM_OK;
  const int A = T * d.top_k;
  const int rows = A + d.n_shared * T;
  if (d.dtype == PRISM_F32) {
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

  // bf16: tile tables for the two GEMMs, then the GEMMs.
  constexpr int BM = 128;
  int32_t* tiles1 = tiles;
  const int groups = d.n_experts + d.n_shared;
  const int max_mtiles = A / BM + d.n_experts + d.n_shared * ceil_div(T, BM);
  (void)groups;
  hipLaunchKernelGGL(build_tiles_kernel, dim3(1), dim3(512), 0, st, local_offsets, d.n_experts,
                     d.n_shared, T, A, BM, tiles1);
  PRISM_CHECK_LAUNCH();

  GemmArgs g1{};
  g1.A = (const uint16_t*)x;
  g1.B0 = w.w_gate; g1.B1 = w.w_up; g1.SB0 = w.shared_w_gate; g1.SB1 = w.shared_w_up;
  g1.C = (uint16_t*)h;
  g1.tiles = tiles1; g1.local_src = local_src;
  g1.K = d.hidden; g1.N = d.ffn; g1.top_k = d.top_k; g1.E = d.n_experts;
  g1.n_ntiles = ceil_div(d.ffn, 64);
  trace(stage_events, PRISM_STAGE_FFN_UP, 0, st);
  PRISM_TRY((launch_gemm<BM, 128, 2, 2, true>(g1, max_mtiles, st)));
  trace(stage_events, PRISM_STAGE_FFN_UP, 1, st);

  GemmArgs g2{};
  g2.A = (const uint16_t*)h;
  g2.B0 = w.w_down; g2.B1 = nullptr; g2.SB0 = w.shared_w_down; g2.SB1 = nullptr;
  g2.C = (uint16_t*)y;
  g2.tiles = tiles1; g2.local_src = local_src;
  g2.K = d.ffn; g2.N = d.hidden; g2.top_k = d.top_k; g2.E = d.n_experts;
  g2.n_ntiles = ceil_div(d.hidden, 128);
  trace(stage_events, PRISM_STAGE_FFN_DOWN, 0, st);
  PRISM_TRY((launch_gemm<BM, 128, 2, 2, false>(g2, max_mtiles, st)));
  trace(stage_events, PRISM_STAGE_FFN_DOWN, 1, st);
  return PRISM_OK;
}

}  // namespace prism
