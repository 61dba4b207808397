// Grouped "NT" GEMM on the bf16 matrix cores of gfx950, used for both halves of
// the SwiGLU expert FFN (paper Sec. III-A, local expert execution):
//
//   GATED   h[r, f] = silu( x[tok(r)] . W_gate^g[f] ) * ( x[tok(r)] . W_up^g[f] )
//   plain   y[r, n] = h[r] . W_down^g[n]
//
// Rows are grouped by expert g; a device-built schedule (tile table + work
// list) gives every workgroup its (row tile, column tile), so the host never
// needs the routing-dependent segment sizes.
//
// Kernel shape: BM x BN output tile per workgroup of 4 wavefronts (WGM x WGN),
// v_mfma_f32_32x32x16_bf16, operand tiles of 64 contraction elements staged in
// LDS in a ring of STAGES stages.  An LDS row holds BK contraction elements
// (128 or 64 bytes) as 16-byte chunks; chunk c of row r sits in slot
// c ^ key(r) (key = (r >> 1) & 7 for 128-byte rows, (r >> 2) & 3 for 64-byte
// rows), so the 16-byte operand reads of 16 consecutive rows hit 16 different
// slots of the 256-byte bank window.  Stages are filled by global_load_lds_dwordx4 (no
// VGPR staging): one instruction fills 1 KiB, and because each lane's LDS slot
// is fixed (lane * 16 bytes), the swizzle is applied to the global chunk a
// lane fetches instead.  Stage k is awaited with s_waitcnt vmcnt(n), n = the
// loads of the younger stages, then one s_barrier per stage orders the ring.
//
// Work order: the hardware hands consecutive workgroup ids to the 8 XCDs in
// turn, each with a private L2.  Workgroup b therefore takes column tile
// 8 j + (b % 8) of work item b / 8, and the work list walks, per expert, its
// row tiles fastest: the ~32 workgroups resident on one XCD share a few weight
// tiles and one expert's activation tiles, and every weight tile is fetched
// into exactly one L2.
#ifndef PRISM_GROUPED_GEMM_H_
#define PRISM_GROUPED_GEMM_H_

#include "prism_internal.h"


namespace prism {
namespace gg {

constexpr int kMaxGroups = PRISM_MAX_EXPERTS + PRISM_MAX_SHARED;
constexpr int kXcds = 8;

// Schedule memory (int32): [0] n_mtiles, [1] n_work, [2] sched offset (ints), [3] unused,
// then 4 ints per row tile:
//   [0] group id g (g < E: routed expert g; else shared expert g - E)
//   [1] first row of the tile in h / y row space
//   [2] rows in the tile (1..BM)
//   [3] first token of the tile for shared experts, -1 for routed ones
// then 2 ints per work item: (row tile index, column-tile octet j).
__global__ __launch_bounds__(512) void build_schedule_kernel(
    const int32_t* __restrict__ local_offsets, int E, int S, int T, int A_total, int BM, int nj8,
    int max_mtiles, int32_t* __restrict__ tiles) {
  __shared__ int s_start[kMaxGroups + 1];
  __shared__ int s_rows[kMaxGroups], s_row0[kMaxGroups];
  const int G = E + S;
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
  __syncthreads();
  if (threadIdx.x == 0) {
    int run = 0;
    for (int g = 0; g < G; ++g) {
      s_start[g] = run;
      run += (s_rows[g] + BM - 1) / BM;
    }
    s_start[G] = run;
    tiles[0] = run;
    tiles[1] = run * nj8;
    tiles[2] = 4 + 4 * max_mtiles;
  }
  __syncthreads();
  const int n_mtiles = s_start[G];
  auto group_of_tile = [&](int i) {   // largest g with s_start[g] <= i (skips empty groups)
    int lo = 0, hi = G;               // invariant: s_start[lo] <= i < s_start[hi]
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (s_start[mid] <= i) lo = mid; else hi = mid;
    }
    return lo;
  };
  for (int i = threadIdx.x; i < n_mtiles; i += blockDim.x) {
    const int g = group_of_tile(i);
    const int mi = i - s_start[g];
    int32_t* out = tiles + 4 + 4 * i;
    out[0] = g;
    out[1] = s_row0[g] + mi * BM;
    out[2] = min(BM, s_rows[g] - mi * BM);
    out[3] = g < E ? -1 : mi * BM;
  }
  int32_t* sched = tiles + 4 + 4 * max_mtiles;
  const int n_work = n_mtiles * nj8;
  for (int w = threadIdx.x; w < n_work; w += blockDim.x) {
    const int g = group_of_tile(w / nj8);          // work of group g starts at s_start[g] * nj8
    const int mg = s_start[g + 1] - s_start[g];
    const int local = w - s_start[g] * nj8;
    sched[2 * w + 0] = s_start[g] + local % mg;    // row tiles fastest
    sched[2 * w + 1] = local / mg;
  }
}

struct GemmArgs {
  const uint16_t* A;        // GATED: x [T, K]; else h [rows, K]
  const void* const* B0;    // routed: W_gate (GATED) or W_down tables
  const void* const* B1;    // routed: W_up table (GATED only)
  const void* const* SB0;   // shared experts, same roles
  const void* const* SB1;
  uint16_t* C;              // GATED: h [rows, N]; else y [rows, N]
  float* Cpart;             // SPLITK: [n_splits][c_rows][N] fp32 partial sums
  int c_rows;               // rows of one partial-sum slice
  const int32_t* tiles;
  const int32_t* local_src;
  uint32_t a_bytes;         // size of A in bytes (buffer range check), < 2^32
  uint32_t b_bytes;         // size of one weight matrix in bytes, < 2^32
  int K;                    // contraction length (H for GEMM1, F for GEMM2)
  int N;                    // output columns (F for GEMM1, H for GEMM2)
  int top_k;
  int E;
  int n_ntiles;
};

constexpr int kGemmThreads = 256;

typedef __attribute__((address_space(3))) void* lds_ptr_t;
constexpr int kBufferFlags = 0x00020000;   // raw buffer, 32-bit data format (gfx9 family)

__device__ __forceinline__ float silu(float z) { return z / (1.0f + __expf(-z)); }

// LDS slot swizzle.  The LDS serves a 16-byte-per-lane read 16 lanes (256 bytes,
// 64 banks) per cycle, so 16 consecutive rows read at the same logical chunk
// must land in 16 different 16-byte slots of the 256-byte bank window: rows
// that share (row * row_bytes) mod 256 get different keys.
template <int BK> __device__ __forceinline__ int swizzle_key(int row) {
  return BK == 64 ? ((row >> 1) & 7) : ((row >> 2) & 3);
}

template <int N> __device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// BM x BN output tile per workgroup; BN counts weight rows in the tile (for
// GATED: BN/2 gate rows and BN/2 up rows).  Wavefronts form a WGM x WGN grid.
// BK contraction elements per LDS stage (32 or 64), STAGES stages in flight.
// SPLITK: blockIdx.y selects a slice of the contraction; the tile is written as
// fp32 partial sums to p.Cpart[slice][row][col] (plain GEMM only).
template <int BM, int BN, int WGM, int WGN, int BK, int STAGES, bool GATED, bool SPLITK = false>
__global__ __launch_bounds__(kGemmThreads) void grouped_gemm_kernel(const GemmArgs p) {
#if defined(__HIP_DEVICE_COMPILE__)   // buffer resources exist in device code only
  static_assert(WGM * WGN == 4, "four wavefronts per workgroup");
  static_assert(BK == 32 || BK == 64, "LDS rows are 64 or 128 bytes");
  constexpr int WM = BM / WGM, WN = BN / WGN;
  constexpr int MI = WM / 32, NJ = WN / 32;
  static_assert(MI >= 1 && NJ >= 1 && (!GATED || NJ % 2 == 0), "tile shape");
  static_assert(!(GATED && SPLITK), "the gated epilogue needs complete sums");
  constexpr int kRowBytes = BK * 2;
  constexpr int CPR = BK / 8;                 // 16-byte chunks per LDS row
  constexpr int RPG = 1024 / kRowBytes;       // rows filled by one wavefront-wide 16-byte load
  static_assert(BM % (4 * RPG) == 0 && BN % (4 * RPG) == 0, "tile rows split over 4 wavefronts");
  constexpr int A_CH = BM / (4 * RPG);        // load instructions per wavefront per stage
  constexpr int B_CH = BN / (4 * RPG);
  constexpr int LPS = A_CH + B_CH;
  constexpr int kStageBytes = (BM + BN) * kRowBytes;
  constexpr int KK = BK / 16;                 // MFMA k-steps per stage
  static_assert((STAGES - 1) * LPS <= 63, "vmcnt is a 6-bit counter");

  extern __shared__ __align__(16) uint8_t smem[];

  const int n_work = p.tiles[1];
  const int xcd = blockIdx.x % kXcds;
  const int item = blockIdx.x / kXcds;
  if (item >= n_work) return;
  const int32_t* sched = p.tiles + p.tiles[2];
  const int mt = sched[2 * item];
  const int nt = sched[2 * item + 1] * kXcds + xcd;
  if (nt >= p.n_ntiles) return;
  const int4 tile = *reinterpret_cast<const int4*>(p.tiles + 4 + 4 * mt);
  const int g = tile.x, row_start = tile.y, row_count = tile.z, tok_base = tile.w;

  const uint16_t* b0 = (const uint16_t*)(g < p.E ? p.B0[g] : p.SB0[g - p.E]);
  const uint16_t* b1 = nullptr;
  if (GATED) b1 = (const uint16_t*)(g < p.E ? p.B1[g] : p.SB1[g - p.E]);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // kept in a scalar register
  const int wm = wave / WGN, wn = wave % WGN;
  const int r32 = lane & 31, q = lane >> 5;

  // ---- global -> LDS assignment ------------------------------------------------
  // Wavefront w fills row groups w, w + 4, ...; a lane owns LDS slot lane % CPR of
  // row lane / CPR of the group and fetches the chunk that belongs in that slot.
  const int sub = lane / CPR;
  const int lrow = wave * RPG + sub;              // + 4 RPG i (>= 32 rows: does not change the key)
  const int c = (lane % CPR) ^ swizzle_key<BK>(lrow);   // global chunk fetched by this lane
  // Buffer resources (base, size for the hardware range check): loads are
  // buffer_load_dwordx4 ... lds with a per-lane 32-bit byte offset that never
  // changes and the k offset in a scalar register, so a load costs no vector ALU
  // work and an out-of-range row can only read zeros.
  const __amdgpu_buffer_rsrc_t a_rsrc =
      __builtin_amdgcn_make_buffer_rsrc((void*)p.A, 0, (int)p.a_bytes, kBufferFlags);
  const __amdgpu_buffer_rsrc_t b0_rsrc =
      __builtin_amdgcn_make_buffer_rsrc((void*)b0, 0, (int)p.b_bytes, kBufferFlags);
  const __amdgpu_buffer_rsrc_t b1_rsrc =
      __builtin_amdgcn_make_buffer_rsrc((void*)(GATED ? b1 : b0), 0, (int)p.b_bytes, kBufferFlags);
  uint32_t a_voff[A_CH];
#pragma unroll
  for (int i = 0; i < A_CH; ++i) {
    const int rr = min(lrow + 4 * RPG * i, row_count - 1);
    uint32_t src;
    if (GATED) src = tok_base >= 0 ? (uint32_t)(tok_base + rr) : (uint32_t)(p.local_src[row_start + rr] / p.top_k);
    else src = (uint32_t)(row_start + rr);
    a_voff[i] = (src * (uint32_t)p.K + c * 8) * 2;
  }
  bool b_up[B_CH];
  uint32_t b_voff[B_CH];
#pragma unroll
  for (int i = 0; i < B_CH; ++i) {
    const int g0 = wave * RPG + 4 * RPG * i;      // first tile row of the group (scalar)
    if (GATED) {
      // tile rows [w WN, w WN + WN/2) are gate rows, the next WN/2 the up rows of the same f
      const int w = g0 / WN, within = g0 % WN;
      b_up[i] = within >= WN / 2;
      const int f = min(nt * (BN / 2) + w * (WN / 2) + (within % (WN / 2)) + sub, p.N - 1);
      b_voff[i] = ((uint32_t)f * (uint32_t)p.K + c * 8) * 2;
    } else {
      const int n = min(nt * BN + g0 + sub, p.N - 1);
      b_up[i] = false;
      b_voff[i] = ((uint32_t)n * (uint32_t)p.K + c * 8) * 2;
    }
  }

  // this workgroup's slice of the contraction, in k-tiles
  const int KT_all = p.K / BK;
  const int kt_first = SPLITK ? (int)((long long)KT_all * blockIdx.y / gridDim.y) : 0;
  const int kt_last = SPLITK ? (int)((long long)KT_all * (blockIdx.y + 1) / gridDim.y) : KT_all;
  const int KT = kt_last - kt_first;
  if (SPLITK && KT <= 0) return;

  // Issues loads [first, last) of the LPS loads that fill one stage with k-tile kt
  // (A row groups first, then B row groups).
  auto issue_loads = [&](int kt, int stage, int first, int last) {
    // wave-uniform LDS base of this wavefront's first row group; lane * 16 is implicit
    uint8_t* base = smem + stage * kStageBytes + wave * RPG * kRowBytes;
    const int koff = (kt_first + kt) * (BK * 2);
#pragma unroll
    for (int i = 0; i < A_CH; ++i)
      if (i >= first && i < last)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(a_rsrc, (lds_ptr_t)(base + i * 4 * RPG * kRowBytes),
                                                 16, a_voff[i], koff, 0, 0);
#pragma unroll
    for (int i = 0; i < B_CH; ++i)
      if (A_CH + i >= first && A_CH + i < last)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(b_up[i] ? b1_rsrc : b0_rsrc,
                                                 (lds_ptr_t)(base + (BM + i * 4 * RPG) * kRowBytes),
                                                 16, b_voff[i], koff, 0, 0);
  };

  f32x16 acc[MI][NJ];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // operand rows of this lane inside the LDS tile
  const int a_off = (wm * WM + r32) * kRowBytes;          // + 32 i rows
  const int b_off = (BM + wn * WN + r32) * kRowBytes;     // + 32 j rows
  const int key_r = swizzle_key<BK>(r32);

  bf16x8 af[2][MI], bfr[2][NJ];
  auto read_frags = [&](int stage, int kk, int buf) {
    const uint8_t* base = smem + stage * kStageBytes;
    const int slot = ((kk * 2 + q) ^ key_r) * 16;
    // in the order the MFMAs below consume them
    af[buf][0] = *reinterpret_cast<const bf16x8*>(base + a_off + slot);
#pragma unroll
    for (int j = 0; j < NJ; ++j)
      bfr[buf][j] = *reinterpret_cast<const bf16x8*>(base + b_off + j * 32 * kRowBytes + slot);
#pragma unroll
    for (int i = 1; i < MI; ++i)
      af[buf][i] = *reinterpret_cast<const bf16x8*>(base + a_off + i * 32 * kRowBytes + slot);
  };

  // Ring protocol (STAGES >= 3).  The prologue fills stages 0..STAGES-2 with
  // k-tiles 0..STAGES-2.  Iteration kt computes from stage kt % STAGES and, spread
  // evenly over its MFMA steps, refills stage (kt - 1) % STAGES -- free since the
  // barrier that ended iteration kt - 1 -- with k-tile kt + STAGES - 1.  In its last
  // step the wavefront waits until k-tile kt + 1 has landed (vmcnt counts only the
  // younger loads), drains its own LDS reads, meets the others at the barrier and
  // reads the first operands of k-tile kt + 1.  The last part of the refill is issued
  // after the barrier so that it, too, sits among MFMAs.  Past the end the refill
  // re-fetches the last k-tile into a stage nobody reads again, which keeps the
  // vmcnt bookkeeping uniform.
  static_assert(STAGES >= 3, "ring needs a free stage to refill during an iteration");
  constexpr int kPart = (LPS + KK - 1) / KK;     // most loads one step issues

#pragma unroll
  for (int s = 0; s < STAGES - 1; ++s) issue_loads(min(s, KT - 1), s, 0, LPS);
  wait_vmcnt<(STAGES - 2) * LPS>();
  __builtin_amdgcn_s_barrier();
  read_frags(0, 0, 0);

  int stage = 0;                       // kt % STAGES
  int fill_stage = STAGES - 1;         // (kt + STAGES - 1) % STAGES
  for (int kt = 0; kt < KT; ++kt) {
    const int next_stage = stage + 1 == STAGES ? 0 : stage + 1;
    const int fill_kt = min(kt + STAGES - 1, KT - 1);
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      constexpr int kReads = MI + NJ;
      constexpr int kMfma = MI * NJ;
      if (kk + 1 < KK) {
        read_frags(stage, kk + 1, (kk + 1) & 1);
      } else {
        wait_vmcnt<(STAGES - 3) * LPS + (KK - 1) * LPS / KK>();
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        read_frags(next_stage, 0, (kk + 1) & 1);
      }
      issue_loads(fill_kt, fill_stage, kk * LPS / KK, (kk + 1) * LPS / KK);
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[kk & 1][j], af[kk & 1][i], acc[i][j], 0, 0, 0);
      // Issue order inside the step: one MFMA first (so the wait for this step's
      // operands precedes any new LDS read), then the next step's operand reads one
      // per MFMA, then this step's share of the refill one per MFMA.
      // (Tiles with too little matrix work per step are left to the compiler.)
      if constexpr (kMfma >= kReads + kPart + 1) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
#pragma unroll
        for (int r = 0; r < kReads; ++r) {
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        }
#pragma unroll
        for (int r = 0; r < kPart; ++r) {
          __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, kMfma - 1 - kReads - kPart, 0);
      }
    }
    stage = next_stage;
    fill_stage = fill_stage + 1 == STAGES ? 0 : fill_stage + 1;
  }

  // ---- epilogue ---------------------------------------------------------------
  // The weight rows are the MFMA's first operand, so accumulator register v of
  // lane (r32, q) is output row (activation row) r32 of subtile i and output
  // column 8 (v / 4) + 4 q + v % 4 of subtile j: four consecutive columns per
  // register quad, written as one 8-byte (bf16) or 16-byte (fp32 partial) store.
#pragma unroll
  for (int i = 0; i < MI; ++i) {
    const int row = wm * WM + i * 32 + r32;
    if (row >= row_count) continue;
    const size_t crow = (size_t)(row_start + row);
    if (GATED) {
      constexpr int NH = NJ / 2;
#pragma unroll
      for (int j = 0; j < NH; ++j)
#pragma unroll
        for (int vg = 0; vg < 4; ++vg) {
          const int f = nt * (BN / 2) + wn * (WN / 2) + j * 32 + vg * 8 + q * 4;
          if (f < p.N) {
            bf16x4 o;
#pragma unroll
            for (int e = 0; e < 4; ++e)
              o[e] = (bf16_t)(silu(acc[i][j][vg * 4 + e]) * acc[i][j + NH][vg * 4 + e]);
            *reinterpret_cast<bf16x4*>(p.C + crow * p.N + f) = o;
          }
        }
    } else {
#pragma unroll
      for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int vg = 0; vg < 4; ++vg) {
          const int n = nt * BN + wn * WN + j * 32 + vg * 8 + q * 4;
          if (n < p.N) {
            if (SPLITK) {
              const f32x4 o = {acc[i][j][vg * 4], acc[i][j][vg * 4 + 1], acc[i][j][vg * 4 + 2],
                               acc[i][j][vg * 4 + 3]};
              *reinterpret_cast<f32x4*>(p.Cpart + ((size_t)blockIdx.y * p.c_rows + crow) * p.N + n) = o;
            } else {
              bf16x4 o;
#pragma unroll
              for (int e = 0; e < 4; ++e) o[e] = (bf16_t)acc[i][j][vg * 4 + e];
              *reinterpret_cast<bf16x4*>(p.C + crow * p.N + n) = o;
            }
          }
        }
    }
  }
#endif  // __HIP_DEVICE_COMPILE__
}

// Upper bound on the number of row tiles for T tokens (host side).
static inline int max_row_tiles(const prism_layer_desc& d, int T, int BM) {
  return T * d.top_k / BM + d.n_experts + d.n_shared * ceil_div(T, BM);
}

// Launches the schedule builder for one GEMM: row tile BM, n_ntiles column tiles.
static inline prism_status launch_build_schedule(const prism_layer_desc& d,
                                                 const int32_t* local_offsets, int T, int BM,
                                                 int n_ntiles, int32_t* tiles, hipStream_t st) {
  hipLaunchKernelGGL(build_schedule_kernel, dim3(1), dim3(512), 0, st, local_offsets, d.n_experts,
                     d.n_shared, T, T * d.top_k, BM, ceil_div(n_ntiles, kXcds),
                     max_row_tiles(d, T, BM), tiles);
  PRISM_CHECK_LAUNCH();
  return PRISM_OK;
}

template <int BM, int BN, int WGM, int WGN, int BK, int STAGES, bool GATED, bool SPLITK = false>
prism_status launch_gemm(const GemmArgs& args, int max_mtiles, hipStream_t st, int n_splits = 1) {
  constexpr int smem = STAGES * (BM + BN) * BK * 2;
  static_assert(smem <= 160 * 1024, "LDS per workgroup");
  auto kernel = grouped_gemm_kernel<BM, BN, WGM, WGN, BK, STAGES, GATED, SPLITK>;
  static bool attr_set = false;
  if (!attr_set) {
    if (hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, smem) != hipSuccess)
      return PRISM_ERR_LAUNCH;
    attr_set = true;
  }
  const long long blocks = (long long)max_mtiles * ceil_div(args.n_ntiles, kXcds) * kXcds;
  if (blocks <= 0) return PRISM_OK;
  if (blocks > 0x7fffffffLL) return PRISM_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(kernel, dim3((unsigned)blocks, SPLITK ? n_splits : 1), dim3(kGemmThreads), smem,
                     st, args);
  PRISM_CHECK_LAUNCH();
  return PRISM_OK;
}

}  // namespace gg
}  // namespace prism
#endif  // PRISM_GROUPED_GEMM_H_
