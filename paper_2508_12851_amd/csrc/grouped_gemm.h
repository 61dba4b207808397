// Grouped "NT" GEMM on the bf16 matrix cores of gfx950, used for both halves of
// the SwiGLU expert FFN (paper Sec. III-A, local expert execution):
//
//   GATED   h[r, f] = silu( x[tok(r)] . W_gate^g[f] ) * ( x[tok(r)] . W_up^g[f] )
//   plain   y[r, n] = h[r] . W_down^g[n]
//
// Rows are grouped by expert g; a device-built schedule gives every workgroup its
// (row tile, column tile) items, so the host never needs the routing-dependent
// segment sizes.
//
// Kernel shape: BM x BN output tile per workgroup of 4 wavefronts (WGM x WGN),
// v_mfma_f32_32x32x16_bf16, operand tiles of BK contraction elements staged in
// LDS in a ring of STAGES stages.  An LDS row holds BK contraction elements
// (128 or 64 bytes) as 16-byte chunks; chunk c of row r sits in slot
// c ^ key(r) (key = (r >> 1) & 7 for 128-byte rows, (r >> 2) & 3 for 64-byte
// rows), so the 16-byte operand reads of 16 consecutive rows hit 16 different
// slots of the 256-byte bank window.  Stages are filled by buffer_load_dwordx4
// ... lds (no VGPR staging): one instruction fills 1 KiB, and because each
// lane's LDS slot is fixed (lane * 16 bytes), the swizzle is applied to the
// global chunk a lane fetches instead.  A stage is awaited with s_waitcnt
// vmcnt(n), n = the loads of the younger stages, then one s_barrier per stage
// orders the ring.
//
// The kernel is persistent: a workgroup walks its list of items, and the ring
// keeps running across items -- while the last k-tiles of one item are being
// multiplied, the first k-tiles of the next are already being fetched, and they
// land while the epilogue of the first stores its results.
//
// Work order: the hardware hands consecutive workgroup ids to the 8 XCDs in
// turn, each with a private L2.  The schedule (schedule.h) gives every XCD one
// list of items in which consecutive items form small rectangles of row tiles x
// column tiles of one expert, so the workgroups resident on an XCD share a few
// activation tiles and a few weight tiles in that XCD's L2.
#ifndef PRISM_GROUPED_GEMM_H_
#define PRISM_GROUPED_GEMM_H_

#include "prism_internal.h"
#include "schedule.h"

namespace prism {
namespace gg {

// Workgroup b builds the schedule p[b] (one launch serves both GEMMs of the FFN).
__global__ __launch_bounds__(512) void build_schedule_kernel(
    const int32_t* __restrict__ local_offsets, int E, int S, int T, int A_total,
    const SchedParams p0, const SchedParams p1) {
  const SchedParams p[1] = {blockIdx.x == 0 ? p0 : p1};
  build_schedules_block<1>(local_offsets, E, S, T, A_total, p);
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
  const int32_t* sched;
  const int32_t* local_src;
  uint32_t src_bytes;       // size of local_src in bytes (T * k * 4)
  uint32_t a_bytes;         // size of A in bytes (buffer range check), < 2^32
  uint32_t b_bytes;         // size of one weight matrix in bytes, < 2^32
  int K;                    // contraction length (H for GEMM1, F for GEMM2)
  int N;                    // output columns (F for GEMM1, H for GEMM2)
  int top_k;
  int E;
  int b_tiled;              // weights in 16 x 32 tiles (prism.h) instead of row-major
};

constexpr int kGemmThreads = 256;

// Epilogue strips: 32 rows x 64 bf16 columns per wavefront at a row pitch of 144 bytes
// (16-byte aligned rows whose starts fall into different banks).  Used by the plain GEMM when a
// wavefront's output is at least 64 bf16 columns wide (the gated GEMM, whose epilogue is
// dominated by the SiLU arithmetic, ran 5-10 % slower with it).
constexpr int kStripPitch = 144;
constexpr int kStripBytes = 32 * kStripPitch;
template <int WN, bool GATED, bool SPLITK> constexpr bool staged_store() {
  return !SPLITK && !GATED && (WN / 32) % 2 == 0;
}
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Schedule entries and pointer tables are written before the kernel starts and
// never during it; reading them through the constant address space lets the
// compiler use scalar loads, which the vector-memory counter does not see.
typedef const __attribute__((address_space(4))) int4* const_int4_ptr;
typedef const __attribute__((address_space(4))) int32_t* const_int_ptr;
typedef const void* const __attribute__((address_space(4)))* const_ptr_table;

// silu(z) = z / (1 + e^-z) with the hardware exp2 and reciprocal (each within 1 ulp;
// the result is rounded to bf16 right after).
__device__ __forceinline__ float silu(float z) {
  return z * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.44269504088896341f * z));
}

// LDS slot swizzle.  The LDS serves a 16-byte-per-lane read 16 lanes (256 bytes,
// 64 banks) per cycle, so 16 consecutive rows read at the same logical chunk
// must land in 16 different 16-byte slots of the 256-byte bank window: rows
// that share (row * row_bytes) mod 256 get different keys.
template <int BK> __device__ __forceinline__ int swizzle_key(int row) {
  return BK == 64 ? ((row >> 1) & 7) : ((row >> 2) & 3);
}

// BM x BN output tile per workgroup; BN counts weight rows in the tile (for
// GATED: BN/2 gate rows and BN/2 up rows).  Wavefronts form a WGM x WGN grid.
// BK contraction elements per LDS stage (32 or 64), STAGES stages in flight.
// SPLITK: n workgroups share every item, each over its own slice of the contraction, n being
// what the schedule builder chose (schedule.h, "Splits"); the tile is written as fp32 partial
// sums to p.Cpart[slice][row][col] (plain GEMM only).
// ROTATE: every item walks its k-tiles cyclically from an item-dependent start, so
// concurrent workgroups read different column ranges of their weight rows (for
// schedules in which workgroups share no weight tiles, i.e. one row tile per group).
// These are the schedules that deal their items to the XCDs one by one; the kernel works out
// its items from the schedule's table of row tiles (schedule.h) instead of reading lists.
// STREAM_B: the weight loads carry the non-temporal hint.  For batches in which every weight
// tile is read by one workgroup only (one row tile per expert) the weights cross the memory
// system once, and reads marked that way stream from HBM about 15 % faster than plain ones
// (7.0-7.2 against 6.2-6.4 TB/s for direct-to-LDS loads on this machine).
// SLICES: the launch takes the schedule's slice entries -- the items of a partly filled last
// round, cut along the contraction (schedule.h, "Last round") -- instead of its item lists: an
// entry covers its own range of k-tiles and leaves its accumulators as an fp32 tile in slot
// `part` of p.Cpart (plain GEMM only).  A launch of its own, so that the kernel that does the
// bulk of the work carries none of this.
template <int BM, int BN, int WGM, int WGN, int BK, int STAGES, bool GATED, bool SPLITK = false,
          bool ROTATE = false, bool STREAM_B = false, bool SLICES = false>
__global__ __launch_bounds__(kGemmThreads) void grouped_gemm_kernel(const GemmArgs p) {
#if defined(__HIP_DEVICE_COMPILE__)   // buffer resources exist in device code only
  static_assert(WGM * WGN == 4, "four wavefronts per workgroup");
  static_assert(BK == 32 || BK == 64, "LDS rows are 64 or 128 bytes");
  constexpr int WM = BM / WGM, WN = BN / WGN;
  constexpr int MI = WM / 32, NJ = WN / 32;
  static_assert(MI >= 1 && NJ >= 1 && (!GATED || NJ % 2 == 0), "tile shape");
  static_assert(!(GATED && SPLITK), "the gated epilogue needs complete sums");
  static_assert(!SLICES || (!GATED && !SPLITK && !ROTATE), "slices are entries of the plain prefill GEMM");
  constexpr int kRowBytes = BK * 2;
  constexpr int CPR = BK / 8;                 // 16-byte chunks per LDS row
  constexpr int RPG = 1024 / kRowBytes;       // rows filled by one wavefront-wide 16-byte load
  static_assert(BM % (4 * RPG) == 0 && BN % (4 * RPG) == 0, "tile rows split over 4 wavefronts");
  constexpr int A_CH = BM / (4 * RPG);        // load instructions per wavefront per stage
  constexpr int B_CH = BN / (4 * RPG);
  constexpr int LPS = A_CH + B_CH;
  constexpr int kStageBytes = (BM + BN) * kRowBytes;
  constexpr int KK = BK / 16;                 // MFMA k-steps per stage
  static_assert(STAGES >= 3, "ring needs a free stage to refill during an iteration");
  static_assert((STAGES - 1) * LPS <= 63, "vmcnt is a 6-bit counter");

  // wide bf16 output tiles are stored through LDS strips (see the epilogue)
  constexpr bool kStagedStore = staged_store<WN, GATED, SPLITK>();
  constexpr int kStripBase = STAGES * kStageBytes + (GATED ? 4096 : 0);

  extern __shared__ __align__(16) uint8_t smem[];

  // ---- this workgroup's items: slot, slot + slots, ... of its XCD's list -----------
  const int xcd = blockIdx.x % kXcds;
  int slot = blockIdx.x / kXcds;
  const const_int_ptr sched_c = (const_int_ptr)p.sched;
  const int count = sched_c[(SLICES ? 20 : 4) + xcd];
  int launched = gridDim.x / kXcds;
  // SPLITK: the schedule says how many workgroups share an item; neighbouring workgroups of an
  // XCD take the splits of one item slot, and those left over when the count does not divide the
  // launch end here.
  const int n_splits = SPLITK ? max(sched_c[2], 1) : 1;
  const int split = SPLITK ? slot % n_splits : 0;
  if (SPLITK) {
    slot /= n_splits;
    launched /= n_splits;
    if (slot >= launched) return;
  }
  if (slot >= count) return;
  // The list takes ceil(count / launched slots) rounds; the fewest workgroups that still
  // finish in that many rounds share it evenly (a workgroup that would sit out the last
  // round only takes memory bandwidth from the others in the rounds before).
  const int rounds = (count + launched - 1) / launched;
  const int slots = (count + rounds - 1) / rounds;
  if (slot >= slots) return;
  // slice entries sit in the last kSliceSlots places of every list
  const const_int4_ptr items =
      (const_int4_ptr)(p.sched + kSchedHeader) +
      ((size_t)xcd * sched_c[1] + (SLICES ? sched_c[1] - kSliceSlots : 0)) * (kItemInts / 4);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // kept in a scalar register
  const int wm = wave / WGN, wn = wave % WGN;
  const int r32 = lane & 31, q = lane >> 5;

  // this workgroup's slice of the contraction, in k-tiles
  const int KT_all = p.K / BK;
  const int kt_first = SPLITK ? (int)((long long)KT_all * split / n_splits) : 0;
  const int kt_last = SPLITK ? (int)((long long)KT_all * (split + 1) / n_splits) : KT_all;
  const int KT = kt_last - kt_first;
  if (KT <= 0) return;

  // ---- global -> LDS assignment ------------------------------------------------
  // Wavefront w fills row groups w, w + 4, ...; a lane owns LDS slot lane % CPR of
  // row lane / CPR of the group and fetches the chunk that belongs in that slot.
  // Loads are buffer_load_dwordx4 ... lds with a per-lane 32-bit byte offset that
  // never changes within an item and the k offset in a scalar register, so a load
  // costs no vector ALU work; the buffer size makes an out-of-range row read zeros.
  const int sub = lane / CPR;
  const int lrow = wave * RPG + sub;              // + 4 RPG i (>= 32 rows: does not change the key)
  const int c = (lane % CPR) ^ swizzle_key<BK>(lrow);   // global chunk fetched by this lane
  const __amdgpu_buffer_rsrc_t a_rsrc =
      __builtin_amdgcn_make_buffer_rsrc((void*)p.A, 0, (int)p.a_bytes, kBufferFlags);

  // Item header as stored in the schedule.
  struct Item {
    int g, row_start, row_count, tok_base, nt;
    int kt0, kt_n, part;     // SLICES: the entry's k-tiles [kt0, kt0 + kt_n) and its partial-tile slot
  };
  // What the loads and the epilogue of an item need.
  struct Ctx {
    int row_start, row_count, nt;
    int kt0, kt_n, part;     // as in Item
    int rot;                 // ROTATE: k-tile this item starts its contraction with
    const void* b0;
    const void* b1;
    uint32_t a_voff[A_CH];
    uint32_t b_voff[B_CH];
  };
  // ROTATE schedules hold one line per row tile instead of item lists (schedule.h)
  const int n_ntiles = (p.N + (GATED ? BN / 2 : BN) - 1) / (GATED ? BN / 2 : BN);
  auto fetch_item = [&](int idx) {   // idx is clamped: the result is only used when idx < count
    const int i = min(idx, count - 1);
    if (ROTATE) {
      const unsigned seq = (unsigned)i * kXcds + (unsigned)xcd;
      const unsigned tile = seq / (unsigned)n_ntiles;
      const int4 h0 = ((const_int4_ptr)(p.sched + kSchedHeader))[tile];
      return Item{h0.x, h0.y, h0.z, h0.w, (int)(seq - tile * (unsigned)n_ntiles), 0, KT, -1};
    }
    const int4 h0 = items[2 * i];
    const int4 h1 = items[2 * i + 1];
    if (SLICES) return Item{h0.x, h0.y, h0.z, h0.w, h1.x, h1.y, h1.z, h1.w};
    return Item{h0.x, h0.y, h0.z, h0.w, h1.x, 0, KT, -1};
  };
  // Second hop: expert pointers (scalar loads) and, for the gathered GEMM, the
  // source rows of the row tile: each wavefront pulls the tile's BM entries of
  // local_src into its own 1 KiB of LDS with one buffer_load ... lds (so the load is
  // counted like the ring's loads and no VGPR waits on it), and reads its lanes'
  // entries from there once the load has surely landed.
  struct Raw {
    const void* b0;
    const void* b1;
  };
  static_assert(!GATED || BM <= 256, "one 1 KiB load brings the source rows of a row tile");
  uint8_t* const src_lds = smem + STAGES * kStageBytes + wave * 1024;
  const __amdgpu_buffer_rsrc_t src_rsrc =
      __builtin_amdgcn_make_buffer_rsrc((void*)p.local_src, 0, (int)p.src_bytes, kBufferFlags);
  auto fetch_raw = [&](const Item& it) {
    Raw r;
    const const_ptr_table t0 = (const_ptr_table)(it.g < p.E ? p.B0 : p.SB0);
    const const_ptr_table t1 = (const_ptr_table)(GATED ? (it.g < p.E ? p.B1 : p.SB1) : (it.g < p.E ? p.B0 : p.SB0));
    const int gi = it.g < p.E ? it.g : it.g - p.E;
    r.b0 = t0[gi];
    r.b1 = t1[gi];
    // Entry j of the LDS slot = local_src[row_start + j].  The whole byte offset sits in the
    // per-lane operand, which the hardware checks against the buffer size (a scalar offset
    // would escape that check), so entries past the end of local_src arrive as zeros instead
    // of being read.  Shared-expert tiles take their tokens from tok_base: their load is
    // issued out of range on purpose, which keeps the count of loads in flight uniform.
    if (GATED)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(
          src_rsrc, (lds_ptr_t)src_lds, 16,
          it.tok_base >= 0 ? kOutOfRange : (uint32_t)it.row_start * 4u + (uint32_t)lane * 16u, 0, 0, 0);
    return r;
  };
  // Byte offset of this lane's 16-byte chunk c of weight row n in k-tile 0 (the k-tile offset
  // is added per load): row-major, or tiles of 16 rows x 32 columns (1 KiB, rows 64 bytes
  // apart) laid out row-tile major -- a 64-wide k-tile spans two neighbouring tiles.
  auto tiled_offset = [&](uint32_t n, uint32_t cols) {
    return (n >> 4) * (cols >> 5) * 1024u + (n & 15u) * 64u + (uint32_t)(c >> 2) * 1024u +
           (uint32_t)(c & 3) * 16u;
  };
  auto weight_row_offset = [&](uint32_t n) {
    return p.b_tiled ? tiled_offset(n, (uint32_t)p.K) : n * (uint32_t)p.K * 2u + (uint32_t)c * 16u;
  };
  auto make_ctx = [&](const Item& it, const Raw& raw) {
    Ctx cx;
    cx.row_start = it.row_start; cx.row_count = it.row_count; cx.nt = it.nt;
    cx.kt0 = it.kt0; cx.kt_n = it.kt_n; cx.part = it.part;
    cx.rot = ROTATE ? (int)((unsigned)(it.nt * 13 + it.g * 29) % (unsigned)KT) : 0;
    cx.b0 = raw.b0; cx.b1 = raw.b1;
#pragma unroll
    for (int i = 0; i < A_CH; ++i) {
      const int rr = min(lrow + 4 * RPG * i, it.row_count - 1);
      uint32_t src;
      if (GATED) {
        const int a = reinterpret_cast<const int*>(src_lds)[rr];
        src = it.tok_base >= 0 ? (uint32_t)(it.tok_base + rr) : (uint32_t)(a / p.top_k);
      } else {
        src = (uint32_t)(it.row_start + rr);
      }
      // Rows past the end of a partly filled tile get an offset beyond the buffer: the
      // hardware then returns zeros, and all-zero operands cost the matrix cores far
      // less power than real data (the chip is power-limited in this kernel).
      cx.a_voff[i] = lrow + 4 * RPG * i < it.row_count ? (src * (uint32_t)p.K + c * 8) * 2 : kOutOfRange;
    }
#pragma unroll
    for (int i = 0; i < B_CH; ++i) {
      const int g0 = wave * RPG + 4 * RPG * i;      // first tile row of the group (scalar)
      if (GATED) {
        // tile rows [w WN, w WN + WN/2) are gate rows, the next WN/2 the up rows of the same f
        const int w = g0 / WN, within = g0 % WN;
        const int f = min(it.nt * (BN / 2) + w * (WN / 2) + (within % (WN / 2)) + sub, p.N - 1);
        cx.b_voff[i] = weight_row_offset((uint32_t)f);
      } else {
        const int n = min(it.nt * BN + g0 + sub, p.N - 1);
        cx.b_voff[i] = weight_row_offset((uint32_t)n);
      }
    }
    return cx;
  };

  // Issues loads [first, last) of the LPS loads that fill one stage with k-tile kt
  // of item cx (A row groups first, then B row groups).
  auto issue_loads = [&](const Ctx& cx, int kt, int stage, int first, int last) {
    // wave-uniform LDS base of this wavefront's first row group; lane * 16 is implicit
    uint8_t* base = smem + stage * kStageBytes + wave * RPG * kRowBytes;
    int kt_mem = kt;
    if (ROTATE) {
      kt_mem += cx.rot;
      if (kt_mem >= KT) kt_mem -= KT;
    }
    const int kel = (kt_first + (SLICES ? cx.kt0 : 0) + kt_mem) * BK;   // first contraction element
    const int koff = kel * 2;
    const int koff_b = p.b_tiled ? (kel >> 5) * 1024 : koff;   // kel is a multiple of 32
    const __amdgpu_buffer_rsrc_t b0_rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void*)cx.b0, 0, (int)p.b_bytes, kBufferFlags);
    const __amdgpu_buffer_rsrc_t b1_rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void*)cx.b1, 0, (int)p.b_bytes, kBufferFlags);
#pragma unroll
    for (int i = 0; i < A_CH; ++i)
      if (i >= first && i < last)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(a_rsrc, (lds_ptr_t)(base + i * 4 * RPG * kRowBytes),
                                                 16, cx.a_voff[i], koff, 0, 0);
#pragma unroll
    for (int i = 0; i < B_CH; ++i)
      if (A_CH + i >= first && A_CH + i < last) {
        const int g0 = wave * RPG + 4 * RPG * i;
        const bool up = GATED && (g0 % WN) >= WN / 2;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(up ? b1_rsrc : b0_rsrc,
                                                 (lds_ptr_t)(base + (BM + i * 4 * RPG) * kRowBytes),
                                                 16, cx.b_voff[i], koff_b, 0, STREAM_B ? kNonTemporal : 0);
      }
  };

  // operand rows of this lane inside the LDS tile
  // Row subtile i of this wavefront is tile rows 32 (i WGM + wm) .. (the subtiles of
  // the WGM wavefront rows interleave).
  const int a_off = (wm * 32 + r32) * kRowBytes;          // + 32 WGM i rows
  const int b_off = (BM + wn * WN + r32) * kRowBytes;     // + 32 j rows
  const int key_r = swizzle_key<BK>(r32);

  bf16x8 af[2][MI], bfr[2][NJ];
  auto read_frags = [&](int stage, int kk, int buf) {
    const uint8_t* base = smem + stage * kStageBytes;
    const int slot_b = ((kk * 2 + q) ^ key_r) * 16;
    // in the order the MFMAs below consume them
    af[buf][0] = *reinterpret_cast<const bf16x8*>(base + a_off + slot_b);
#pragma unroll
    for (int j = 0; j < NJ; ++j)
      bfr[buf][j] = *reinterpret_cast<const bf16x8*>(base + b_off + j * 32 * kRowBytes + slot_b);
#pragma unroll
    for (int i = 1; i < MI; ++i)
      af[buf][i] = *reinterpret_cast<const bf16x8*>(base + a_off + i * WGM * 32 * kRowBytes + slot_b);
  };

  f32x16 acc[MI][NJ];

  // Ring protocol.  The k-tiles of this workgroup's items form one stream; stream
  // position g is computed from stage g % STAGES.  The prologue fills stages
  // 0..STAGES-2.  Iteration g, spread evenly over its MFMA steps, refills stage
  // (g - 1) % STAGES -- free since the barrier that ended iteration g - 1 -- with
  // stream position g + STAGES - 1 (which may belong to the next item).  In its last
  // step the wavefront waits until position g + 1 has landed (vmcnt counts only the
  // younger loads), drains its own LDS reads, meets the others at the barrier and
  // reads the first operands of position g + 1.  The last part of the refill is
  // issued after the barrier so that it, too, sits among MFMAs.
  constexpr int kPart = (LPS + KK - 1) / KK;     // most loads one step issues
  int stage = 0;                       // g % STAGES
  int fill_stage = STAGES - 1;         // (g + STAGES - 1) % STAGES
  auto k_iteration = [&](const Ctx& fill_cx, int fill_kt) {
    const int next_stage = stage + 1 == STAGES ? 0 : stage + 1;
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
      issue_loads(fill_cx, fill_kt, fill_stage, kk * LPS / KK, (kk + 1) * LPS / KK);
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j0 = 0; j0 < NJ; ++j0) {
          // snake order over the grid of accumulators: every MFMA shares an operand with the one
          // before it (0.5 % on the power-limited prefill GEMMs)
          const int j = (i & 1) ? NJ - 1 - j0 : j0;
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[kk & 1][j], af[kk & 1][i], acc[i][j], 0, 0, 0);
        }
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
      } else if constexpr (kMfma >= (kReads > kPart ? kReads : kPart) + 1) {
        // fewer MFMAs per step: an operand read and a refill load share the gap after an MFMA
        constexpr int kGaps = kReads > kPart ? kReads : kPart;
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
#pragma unroll
        for (int r = 0; r < kGaps; ++r) {
          if (r < kReads) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
          if (r < kPart) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, kMfma - 1 - kGaps, 0);
      }
    }
    stage = next_stage;
    fill_stage = fill_stage + 1 == STAGES ? 0 : fill_stage + 1;
  };

  // The weight rows are the MFMA's first operand, so accumulator register v of
  // lane (r32, q) is output row (activation row) r32 of subtile i and output
  // column 8 (v / 4) + 4 q + v % 4 of subtile j: four consecutive columns per
  // register quad, i.e. one 8-byte (bf16) or 16-byte (fp32 partial) piece.
  //
  // Stored straight from there, an instruction writes 16 bytes to each of 32 rows, and the
  // write path then takes a fifth of a short-contraction item (12.6k clocks against 54k of
  // k-loop for the 1408-long down projection).  Wide bf16 tiles therefore pass every strip
  // of 32 rows x 64 columns through a 4.5 KiB LDS buffer of the wavefront's own (row pitch
  // 144 bytes) and store it with 16 bytes per lane, 8 lanes per row: whole 128-byte lines.
  // The LDS instructions come from assembly: for LDS accesses it sees, the compiler would
  // first wait for every direct-to-LDS load in flight (the next item's operands).  A
  // wavefront's LDS instructions execute in order, so the read-back needs no wait after the
  // writes, nor the next strip's writes after the read-back.
  auto epilogue_staged = [&](const Ctx& cx) {
    constexpr int NO = GATED ? NJ / 2 : NJ;                 // output column subtiles of 32
    constexpr int kPairs = NO / 2 > 0 ? NO / 2 : 1;         // (instantiated for narrow tiles too, never called)
    constexpr int kStrips = MI * kPairs;                  // strip s: row subtile s / kPairs, column pair s % kPairs
    const uint32_t strip = (uint32_t)(uintptr_t)(lds_ptr_t)(smem + kStripBase) + wave * kStripBytes;
    const uint32_t wr = strip + r32 * kStripPitch + q * 8;  // + 2 (32 jl + 8 vg)
    const int rd_row = lane >> 3, rd_chunk = lane & 7;       // + 8 t rows
    const uint32_t rd = strip + rd_row * kStripPitch + rd_chunk * 16;
    const int col0 = (GATED ? cx.nt * (BN / 2) + wn * (WN / 2) : cx.nt * BN + wn * WN) + rd_chunk * 8;
    // the values of a strip as this lane holds them: 2 subtiles x 4 quads of 4 bf16
    auto strip_values = [&](int st, u32x2 (&o)[8]) {
      const int i = st / kPairs, jp = st % kPairs;
#pragma unroll
      for (int jl = 0; jl < 2; ++jl)
#pragma unroll
        for (int vg = 0; vg < 4; ++vg) {
          const int j = jp * 2 + jl;
          bf16x4 b;
#pragma unroll
          for (int e = 0; e < 4; ++e)
            b[e] = GATED ? (bf16_t)(silu(acc[i][j][vg * 4 + e]) * acc[i][j + NO][vg * 4 + e])
                         : (bf16_t)acc[i][j][vg * 4 + e];
          o[jl * 4 + vg] = __builtin_bit_cast(u32x2, b);
        }
    };
    // Strip st + 1 is computed while the writes of strip st are on their way.
    u32x2 cur[8], nxt[8];
    strip_values(0, cur);
#pragma unroll
    for (int st = 0; st < kStrips; ++st) {
      const int i = st / kPairs, jp = st % kPairs;
      const int row0 = (i * WGM + wm) * 32;
      const bool live = row0 < cx.row_count;                // wavefront-uniform
      // keep every strip's instructions together: moved up by the scheduler, the accumulator
      // reads of all strips would be live at once and push other values into scratch memory
      __builtin_amdgcn_sched_barrier(0);
      if (live) {
#pragma unroll
        for (int w8 = 0; w8 < 8; ++w8)
          asm volatile("ds_write_b64 %0, %1 offset:%2"
                       :: "v"(wr), "v"(cur[w8]), "n"(((w8 / 4) * 32 + (w8 % 4) * 8) * 2) : "memory");
      }
      if (st + 1 < kStrips) strip_values(st + 1, nxt);
      if (live) {
        // one statement up to the wait: the compiler takes an output for valid as soon as its
        // statement ends (and may copy it elsewhere right away)
        u32x4 v0, v1, v2, v3;
        asm volatile(
            "ds_read_b128 %0, %4 offset:%5\n\tds_read_b128 %1, %4 offset:%6\n\t"
            "ds_read_b128 %2, %4 offset:%7\n\tds_read_b128 %3, %4 offset:%8\n\ts_waitcnt lgkmcnt(0)"
            : "=&v"(v0), "=&v"(v1), "=&v"(v2), "=&v"(v3)
            : "v"(rd), "n"(0), "n"(8 * kStripPitch), "n"(16 * kStripPitch), "n"(24 * kStripPitch)
            : "memory");
        const u32x4 v[4] = {v0, v1, v2, v3};
        const int col = col0 + jp * 64;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const int row = row0 + t * 8 + rd_row;
          if (row < cx.row_count && col < p.N)
            *reinterpret_cast<u32x4*>(p.C + (size_t)(cx.row_start + row) * p.N + col) = v[t];
        }
      }
#pragma unroll
      for (int w8 = 0; w8 < 8; ++w8) cur[w8] = nxt[w8];
    }
  };
  auto epilogue = [&](const Ctx& cx) {
    if constexpr (SLICES) {
      // the accumulators as they are, an fp32 tile [BM][BN] in slot cx.part
      float* tile = p.Cpart + (size_t)cx.part * (BM * BN);
#pragma unroll
      for (int i = 0; i < MI; ++i) {
        if ((i * WGM + wm) * 32 >= cx.row_count) continue;    // wave-uniform
        const int row = (i * WGM + wm) * 32 + r32;
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
          for (int vg = 0; vg < 4; ++vg) {
            const int n = wn * WN + j * 32 + vg * 8 + q * 4;
            const f32x4 o = {acc[i][j][vg * 4], acc[i][j][vg * 4 + 1], acc[i][j][vg * 4 + 2],
                             acc[i][j][vg * 4 + 3]};
            *reinterpret_cast<f32x4*>(tile + (size_t)row * BN + n) = o;
          }
      }
      return;
    }
    if constexpr (kStagedStore) {
      epilogue_staged(cx);
      return;
    }
#pragma unroll
    for (int i = 0; i < MI; ++i) {
      const int row = (i * WGM + wm) * 32 + r32;
      if (row >= cx.row_count) continue;
      const size_t crow = (size_t)(cx.row_start + row);
      if (GATED) {
        constexpr int NH = NJ / 2;
#pragma unroll
        for (int j = 0; j < NH; ++j)
#pragma unroll
          for (int vg = 0; vg < 4; ++vg) {
            const int f = cx.nt * (BN / 2) + wn * (WN / 2) + j * 32 + vg * 8 + q * 4;
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
            const int n = cx.nt * BN + wn * WN + j * 32 + vg * 8 + q * 4;
            if (n < p.N) {
              if (SPLITK) {
                const f32x4 o = {acc[i][j][vg * 4], acc[i][j][vg * 4 + 1], acc[i][j][vg * 4 + 2],
                                 acc[i][j][vg * 4 + 3]};
                *reinterpret_cast<f32x4*>(p.Cpart + ((size_t)split * p.c_rows + crow) * p.N + n) = o;
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
  };

  // ---- walk the items ---------------------------------------------------------------
  // Item headers are fetched two items ahead and their pointers / source rows one
  // item ahead, so nothing on the critical path waits for them.
  int idx = slot;
  Item it_cur = fetch_item(idx);
  const Raw raw_cur = fetch_raw(it_cur);
  wait_vmcnt<0>();                       // the first item's source rows
  Ctx cur = make_ctx(it_cur, raw_cur);
  Item it_next = fetch_item(idx + slots);

#pragma unroll
  for (int s = 0; s < STAGES - 1; ++s) issue_loads(cur, min(s, cur.kt_n - 1), s, 0, LPS);
  wait_vmcnt<(STAGES - 2) * LPS>();
  __builtin_amdgcn_s_barrier();
  read_frags(0, 0, 0);

  while (true) {
    const bool has_next = idx + slots < count;
    const Item it_next2 = fetch_item(idx + 2 * slots);
    const Item& it_fill = has_next ? it_next : it_cur;
    const Raw raw_next = fetch_raw(it_fill);      // one more counted load, older than all that follow

#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // refills still inside this item
    const int kt_n = SLICES ? cur.kt_n : KT;   // (every entry has at least STAGES - 1 k-tiles)
    for (int kt = 0; kt + (STAGES - 1) < kt_n; ++kt) k_iteration(cur, kt + STAGES - 1);
    // The source rows of the next item were requested before those iterations; loads
    // complete in order, so they have landed once enough younger loads have been
    // waited for, which the iterations above guarantee only if there were enough.
    if (GATED && KT < 2 * (STAGES - 1)) wait_vmcnt<0>();
    // refills that already belong to the next item (for the last item: a harmless
    // re-fetch of this item's first k-tiles, which keeps the vmcnt bookkeeping uniform)
    const Ctx nxt = make_ctx(it_fill, raw_next);
    for (int kt = max(kt_n - (STAGES - 1), 0); kt < kt_n; ++kt)
      k_iteration(nxt, min(kt + (STAGES - 1) - kt_n, (SLICES ? nxt.kt_n : KT) - 1));

    epilogue(cur);
    if (!has_next) break;
    cur = nxt;
    it_cur = it_next;
    it_next = it_next2;
    idx += slots;
  }
  wait_vmcnt<0>();   // the last refills must land before this LDS allocation is released
#endif  // __HIP_DEVICE_COMPILE__
}

// Launches the schedule builder for the two GEMMs of the FFN of a batch of T tokens.
static inline prism_status launch_build_schedules(const prism_layer_desc& d,
                                                  const int32_t* local_offsets, int T,
                                                  int32_t* tiles, hipStream_t st) {
  SchedParams p0, p1;
  ffn_sched_params(d, T, tiles, &p0, &p1);
  hipLaunchKernelGGL(build_schedule_kernel, dim3(2), dim3(512), 0, st, local_offsets, d.n_experts,
                     d.n_shared, T, T * d.top_k, p0, p1);
  PRISM_CHECK_LAUNCH();
  return PRISM_OK;
}

// LDS of one workgroup of a tile shape, and how many of them a CU holds.
template <int BM, int BN, int WGN, int BK, int STAGES, bool GATED, bool SPLITK>
constexpr int gemm_lds_bytes() {
  return STAGES * (BM + BN) * BK * 2 + (GATED ? 4096 : 0) +           // ring + source-row slots
         (staged_store<BN / WGN, GATED, SPLITK>() ? 4 * kStripBytes : 0);   // + strips
}
constexpr int kCusPerXcd = 32;
template <int BM, int BN, int WGN, int BK, int STAGES, bool GATED, bool SPLITK>
constexpr int gemm_wgs_per_xcd() {
  return kCusPerXcd * ((160 * 1024) / gemm_lds_bytes<BM, BN, WGN, BK, STAGES, GATED, SPLITK>());
}

// capacity: items per XCD list (sched_capacity).  The grid holds as many workgroups
// as fit on the machine at once (each then walks several items), or one per item.
template <int BM, int BN, int WGM, int WGN, int BK, int STAGES, bool GATED, bool SPLITK = false,
          bool ROTATE = false, bool STREAM_B = false, bool SLICES = false>
prism_status launch_gemm(const GemmArgs& args, int capacity, hipStream_t st, int max_slots = 0) {
  constexpr int smem = gemm_lds_bytes<BM, BN, WGN, BK, STAGES, GATED, SPLITK>();
  static_assert(smem <= 160 * 1024, "LDS per workgroup");
  auto kernel = grouped_gemm_kernel<BM, BN, WGM, WGN, BK, STAGES, GATED, SPLITK, ROTATE, STREAM_B, SLICES>;
  static LdsLimitOnce lds_limit;   // one per instantiation
  if (!raise_lds_limit(lds_limit, (const void*)kernel, smem)) return PRISM_ERR_LAUNCH;
  if (capacity <= 0) return PRISM_OK;
  // persistent workgroups per XCD: as many as are resident at once (SPLITK: the schedule says
  // how they pair up, so the launch is never cut down to the list length)
  int slots = gemm_wgs_per_xcd<BM, BN, WGN, BK, STAGES, GATED, SPLITK>();
  if (max_slots > 0) slots = max_slots;
  if (!SPLITK && slots > capacity) slots = capacity;
  hipLaunchKernelGGL(kernel, dim3((unsigned)(slots * kXcds)), dim3(kGemmThreads), smem, st, args);
  PRISM_CHECK_LAUNCH();
  return PRISM_OK;
}

}  // namespace gg
}  // namespace prism
#endif  // PRISM_GROUPED_GEMM_H_
