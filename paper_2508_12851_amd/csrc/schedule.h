// Work schedule of the grouped GEMMs: layout, the device-side builder and the
// host-side size bounds.
#ifndef PRISM_SCHEDULE_H_
#define PRISM_SCHEDULE_H_

#include "prism_internal.h"

namespace prism {
namespace gg {

constexpr int kMaxGroups = PRISM_MAX_EXPERTS + PRISM_MAX_SHARED;
constexpr int kXcds = 8;
constexpr int kSchedHeader = 32;     // ints
constexpr int kItemInts = 8;         // ints per work item
constexpr int kMaxSlices = 16;       // contraction slices of one sliced item, at most
constexpr int kMinSliceKt = 8;       // k-tiles of one slice, at least
constexpr int kSliceSlots = 32;      // workgroups per XCD that sliced lists are cut for
constexpr int kReduceInts = 8;       // ints per entry of the list of sliced items

// Schedule memory (int32):
//   [0] n_mtiles  [1] capacity of one XCD list (entries)  [2] contraction splits (see "Splits")
//   [4 + x] items in the list of XCD x
//   [20 + x] slice entries of XCD x (they occupy the last kSliceSlots places of its list)
//   then, from int kSchedHeader on, for schedules that deal their items to the XCDs one by
//   one (interleave): one line of 4 ints per row tile, [0]..[3] as below -- item number seq is
//   row tile seq / (column tiles), column tile seq mod (column tiles), and XCD x runs the items
//   x, x + 8, ...; the kernel works that out itself, which keeps the builder, a serial step on
//   the critical path of a decode layer, from writing a thousand entries --
//   for all other schedules 8 lists of `capacity` entries of 8 ints:
//     [0] group id g (g < E: routed expert g; else shared expert g - E)
//     [1] first row of the row tile in h / y row space
//     [2] rows in the tile (1..BM)
//     [3] first token of the tile for shared experts, -1 for routed ones
//     [4] column tile
//     slice entries only: [5] first k-tile, [6] number of k-tiles, [7] slot of the fp32
//     partial tile the entry writes
//   then 8 x kSliceSlots / 2 entries of 8 ints, the sliced items for the kernel that sums their
//   slices: [0] first row [1] rows [2] column tile [3] first partial slot [4] slices (0: unused)
//
// Last round.  With n items on w workgroups an XCD needs ceil(n / w) rounds, and the last one
// keeps only n mod w workgroups busy for a whole item.  If the caller allows it (slice_kt),
// the items of that round are cut along the contraction into s = floor(w / (n mod w)) slices
// (at most kMaxSlices, each at least kMinSliceKt k-tiles), which are entries of their own:
// the last round then takes 1 / s of an item.  The slice entries are run by a launch of their
// own (one entry per workgroup), each leaving its accumulators as an fp32 partial tile; a
// small kernel adds the slices of a tile in slice order afterwards.
//
// Splits.  The down projection of a batch that is bound by streaming the weights has few
// items (a decode batch of the 4096 x 14336 layer: 32 column tiles per expert that received a
// token), so every item is run by `splits` workgroups, each over its own range of k-tiles,
// leaving fp32 partial sums for a later kernel to add.  How many is decided here, where the
// number of items is known: s workgroups per item leave floor(w / s) item slots among the w
// workgroups of an XCD, the list takes ceil(items / slots) rounds of ceil(k-tiles / s) k-tiles
// each plus a fixed cost per round, and every split writes (and the summing kernel reads) one
// more fp32 copy of all rows; the s with the lowest sum is taken.  (A model in which the
// workgroups of a round share the memory bandwidth, so that a thin last round costs less than a
// full one, was fitted to the same measurements and chose worse: it leaves the 20 items per XCD
// of five hosted experts whole, 109 us against 96 us with three splits.)
//
// Work order.  A group's row tiles are split into equal parts of at most kRectRows.  All
// items -- groups in order, then row parts, then the column tiles of a row part, the row tiles
// of a column running fastest -- form one sequence, and XCD x gets the x-th eighth of it.  So
// the 32 workgroups resident on an XCD work at any time on a rectangle of about 8 row tiles x
// 4 column tiles -- 8 activation tiles and 4 weight tiles for 32 items instead of one of each
// per item -- which is what the XCD's L2 can share among them, and the eight lists have the
// same length to within one item.
// The number of items (row tiles x column tiles) must stay below 2^31, which the int
// capacity of a list already implies.
#ifndef PRISM_RECT_ROWS
#define PRISM_RECT_ROWS 8   // other values: for measurements of the work order (build.py --define)
#endif
constexpr int kRectRows = PRISM_RECT_ROWS;

struct SchedParams {
  int BM;            // row tile
  int n_ntiles;      // column tiles
  int capacity;      // items one XCD list can hold
  int32_t* sched;
  int interleave;    // 1: deal the sequence to the XCDs item by item instead of in eighths
                     // (schedules whose items share nothing: every XCD then reads from all
                     // parts of the weight matrices at any time); the schedule then holds a
                     // table of row tiles instead of item lists
  int slice_kt;      // k-tiles of the contraction if the items of a partly filled last round may be
                     // cut along it (the launch then has kSliceSlots workgroups per XCD); else 0
  // Contraction splits of every item ("Splits" above); split_kt == 0: the items are not split.
  int split_kt;      // k-tiles of the contraction
  int split_max;     // most splits allowed (fp32 copies the partial-sum buffer holds)
  int split_min_kt;  // fewest k-tiles a split may have (the depth of the kernel's ring)
  int split_wgs;     // workgroups per XCD of the launch
  float split_round_kt;   // fixed cost of a round, in k-tiles of one workgroup
  float split_row_kt;     // cost of one more fp32 copy of one row, in k-tiles of one workgroup
};

// Where the list of sliced items starts (ints from the start of the schedule).
__host__ __device__ inline size_t sched_reduce_offset(int capacity) {
  return (size_t)kSchedHeader + (size_t)kXcds * capacity * kItemInts;
}

// Equal split of `count` things into the fewest parts of at most `part_max`: which part
// holds element i, where that part starts and how long it is.
struct PartOf {
  int first, len;
};
__device__ __forceinline__ PartOf part_of(int i, int count, int part_max) {
  const int parts = (count + part_max - 1) / part_max;
  const int base = count / parts, extra = count % parts;     // `extra` parts have base + 1
  const int split = extra * (base + 1);
  if (i < split) {
    const int q = i / (base + 1);
    return PartOf{q * (base + 1), base + 1};
  }
  const int q = (i - split) / base;
  return PartOf{split + q * base, base};
}

// How the last round of an XCD list of n items is cut: its `items` items into `slices` entries
// each (slices == 0: not cut).
struct Slicing {
  int items, slices;
};
__device__ __forceinline__ Slicing slicing_of(int n, int slice_kt) {
  const int left = n % kSliceSlots;
  if (slice_kt <= 0 || left == 0) return Slicing{0, 0};
  int s = kSliceSlots / left;
  s = min(s, min(kMaxSlices, slice_kt / kMinSliceKt));
  return s >= 2 ? Slicing{left, s} : Slicing{0, 0};
}

// Builds NS (1 or 2) schedules of the same row groups side by side; called by every
// thread of a workgroup (any size that is a multiple of 64, at least NS wavefronts).  Inside, only LDS data
// crosses between threads, so the barriers do not wait for the global stores.
// local_offsets (global memory or LDS) may have been written earlier in the same kernel by
// this workgroup (with a barrier in between), hence no __restrict__ on it.
// Several workgroups can share the work: workgroup `part` of `n_parts` writes every
// n_parts-th group of blockDim.x items, part 0 also the header.
template <int NS>
__device__ __forceinline__ void build_schedules_block(const int32_t* local_offsets, int E, int S,
                                                      int T, int A_total,
                                                      const SchedParams (&p)[NS], int part = 0,
                                                      int n_parts = 1) {
  __shared__ int s_rows[kMaxGroups], s_row0[kMaxGroups];
  __shared__ int s_start[NS][kMaxGroups + 1];            // first row tile of group g
  const int G = E + S;
  // p[s] for a thread-dependent s, without indexing the parameter array at run time
  // (that would put it in scratch memory)
  auto pick = [&](int s) { return NS == 1 || s == 0 ? p[0] : p[NS - 1]; };
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
  lds_barrier();
  // Wavefront s prepares schedule s: first row tile of every group (a scan over the groups, 64
  // at a time), the header, and the number of contraction splits -- in parallel over its lanes,
  // because this is a serial step on the critical path of a decode layer.
  const int lane = threadIdx.x & 63;
  if ((int)(threadIdx.x >> 6) < NS) {
    const int s = threadIdx.x >> 6;
    const SchedParams ps = pick(s);
    int run = 0;
    for (int g0 = 0; g0 < G; g0 += 64) {
      const int g = g0 + lane;
      const int rows = g < G ? s_rows[g] : 0;
      const int tiles = (rows + ps.BM - 1) / ps.BM;
      const int incl = wave_inclusive_scan(tiles);
      if (g < G) s_start[s][g] = run + incl - tiles;
      run += __builtin_amdgcn_readlane(incl, 63);
    }
    const int rows_total = s_row0[E - 1] + s_rows[E - 1] + S * T;   // all rows of all groups
    if (lane == 0) s_start[s][G] = run;
    const unsigned total = (unsigned)run * (unsigned)ps.n_ntiles;
    const unsigned per_xcd = (total + kXcds - 1) / kXcds;
    if (part == 0) {
      if (lane == 0) {
        ps.sched[0] = run;
        ps.sched[1] = ps.capacity;
      }
      if (lane < kXcds) {
        const unsigned x = lane;
        unsigned count;
        if (ps.interleave)   // items x, x + 8, ...
          count = total > x ? (total - x + kXcds - 1) / kXcds : 0;
        else                 // every list holds per_xcd items, the last non-empty one the remainder
          count = total > x * per_xcd ? min(per_xcd, total - x * per_xcd) : 0;
        const Slicing sl = slicing_of((int)count, ps.slice_kt);
        ps.sched[4 + x] = (int)count - sl.items;
        ps.sched[20 + x] = sl.items * sl.slices;
      }
      // lane sp - 1 prices sp splits; the cheapest wins, the lower count on ties
      const int sp = lane + 1;
      const int slots = ps.split_wgs / sp;
      float cost = INFINITY;
      if (ps.split_kt > 0 && sp <= min(ps.split_max, 8) && slots >= 1 && ps.split_kt / sp >= ps.split_min_kt) {
        const int rounds = ((int)per_xcd + slots - 1) / slots;   // per_xcd: the longest XCD list
        cost = (float)rounds * ((float)((ps.split_kt + sp - 1) / sp) + ps.split_round_kt) +
               (float)sp * (float)rows_total * ps.split_row_kt;
      }
      static_assert(kDecodeSplits <= 8, "the candidates sit in lanes 0..7");
      int best = sp;
      auto meet = [&](float oc, int ob) {
        if (oc < cost || (oc == cost && ob < best)) {
          cost = oc;
          best = ob;
        }
      };
      meet(row_xor<4>(cost), row_xor<4>(best));
      meet(row_xor<2>(cost), row_xor<2>(best));
      meet(row_xor<1>(cost), row_xor<1>(best));
      if (lane == 0) ps.sched[2] = cost < INFINITY ? best : 1;
    }
  }
  lds_barrier();
#pragma unroll
  for (int s = 0; s < NS; ++s) {
    const int BM = p[s].BM, n_ntiles = p[s].n_ntiles, capacity = p[s].capacity;
    const bool interleave = p[s].interleave != 0;
    const int n_mtiles = s_start[s][G];
    auto group_of_tile = [&](int i) {   // largest g with s_start[g] <= i (skips empty groups)
      int lo = 0, hi = G;               // invariant: s_start[lo] <= i < s_start[hi]
      while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (s_start[s][mid] <= i) lo = mid; else hi = mid;
      }
      return lo;
    };
    const unsigned n_items = (unsigned)n_mtiles * (unsigned)n_ntiles;
    const unsigned per_xcd = (n_items + kXcds - 1) / kXcds;
    if (interleave) {
      // no lists: the kernel derives item seq = tile * n_ntiles + column tile from its position
      // (XCD x takes seq = x, x + 8, ...) and reads the row tile's line of this table
      int4* table = reinterpret_cast<int4*>(p[s].sched + kSchedHeader);
      for (int i = part * blockDim.x + threadIdx.x; i < n_mtiles; i += n_parts * blockDim.x) {
        const int g = group_of_tile(i);
        const int mi = i - s_start[s][g];
        table[i] = int4{g, s_row0[g] + mi * BM, min(BM, s_rows[g] - mi * BM), g < E ? -1 : mi * BM};
      }
      continue;
    }
    for (unsigned w = part * blockDim.x + threadIdx.x; w < n_items; w += n_parts * blockDim.x) {
      const int nt = (int)(w / (unsigned)n_mtiles), i = (int)(w - (unsigned)nt * (unsigned)n_mtiles);
      const int g = group_of_tile(i);
      const int mi = i - s_start[s][g];
      const int m = s_start[s][g + 1] - s_start[s][g];
      // this item's row part (most groups have a single one: no division then)
      const PartOf rp = m <= kRectRows ? PartOf{0, m} : part_of(mi, m, kRectRows);
      // items before it: earlier groups, earlier row parts of its group, earlier columns of its
      // row part (which is the rectangle order: the rectangles of a row part follow each other
      // column by column), earlier rows of its column
      const unsigned seq = (unsigned)(s_start[s][g] + rp.first) * (unsigned)n_ntiles +
                           (unsigned)(nt * rp.len + (mi - rp.first));
      const unsigned x = seq / per_xcd;
      const unsigned pos = seq - x * per_xcd;
      const int4 head = int4{g, s_row0[g] + mi * BM, min(BM, s_rows[g] - mi * BM), g < E ? -1 : mi * BM};
      int4* list = reinterpret_cast<int4*>(p[s].sched + kSchedHeader + (size_t)x * capacity * kItemInts);
      const unsigned in_list = n_items > x * per_xcd ? min(per_xcd, n_items - x * per_xcd) : 0u;
      const Slicing sl = slicing_of((int)in_list, p[s].slice_kt);
      const int first_sliced = (int)in_list - sl.items;
      if ((int)pos < first_sliced || sl.slices == 0) {
        list[2 * pos] = head;
        list[2 * pos + 1] = int4{nt, 0, 0, 0};
      } else {
        // the li-th item of the last round: sl.slices entries, slice after slice, and its line
        // in the list of sliced items
        const int li = (int)pos - first_sliced;
        const int kt_all = p[s].slice_kt;
        for (int c = 0; c < sl.slices; ++c) {
          const int e = capacity - kSliceSlots + li * sl.slices + c;
          const int k0 = (int)((long long)kt_all * c / sl.slices), k1 = (int)((long long)kt_all * (c + 1) / sl.slices);
          list[2 * e] = head;
          list[2 * e + 1] = int4{nt, k0, k1 - k0, (int)x * kSliceSlots + li * sl.slices + c};
        }
        int4* red = reinterpret_cast<int4*>(p[s].sched + sched_reduce_offset(capacity)) +
                    ((size_t)x * (kSliceSlots / 2) + li) * (kReduceInts / 4);
        red[0] = int4{head.y, head.z, nt, (int)x * kSliceSlots + li * sl.slices};
        red[1] = int4{sl.slices, 0, 0, 0};
      }
    }
    // lines of the list of sliced items that this call does not use are marked empty
    if (p[s].slice_kt > 0)
      for (int r = part * blockDim.x + threadIdx.x; r < kXcds * (kSliceSlots / 2); r += n_parts * blockDim.x) {
        const unsigned x = (unsigned)r / (kSliceSlots / 2);
        const int li = r % (kSliceSlots / 2);
        const unsigned in_list = n_items > x * per_xcd ? min(per_xcd, n_items - x * per_xcd) : 0u;
        const Slicing sl = slicing_of((int)in_list, p[s].slice_kt);
        if (li >= sl.items || sl.slices == 0)
          reinterpret_cast<int4*>(p[s].sched + sched_reduce_offset(capacity))[(size_t)r * (kReduceInts / 4) + 1] =
              int4{0, 0, 0, 0};
      }
  }
}

// Upper bound on the number of row tiles for T tokens (host side).
static inline int max_row_tiles(const prism_layer_desc& d, int T, int BM) {
  return T * d.top_k / BM + d.n_experts + d.n_shared * ceil_div(T, BM);
}

// Entries one XCD list must be able to hold: every row tile times its share of the column
// tiles, plus the slices a cut last round adds (at most one entry per workgroup).
static inline int sched_capacity(const prism_layer_desc& d, int T, int BM, int n_ntiles) {
  return max_row_tiles(d, T, BM) * ceil_div(n_ntiles, kXcds) + kSliceSlots;
}

// Parameters of the two schedules of launch_expert_ffn for a bf16 batch of T tokens, which live
// side by side in `tiles` (2 x tile_table_ints): what every kernel that builds them is given.
static inline void ffn_sched_params(const prism_layer_desc& d, int T, int32_t* tiles, SchedParams* p0,
                                    SchedParams* p1) {
  const FfnShapes f = ffn_schedule_shapes(d, T);
  *p0 = SchedParams{f.bm1, f.nt1, sched_capacity(d, T, f.bm1, f.nt1), tiles, f.interleave ? 1 : 0,
                    0, 0, 0, 0, 0, 0.f, 0.f};
  *p1 = SchedParams{f.bm2, f.nt2, sched_capacity(d, T, f.bm2, f.nt2), tiles + tile_table_ints(d, T),
                    f.interleave ? 1 : 0, f.slice_kt2, f.split_kt2, max_splits(d, T), f.split_min_kt2,
                    f.split_wgs2, f.split_round_kt2, f.split_row_kt2};
}

}  // namespace gg
}  // namespace prism
#endif  // PRISM_SCHEDULE_H_
