// Which piece of the grouped GEMM does a workgroup own?  The index arithmetic
// that turns (workgroup id, tile plan) into (expert, rows, column tile, k range)
// for moe_expert_ffn_grouped (paper Section 2.2 / Fig. 2b, the expert FFN over
// ragged per-expert buckets), kept apart from the kernels so that it can also
// be compiled for the host and checked exhaustively there: every
// (bucket, row tile, column tile, k tile) must be owned exactly once.
#pragma once
#include "ffn_plan.h"

namespace moe {

constexpr int kXcds = 8;
constexpr int kMaxSplit = 8;
constexpr int kMinSplitKT = 8;                  // a k part is at least this many k tiles
constexpr int kMinSplitGain = 16;               // k tiles of time a split tail must save to be worth its fix-up
constexpr int kMaxCusPerXcd = 48;               // two fp32 partial-tile slots exist per compute unit, for at most this many

struct WorkItem {
    int expert, row0, rows, nt;
    int kt0, kt1;        // k tile range
    int partial;         // slot of the fp32 partial tile, or -1 for a whole tile
};

struct XcdShare {
    int q, rem;          // column tiles owned outright by every XCD; left-over column tiles (NT % 8)
    long long main;      // tiles of the owned columns: row tiles x q
    long long rem_begin; // this XCD's first tile in the list of left-over-column tiles
    int full;            // tiles run whole
    int tail;            // tiles run in `split` k parts each
    int split;
};

// The tiles of XCD x.  Every XCD owns NT / 8 column tiles of every expert outright, so each weight
// panel is fetched through one L2 only and all XCDs get the same mix of large and small experts; the
// tiles of the NT % 8 left-over column tiles are dealt to the XCDs in equal contiguous ranges.
__host__ __device__ __forceinline__ XcdShare xcd_share(int MT, int NT, int x, int KT, int cus_per_xcd, bool allow_split) {
    XcdShare s;
    s.q = NT / kXcds;
    s.rem = NT - s.q * kXcds;
    s.main = (long long)MT * s.q;
    const long long rem_total = (long long)MT * s.rem;
    const long long chunk = (rem_total + kXcds - 1) / kXcds;
    s.rem_begin = (long long)x * chunk;
    long long rcnt = rem_total - s.rem_begin;
    rcnt = rcnt < 0 ? 0 : (rcnt > chunk ? chunk : rcnt);
    const long long cnt = s.main + rcnt;
    s.full = (int)cnt;
    s.tail = 0;
    s.split = 1;
    if (allow_split) {
        // r tiles in the last round: cut each into sp k parts so that the r * sp parts (at most two per
        // compute unit: that many partial tiles exist) fill the compute units in as few, short rounds as
        // possible; taken when the tail then lasts at most three quarters of a whole round
        const int r = (int)(cnt % cus_per_xcd);
        if (r > 0) {
            int best = 1, best_num = 1, best_den = 1;           // tail time = best_num / best_den rounds
            for (int sp = 2; sp <= kMaxSplit; ++sp) {
                if (r * sp > 2 * cus_per_xcd || KT / sp < kMinSplitKT) break;
                const int rounds = (r * sp + cus_per_xcd - 1) / cus_per_xcd;
                if (rounds * best_den < best_num * sp) { best = sp; best_num = rounds; best_den = sp; }
            }
            // ... and saves at least kMinSplitGain k tiles of time: the partial tiles and the fix-up launch cost
            // about that much, so short reductions (the many-expert layer: 22 k tiles) run their tail whole
            if (best > 1 && 4 * best_num <= 3 * best_den && (best_den - best_num) * KT >= kMinSplitGain * best_den) {
                s.full = (int)cnt - r;
                s.tail = r;
                s.split = best;
            }
        }
    }
    return s;
}

// Tile order inside one expert: row tiles are taken in chunks of `row_chunk`, and within a chunk the
// column tile advances before the chunk does, so the ~32 tiles that run together on an XCD form a
// row_chunk x (32 / row_chunk) block that streams row_chunk activation panels and 32 / row_chunk
// weight panels through that XCD's L2 (a large expert would otherwise run as a 32 x 1 strip that
// re-reads its activations once per column tile).  Every chunk re-reads the expert's weights, which
// come from DRAM, while re-read activations come from the Infinity Cache as long as they fit there:
// chunks of 8 row tiles then, of 4 (the split that moves the fewest bytes) for larger batches.
constexpr size_t kActivationsFitCache = (size_t)128 << 20;
static inline int row_chunk_for(size_t activation_bytes) { return activation_bytes <= kActivationsFitCache ? 8 : 4; }

// tile number `tile` of a list that walks NT column tiles of every listed bucket
__host__ __device__ __forceinline__ void locate_tile(const int32_t* __restrict__ plan, const int32_t* __restrict__ prefix, int NT,
                                                     long long tile, int BM, int row_chunk, WorkItem& w) {
    const int n_exp = plan[0];
    int i = 0;
    while (i + 1 < n_exp && (long long)prefix[i + 1] * NT <= tile) ++i;
    const int mt_e = prefix[i + 1] - prefix[i];
    const int rem = (int)(tile - (long long)prefix[i] * NT);
    const int per_chunk = row_chunk * NT;
    const int q = rem / per_chunk;                       // chunk of row tiles
    const int in_chunk = rem - q * per_chunk;
    const int left = mt_e - q * row_chunk;
    const int rows_here = row_chunk < left ? row_chunk : left;
    w.nt = in_chunk / rows_here;
    const int mt = q * row_chunk + (in_chunk - w.nt * rows_here);
    w.expert = plan[kPlanExpert + i];
    w.row0 = plan[kPlanStart + i] + mt * BM;
    const int rows_left = plan[kPlanCount + i] - mt * BM;
    w.rows = BM < rows_left ? BM : rows_left;
}

// tile `idx` of XCD x's list: first the tiles of its own column tiles, then its share of the left-over ones
__host__ __device__ __forceinline__ void locate_xcd_tile(const int32_t* __restrict__ plan, const int32_t* __restrict__ prefix,
                                                         const XcdShare& sh, int x, int idx, int BM, int row_chunk, WorkItem& w) {
    if (idx < sh.main) {
        locate_tile(plan, prefix, sh.q, idx, BM, row_chunk, w);
        w.nt += x * sh.q;
    } else {
        locate_tile(plan, prefix, sh.rem, sh.rem_begin + (idx - sh.main), BM, row_chunk, w);
        w.nt += kXcds * sh.q;
    }
}

// The work of workgroup `block` of a GEMM launch (blocks are dealt round-robin to the XCDs by the hardware:
// XCD = block % 8, and `slot` = block / 8 counts within the XCD): a whole tile, or one k part of a tail tile
// with its partial-tile slot.  False when the launch holds more workgroups than this XCD has work.
__host__ __device__ __forceinline__ bool workgroup_item(const int32_t* __restrict__ plan, const int32_t* __restrict__ prefix,
                                                        int NT, int KT, int BM, unsigned block, int cus_per_xcd, int row_chunk,
                                                        bool allow_split, WorkItem& w) {
    const int x = (int)(block % kXcds), slot = (int)(block / kXcds);
    const XcdShare sh = xcd_share(prefix[plan[0]], NT, x, KT, cus_per_xcd, allow_split);
    if (slot >= sh.full + sh.tail * sh.split) return false;
    if (slot < sh.full) {
        locate_xcd_tile(plan, prefix, sh, x, slot, BM, row_chunk, w);
        w.kt0 = 0; w.kt1 = KT; w.partial = -1;
    } else {
        const int j = slot - sh.full;
        const int part = j % sh.split;
        locate_xcd_tile(plan, prefix, sh, x, sh.full + j / sh.split, BM, row_chunk, w);
        w.kt0 = (int)((long long)part * KT / sh.split);
        w.kt1 = (int)((long long)(part + 1) * KT / sh.split);
        w.partial = x * 2 * cus_per_xcd + j;
    }
    return true;
}

// Tail tile q of XCD x, for the fix-up that adds its k parts: the tile, the slot of its first partial tile
// and the number of parts (their slots follow each other).  False when the XCD has fewer tail tiles.
__host__ __device__ __forceinline__ bool fixup_item(const int32_t* __restrict__ plan, const int32_t* __restrict__ prefix, int NT,
                                                    int KT, int BM, int x, int q, int cus_per_xcd, int row_chunk, WorkItem& w,
                                                    int& first_partial, int& parts) {
    const XcdShare sh = xcd_share(prefix[plan[0]], NT, x, KT, cus_per_xcd, true);
    if (q >= sh.tail) return false;
    locate_xcd_tile(plan, prefix, sh, x, sh.full + q, BM, row_chunk, w);
    first_partial = x * 2 * cus_per_xcd + q * sh.split;
    parts = sh.split;
    return true;
}

// Workgroups a GEMM launch needs for N rows in E buckets, whatever the bucket sizes (only the device knows
// them): the sum of ceil(n_e / bm) never exceeds N / bm + min(E, N), and the split tail adds at most two
// parts per compute unit.
static inline long long ffn_grid(int N, int E, long long nt, int bm, bool split, int cus_per_xcd) {
    const long long mt_max = (N + bm - 1) / bm + (E < N ? E : N);
    const long long per_xcd = mt_max * (nt / kXcds) + (mt_max * (nt % kXcds) + kXcds - 1) / kXcds;
    return (long long)kXcds * (per_xcd + (split ? 2 * cus_per_xcd : 0));
}

}  // namespace moe
