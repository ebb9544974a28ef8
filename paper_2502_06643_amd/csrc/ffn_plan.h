// Tile plan of the grouped expert FFN, built on the device from expert_counts
// so that no bucket size ever travels to the host.
//
// The plan lists the experts resident on local_gpu that received at least one
// route (or, on the receiving side of the all-to-all, the (source GPU, expert)
// segments of the receive buffer, each naming the expert whose weights it
// uses), largest bucket first (ties: lower expert id), with sanitised bucket
// bounds and, for up to two row-tile heights, the exclusive prefix of their
// row-tile counts.  A GEMM workgroup turns a global row-tile index into
// (expert, first row, row count) by scanning that prefix.
#pragma once
#include "common.h"

namespace moe {

constexpr int kPlanHeader = 16;
constexpr int kPlanExpert = kPlanHeader;                       // [256] expert id
constexpr int kPlanStart = kPlanExpert + MOE_MAX_EXPERTS;      // [256] first row
constexpr int kPlanCount = kPlanStart + MOE_MAX_EXPERTS;       // [256] rows
constexpr int kPlanTiles0 = kPlanCount + MOE_MAX_EXPERTS;      // [257] prefix for tile height bm0
constexpr int kPlanTiles1 = kPlanTiles0 + MOE_MAX_EXPERTS + 4; // [257] prefix for tile height bm1
constexpr int kPlanInts = kPlanTiles1 + MOE_MAX_EXPERTS + 4;
static_assert(kPlanInts * sizeof(int32_t) <= kPlanBytes, "plan area too small");
// header: [0] number of listed experts, [1] total row tiles (bm0), [2] total row tiles (bm1),
//         [3] which of the two tile heights the bf16 GEMMs use: 0 = bm0, 1 = bm1 (see `choice`)

// E groups of rows (counts/starts); group g multiplies with the weights of expert group_expert[g]
// (g itself when group_expert is NULL), of which there are n_weights; placement may be NULL when
// local_gpu < 0.
// choice: 0 or 1 fixes header [3]; -1 lets the device decide from the listed buckets: bm0 when they hold
// at least kLargeBucketRows rows on average, else bm1.
constexpr int kLargeBucketRows = 544;     // measured crossover at the Mixtral shape: 512 rows per bucket favour 256-row tiles by 1 %, 640 favour 384 by 5 %
int launch_ffn_plan(const int32_t* counts, const int32_t* starts, const int32_t* placement, int local_gpu,
                    const int32_t* group_expert, int n_weights, int E, int N, int bm0, int bm1, int choice, int32_t* plan,
                    hipStream_t s);

struct RowTile { int expert; int row0; int rows; };

// Which expert does global row tile `mt` belong to?  `prefix` is one of the two
// prefix arrays of the plan.  Returns false when mt is past the last tile.
__device__ __forceinline__ bool find_row_tile(const int32_t* __restrict__ plan, const int32_t* __restrict__ prefix,
                                              int mt, int bm, RowTile& out) {
    const int n = plan[0];
    if (mt >= prefix[n]) return false;
    int i = 0;
    while (i + 1 < n && prefix[i + 1] <= mt) ++i;
    const int r0 = (mt - prefix[i]) * bm;
    out.expert = plan[kPlanExpert + i];
    out.row0 = plan[kPlanStart + i] + r0;
    const int left = plan[kPlanCount + i] - r0;
    out.rows = left < bm ? left : bm;
    return true;
}

}  // namespace moe
