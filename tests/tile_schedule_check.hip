// Host-side exhaustive check of the grouped GEMM's work distribution (csrc/ffn_tiles.h): for random tile plans
// and launch shapes, walk every workgroup id of the launch exactly as the kernels do and verify that every
// (bucket, row tile, column tile, k tile) is owned exactly once, that partial-tile slots are unique and inside
// their XCD's range, that the fix-up finds exactly the split tiles with their parts in k order, and that the
// grid the host launches is large enough.  Runs on the CPU: no HIP call is made.
// Built and run by tests/test_tile_schedule.py.
#include "ffn_tiles.h"

#include <cstdio>
#include <cstdlib>
#include <map>
#include <random>
#include <tuple>
#include <vector>

using namespace moe;

#define CHECK(cond, ...)                                                            \
    do {                                                                            \
        if (!(cond)) {                                                              \
            std::printf("FAILED %s (line %d): ", #cond, __LINE__);                  \
            std::printf(__VA_ARGS__);                                               \
            std::printf("\n");                                                      \
            return 1;                                                               \
        }                                                                           \
    } while (0)

struct Part { int bucket, mt, nt, kt0, kt1; };

static int check_case(std::mt19937& rng, long long& units) {
    const int bms[2] = {256, 384};
    const int nts[10] = {1, 2, 5, 8, 11, 16, 23, 32, 57, 112};
    const int kts[8] = {4, 9, 22, 32, 64, 100, 224, 448};
    const int cpxs[4] = {32, 38, 48, 4};
    const int BM = bms[rng() % 2], NT = nts[rng() % 10], KT = kts[rng() % 8], cpx = cpxs[rng() % 4];
    const int row_chunk = (rng() % 2) ? 8 : 4;
    const bool split = rng() % 2;
    const int n = 1 + (int)(rng() % ((rng() % 8 == 0) ? 256 : 12));
    std::vector<int32_t> plan(kPlanInts, 0);
    std::vector<int> start(n), count(n), tiles(n);
    long long N = 0;
    for (int i = 0; i < n; ++i) {
        const int kind = rng() % 4;
        count[i] = kind == 0 ? 1 + rng() % 40 : (kind == 1 ? 1 + rng() % 400 : (kind == 2 ? 1 + rng() % 3000 : BM * (1 + rng() % 4)));
        if (n > 64) count[i] = 1 + rng() % 300;
        start[i] = (int)N + (int)(rng() % 3);            // gaps between buckets are allowed
        N = start[i] + count[i];
        tiles[i] = (count[i] + BM - 1) / BM;
    }
    plan[0] = n;
    int32_t* prefix = plan.data() + kPlanTiles0;
    int mt_total = 0;
    for (int i = 0; i < n; ++i) {
        plan[kPlanExpert + i] = 1000 + i;                 // any id: the check maps it back
        plan[kPlanStart + i] = start[i];
        plan[kPlanCount + i] = count[i];
        prefix[i] = mt_total;
        mt_total += tiles[i];
    }
    prefix[n] = mt_total;

    const long long grid = ffn_grid((int)N, n, NT, BM, split, cpx);
    CHECK(grid > 0 && grid < (1ll << 31), "grid %lld", grid);
    std::map<std::tuple<int, int, int>, std::vector<char>> covered;
    std::map<int, Part> partial_of;
    long long active = 0;
    for (long long block = 0; block < grid + 64; ++block) {      // a few ids past the grid must find no work either
        WorkItem w;
        if (!workgroup_item(plan.data(), prefix, NT, KT, BM, (unsigned)block, cpx, row_chunk, split, w)) continue;
        CHECK(block < grid, "work at block %lld beyond the launched grid %lld (BM %d NT %d KT %d cpx %d n %d split %d)", block, grid, BM, NT, KT, cpx, n, (int)split);
        ++active;
        const int i = w.expert - 1000;
        CHECK(i >= 0 && i < n, "expert %d", w.expert);
        const int off = w.row0 - start[i];
        CHECK(off >= 0 && off % BM == 0, "row0 %d of bucket %d", w.row0, i);
        const int mt = off / BM;
        CHECK(mt < tiles[i], "row tile %d of %d", mt, tiles[i]);
        const int want_rows = count[i] - mt * BM < BM ? count[i] - mt * BM : BM;
        CHECK(w.rows == want_rows && w.rows > 0, "rows %d, want %d", w.rows, want_rows);
        CHECK(w.nt >= 0 && w.nt < NT, "column tile %d of %d", w.nt, NT);
        CHECK(0 <= w.kt0 && w.kt0 < w.kt1 && w.kt1 <= KT, "k range %d..%d of %d", w.kt0, w.kt1, KT);
        const int x = (int)(block % kXcds);
        if (w.partial < 0) {
            CHECK(w.kt0 == 0 && w.kt1 == KT, "a whole tile with k range %d..%d", w.kt0, w.kt1);
        } else {
            CHECK(split, "partial tile without a split launch");
            CHECK(w.partial >= x * 2 * cpx && w.partial < (x + 1) * 2 * cpx, "slot %d outside XCD %d's range", w.partial, x);
            CHECK(!partial_of.count(w.partial), "slot %d used twice", w.partial);
            CHECK(w.kt1 - w.kt0 >= kMinSplitKT, "k part of %d tiles", w.kt1 - w.kt0);
            partial_of[w.partial] = Part{i, mt, w.nt, w.kt0, w.kt1};
        }
        auto& c = covered[std::make_tuple(i, mt, w.nt)];
        if (c.empty()) c.assign(KT, 0);
        for (int kt = w.kt0; kt < w.kt1; ++kt) {
            CHECK(!c[kt], "k tile %d of (bucket %d, row tile %d, column tile %d) owned twice", kt, i, mt, w.nt);
            c[kt] = 1;
            ++units;
        }
    }
    for (int i = 0; i < n; ++i)
        for (int mt = 0; mt < tiles[i]; ++mt)
            for (int nt = 0; nt < NT; ++nt) {
                auto it = covered.find(std::make_tuple(i, mt, nt));
                CHECK(it != covered.end(), "tile (bucket %d, row tile %d, column tile %d) has no owner (BM %d NT %d KT %d cpx %d n %d split %d)", i, mt, nt, BM, NT, KT, cpx, n, (int)split);
                for (int kt = 0; kt < KT; ++kt) CHECK(it->second[kt], "k tile %d of (%d, %d, %d) has no owner", kt, i, mt, nt);
            }
    CHECK((long long)covered.size() == (long long)mt_total * NT, "%zu tiles owned, %lld exist", covered.size(), (long long)mt_total * NT);

    // the fix-up: every split tile exactly once, its parts in consecutive slots and in k order from 0 to KT
    size_t parts_seen = 0;
    std::map<std::tuple<int, int, int>, int> fixed;
    for (int x = 0; x < kXcds; ++x)
        for (int q = 0; q < cpx; ++q) {                  // the host launches cpx fix-up tiles per XCD
            WorkItem w;
            int first = -1, parts = 0;
            if (!fixup_item(plan.data(), prefix, NT, KT, BM, x, q, cpx, row_chunk, w, first, parts)) continue;
            CHECK(split || partial_of.empty(), "fix-up work although nothing was split");
            if (!split) continue;                        // a launch without split never runs the fix-up's result: its tiles were written whole
            const int i = w.expert - 1000, mt = (w.row0 - start[i]) / BM;
            CHECK(++fixed[std::make_tuple(i, mt, w.nt)] == 1, "tile fixed up twice");
            int at = 0;
            for (int p = 0; p < parts; ++p) {
                auto it = partial_of.find(first + p);
                CHECK(it != partial_of.end(), "fix-up reads slot %d that nobody wrote", first + p);
                const Part& pt = it->second;
                CHECK(pt.bucket == i && pt.mt == mt && pt.nt == w.nt, "slot %d belongs to another tile", first + p);
                CHECK(pt.kt0 == at, "parts out of k order");
                at = pt.kt1;
                ++parts_seen;
            }
            CHECK(at == KT, "parts end at k tile %d of %d", at, KT);
        }
    if (split) CHECK(parts_seen == partial_of.size(), "%zu parts fixed up, %zu written", parts_seen, partial_of.size());
    (void)active;
    return 0;
}

int main(int argc, char** argv) {
    const int cases = argc > 1 ? std::atoi(argv[1]) : 2000;
    std::mt19937 rng(20250209);
    long long units = 0;
    for (int c = 0; c < cases; ++c)
        if (check_case(rng, units)) {
            std::printf("case %d\n", c);
            return 1;
        }
    std::printf("ok: %d launches, %lld k tiles owned exactly once\n", cases, units);
    return 0;
}
