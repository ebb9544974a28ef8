// moe_transition_counts: the layer-l -> layer-(l+1) routing history table
// R_{e1,e2,l} of the paper (Section 2.4; Section 3.1 "Token Routing Profile";
// ILP 2 inputs).
//
// Each workgroup keeps private int32 copies of the E_l x E_l1 table in LDS
// (as many copies as fit, up to 32, selected by lane so that lanes hitting the
// same hot bin mostly land on different addresses), counts its tokens'
// k_l * k_l1 expert pairs (or only its top-1 pair) there with LDS atomics, and then adds its non-zero
// bins to the int64 table in memory.  Integer adds commute, so the result is
// exact whatever the order.  Tables too large for LDS are counted straight
// into memory.
#include "common.h"

namespace moe {

constexpr int kLdsBins = 12288;          // 48 KB of int32 per workgroup
constexpr int kTokPerThread = 4;

template <bool USE_LDS, int kTransThreads>
__global__ __launch_bounds__(kTransThreads) void transition_kernel(const int32_t* __restrict__ idx_l, const int32_t* __restrict__ idx_l1,
                                                         int T, int k_l, int k_l1, int use_l, int use_l1, int E_l, int E_l1,
                                                         int copies, int pairs_of_two, unsigned long long* __restrict__ R) {
    extern __shared__ int hist[];
    const int bins = E_l * E_l1;
    const int my_copy = threadIdx.x & (copies - 1);
    if (USE_LDS) {
        for (int b = threadIdx.x; b < bins * copies; b += kTransThreads) hist[b] = 0;
        __syncthreads();
    }
    const long long stride = (long long)gridDim.x * kTransThreads;
    auto count = [&](int e1, int e2) {
        if ((unsigned)e1 >= (unsigned)E_l || (unsigned)e2 >= (unsigned)E_l1) return;
        if (USE_LDS) atomicAdd(&hist[(e1 * E_l1 + e2) * copies + my_copy], 1);
        else atomicAdd(&R[e1 * E_l1 + e2], 1ull);
    };
    long long t = (long long)blockIdx.x * kTransThreads + threadIdx.x;
    if (pairs_of_two) {
        // top-2 in both layers (the usual case) and 8-byte aligned arrays: 8-byte loads, eight tokens per thread in flight at a time
        const int2* a2 = reinterpret_cast<const int2*>(idx_l);
        const int2* b2 = reinterpret_cast<const int2*>(idx_l1);
        auto count_pairs = [&](int2 a, int2 b) {
            count(a.x, b.x);
            if (use_l1 > 1) count(a.x, b.y);
            if (use_l > 1) {
                count(a.y, b.x);
                if (use_l1 > 1) count(a.y, b.y);
            }
        };
        for (; t + 7 * stride < T; t += 8 * stride) {
            int2 a[8], b[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) { a[u] = a2[t + u * stride]; b[u] = b2[t + u * stride]; }
#pragma unroll
            for (int u = 0; u < 8; ++u) count_pairs(a[u], b[u]);
        }
        for (; t < T; t += 4 * stride) {                   // the tail: slots past the batch hold -1, which count() ignores
            int2 a[4], b[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const bool in = t + u * stride < T;
                a[u] = in ? a2[t + u * stride] : make_int2(-1, -1);
                b[u] = in ? b2[t + u * stride] : make_int2(-1, -1);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) count_pairs(a[u], b[u]);
        }
    }
    if (use_l <= 8 && use_l1 <= 8) {
        // up to 8 x 8 pairs per token: both index lists go to registers first (all loads in flight together;
        // slots past use_l / use_l1 hold -1, which count() ignores)
        for (; t < T; t += stride) {
            int e1s[8], e2s[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                e1s[j] = j < use_l ? idx_l[t * k_l + j] : -1;
                e2s[j] = j < use_l1 ? idx_l1[t * k_l1 + j] : -1;
            }
#pragma unroll
            for (int j1 = 0; j1 < 8; ++j1) {
                if (j1 >= use_l) break;
#pragma unroll
                for (int j2 = 0; j2 < 8; ++j2) count(e1s[j1], e2s[j2]);
            }
        }
    }
    for (; t < T; t += stride) {
        for (int j1 = 0; j1 < use_l; ++j1) {              // the first use_l of the k_l slots (all of them, or the top-1)
            const int e1 = idx_l[t * k_l + j1];
            for (int j2 = 0; j2 < use_l1; ++j2)
                count(e1, idx_l1[t * k_l1 + j2]);         // re-read per pair: it stays in L1, and no private array is needed
        }
    }
    if (USE_LDS) {
        __syncthreads();
        for (int b = threadIdx.x; b < bins; b += kTransThreads) {
            int c = 0;
            for (int i = 0; i < copies; ++i) c += hist[b * copies + ((i + threadIdx.x) & (copies - 1))];
            if (c) atomicAdd(&R[b], (unsigned long long)c);
        }
    }
}

int launch_transition(const int32_t* idx_l, const int32_t* idx_l1, int T, int k_l, int k_l1, int E_l, int E_l1,
                      bool top1_only, int64_t* R, hipStream_t s) {
    const int use_l = top1_only ? 1 : k_l, use_l1 = top1_only ? 1 : k_l1;
    const int pairs_of_two = k_l == 2 && k_l1 == 2 && ((uintptr_t)idx_l & 7) == 0 && ((uintptr_t)idx_l1 & 7) == 0;
    const int bins = E_l * E_l1;
    // tokens per thread: four for top-2 x top-2, one when a token has 16 pairs or more
    const int pairs = use_l * use_l1;
    const int tpt = pairs >= 16 ? 1 : (pairs >= 8 ? 2 : kTokPerThread);
    // Every workgroup ends with one global atomic per non-zero bin, all workgroups on the same few lines: at most 512
    // workgroups of 256 threads; batches that would need more run 256 workgroups of 1024 threads instead (as many
    // threads, half the atomics: 24.7 -> 18.5 us at 4 M tokens, top-2 x top-2), which a small batch cannot afford
    // (one large workgroup starts more slowly than four small ones)
    const long long want256 = ((long long)T + 256 * tpt - 1) / (256 * tpt);
    const bool large = want256 > 512;
    const long long want = large ? ((long long)T + 1024 * tpt - 1) / (1024 * tpt) : want256;
    const long long cap = large ? 256 : 512;
    const unsigned grid = (unsigned)(want < 1 ? 1 : (want > cap ? cap : want));
    int copies = 1;
    while (copies < 32 && bins * copies * 2 <= kLdsBins) copies *= 2;
    LaunchTimer timer(MOE_K_TRANSITION, s);
#define MOE_LAUNCH_TRANSITION(LDS, THREADS, SMEM, COPIES)                                                                          \
    hipLaunchKernelGGL((transition_kernel<LDS, THREADS>), dim3(grid), dim3(THREADS), SMEM, s, idx_l, idx_l1, T, k_l, k_l1, use_l, use_l1, \
                       E_l, E_l1, COPIES, pairs_of_two, (unsigned long long*)R)
    if (bins <= kLdsBins) {
        if (large) MOE_LAUNCH_TRANSITION(true, 1024, bins * copies * sizeof(int), copies);
        else MOE_LAUNCH_TRANSITION(true, 256, bins * copies * sizeof(int), copies);
    } else {
        if (large) MOE_LAUNCH_TRANSITION(false, 1024, 0, 1);
        else MOE_LAUNCH_TRANSITION(false, 256, 0, 1);
    }
#undef MOE_LAUNCH_TRANSITION
    return check_launch("moe_transition_counts launch");
}

}  // namespace moe
