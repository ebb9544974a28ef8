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

template <bool USE_LDS>
__global__ __launch_bounds__(256) void transition_kernel(const int32_t* __restrict__ idx_l, const int32_t* __restrict__ idx_l1,
                                                         int T, int k_l, int k_l1, int use_l, int use_l1, int E_l, int E_l1,
                                                         int copies, int pairs_of_two, unsigned long long* __restrict__ R) {
    extern __shared__ int hist[];
    const int bins = E_l * E_l1;
    const int my_copy = threadIdx.x & (copies - 1);
    if (USE_LDS) {
        for (int b = threadIdx.x; b < bins * copies; b += 256) hist[b] = 0;
        __syncthreads();
    }
    const long long stride = (long long)gridDim.x * 256;
    auto count = [&](int e1, int e2) {
        if ((unsigned)e1 >= (unsigned)E_l || (unsigned)e2 >= (unsigned)E_l1) return;
        if (USE_LDS) atomicAdd(&hist[(e1 * E_l1 + e2) * copies + my_copy], 1);
        else atomicAdd(&R[e1 * E_l1 + e2], 1ull);
    };
    long long t = (long long)blockIdx.x * 256 + threadIdx.x;
    if (pairs_of_two) {
        // top-2 in both layers (the usual case) and 8-byte aligned arrays: 8-byte loads, four tokens per thread in flight at a time
        const int2* a2 = reinterpret_cast<const int2*>(idx_l);
        const int2* b2 = reinterpret_cast<const int2*>(idx_l1);
        for (; t + 3 * stride < T; t += 4 * stride) {
            int2 a[4], b[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) { a[u] = a2[t + u * stride]; b[u] = b2[t + u * stride]; }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                count(a[u].x, b[u].x);
                if (use_l1 > 1) count(a[u].x, b[u].y);
                if (use_l > 1) {
                    count(a[u].y, b[u].x);
                    if (use_l1 > 1) count(a[u].y, b[u].y);
                }
            }
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
        for (int b = threadIdx.x; b < bins; b += 256) {
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
    long long want = ((long long)T + 256 * tpt - 1) / (256 * tpt);
    const unsigned grid = (unsigned)(want < 1 ? 1 : (want > 512 ? 512 : want));
    int copies = 1;
    while (copies < 32 && bins * copies * 2 <= kLdsBins) copies *= 2;
    LaunchTimer timer(MOE_K_TRANSITION, s);
    if (bins <= kLdsBins)
        hipLaunchKernelGGL(transition_kernel<true>, dim3(grid), dim3(256), bins * copies * sizeof(int), s, idx_l, idx_l1, T, k_l, k_l1,
                           use_l, use_l1, E_l, E_l1, copies, pairs_of_two, (unsigned long long*)R);
    else
        hipLaunchKernelGGL(transition_kernel<false>, dim3(grid), dim3(256), 0, s, idx_l, idx_l1, T, k_l, k_l1, use_l, use_l1, E_l, E_l1, 1,
                           pairs_of_two, (unsigned long long*)R);
    return check_launch("moe_transition_counts launch");
}

}  // namespace moe
