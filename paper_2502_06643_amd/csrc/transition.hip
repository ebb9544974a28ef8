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
                                                         int copies, unsigned long long* __restrict__ R) {
    extern __shared__ int hist[];
    const int bins = E_l * E_l1;
    const int my_copy = threadIdx.x & (copies - 1);
    if (USE_LDS) {
        for (int b = threadIdx.x; b < bins * copies; b += 256) hist[b] = 0;
        __syncthreads();
    }
    const long long stride = (long long)gridDim.x * 256;
    for (long long t = (long long)blockIdx.x * 256 + threadIdx.x; t < T; t += stride) {
        for (int j1 = 0; j1 < use_l; ++j1) {              // the first use_l of the k_l slots (all of them, or the top-1)
            const int e1 = idx_l[t * k_l + j1];
            if ((unsigned)e1 >= (unsigned)E_l) continue;
            for (int j2 = 0; j2 < use_l1; ++j2) {
                const int e2 = idx_l1[t * k_l1 + j2];        // re-read per pair: it stays in L1, and no private array is needed
                if ((unsigned)e2 >= (unsigned)E_l1) continue;
                if (USE_LDS) atomicAdd(&hist[(e1 * E_l1 + e2) * copies + my_copy], 1);
                else atomicAdd(&R[e1 * E_l1 + e2], 1ull);
            }
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
    const int bins = E_l * E_l1;
    long long want = ((long long)T + 256 * kTokPerThread - 1) / (256 * kTokPerThread);
    const unsigned grid = (unsigned)(want < 1 ? 1 : (want > 512 ? 512 : want));
    int copies = 1;
    while (copies < 32 && bins * copies * 2 <= kLdsBins) copies *= 2;
    LaunchTimer timer(MOE_K_TRANSITION, s);
    if (bins <= kLdsBins)
        hipLaunchKernelGGL(transition_kernel<true>, dim3(grid), dim3(256), bins * copies * sizeof(int), s, idx_l, idx_l1, T, k_l, k_l1,
                           use_l, use_l1, E_l, E_l1, copies, (unsigned long long*)R);
    else
        hipLaunchKernelGGL(transition_kernel<false>, dim3(grid), dim3(256), 0, s, idx_l, idx_l1, T, k_l, k_l1, use_l, use_l1, E_l, E_l1, 1,
                           (unsigned long long*)R);
    return check_launch("moe_transition_counts launch");
}

}  // namespace moe
