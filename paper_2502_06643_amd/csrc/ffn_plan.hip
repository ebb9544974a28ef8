#include "ffn_plan.h"

namespace moe {

__global__ __launch_bounds__(256) void ffn_plan_kernel(const int32_t* __restrict__ counts, const int32_t* __restrict__ starts,
                                                       const int32_t* __restrict__ placement, int local_gpu,
                                                       const int32_t* __restrict__ group_expert, int n_weights, int E, int N,
                                                       int bm0, int bm1, int32_t* __restrict__ plan) {
    __shared__ int cnt[MOE_MAX_EXPERTS];
    __shared__ int rank[MOE_MAX_EXPERTS];
    __shared__ int tiles0[MOE_MAX_EXPERTS];
    __shared__ int tiles1[MOE_MAX_EXPERTS];
    const int e = threadIdx.x;
    int c = 0, st = 0, wt = e;                    // wt: whose weights this group multiplies with
    if (e < E) {
        const bool local = local_gpu < 0 || placement[e] == local_gpu;
        c = counts[e];
        st = starts[e];
        if (group_expert) wt = group_expert[e];
        // a bucket that does not lie inside [0,N), or names weights that do not exist, is ignored rather than trusted
        if (!local || c <= 0 || st < 0 || (long long)st + c > N || (unsigned)wt >= (unsigned)n_weights) c = 0;
    }
    cnt[e] = c;
    tiles0[e] = (c + bm0 - 1) / bm0;
    tiles1[e] = (c + bm1 - 1) / bm1;
    __syncthreads();
    int r = 0;
    if (c > 0) {
#pragma unroll 8
        for (int o = 0; o < E; ++o) {
            const int co = cnt[o];
            r += (co > c) | ((co == c) & (o < e));
        }
    }
    rank[e] = (c > 0) ? r : -1;
    __syncthreads();
    if (c > 0) {
        int t0 = 0, t1 = 0;
#pragma unroll 8
        for (int o = 0; o < E; ++o) {
            const int ro = rank[o];
            const int take = (ro >= 0) & (ro < r);
            t0 += take ? tiles0[o] : 0;
            t1 += take ? tiles1[o] : 0;
        }
        plan[kPlanExpert + r] = wt;
        plan[kPlanStart + r] = st;
        plan[kPlanCount + r] = c;
        plan[kPlanTiles0 + r] = t0;
        plan[kPlanTiles1 + r] = t1;
    }
    if (e == 0) {
        int n = 0, t0 = 0, t1 = 0;
#pragma unroll 8
        for (int o = 0; o < E; ++o) {
            n += cnt[o] > 0;
            t0 += tiles0[o];
            t1 += tiles1[o];
        }
        plan[0] = n;
        plan[1] = t0;
        plan[2] = t1;
        plan[kPlanTiles0 + n] = t0;
        plan[kPlanTiles1 + n] = t1;
    }
}

int launch_ffn_plan(const int32_t* counts, const int32_t* starts, const int32_t* placement, int local_gpu,
                    const int32_t* group_expert, int n_weights, int E, int N, int bm0, int bm1, int32_t* plan, hipStream_t s) {
    LaunchTimer timer(MOE_K_FFN_PLAN, s);
    hipLaunchKernelGGL(ffn_plan_kernel, dim3(1), dim3(256), 0, s, counts, starts, placement, local_gpu, group_expert, n_weights, E, N, bm0, bm1, plan);
    return check_launch("moe_expert_ffn_grouped plan launch");
}

}  // namespace moe
