#include "ffn_plan.h"

namespace moe {

__global__ __launch_bounds__(256) void ffn_plan_kernel(const int32_t* __restrict__ counts, const int32_t* __restrict__ starts,
                                                       const int32_t* __restrict__ placement, int local_gpu,
                                                       const int32_t* __restrict__ group_expert, int n_weights, int E, int N,
                                                       int bm0, int bm1, int choice, int32_t* __restrict__ plan) {
    __shared__ __attribute__((aligned(16))) int cnt[MOE_MAX_EXPERTS];
    __shared__ __attribute__((aligned(16))) int rank[MOE_MAX_EXPERTS];
    __shared__ __attribute__((aligned(16))) int tiles0[MOE_MAX_EXPERTS];
    __shared__ __attribute__((aligned(16))) int tiles1[MOE_MAX_EXPERTS];
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
    // the loops below read the shared arrays four entries at a time; entries from E on hold zeros / -1
    const int E4 = (E + 3) / 4;
    int r = 0;
    if (c > 0) {
        const int4* cnt4 = reinterpret_cast<const int4*>(cnt);
        for (int q = 0; q < E4; ++q) {
            const int4 co = cnt4[q];
            const int o = 4 * q;
            r += ((co.x > c) | ((co.x == c) & (o < e))) + ((co.y > c) | ((co.y == c) & (o + 1 < e))) +
                 ((co.z > c) | ((co.z == c) & (o + 2 < e))) + ((co.w > c) | ((co.w == c) & (o + 3 < e)));
        }
    }
    rank[e] = (c > 0) ? r : -1;
    __syncthreads();
    if (c > 0) {
        int t0 = 0, t1 = 0;
        const int4* rank4 = reinterpret_cast<const int4*>(rank);
        const int4* tl0 = reinterpret_cast<const int4*>(tiles0);
        const int4* tl1 = reinterpret_cast<const int4*>(tiles1);
        for (int q = 0; q < E4; ++q) {
            const int4 ro = rank4[q], a = tl0[q], b = tl1[q];
            const bool k0 = (ro.x >= 0) & (ro.x < r), k1 = (ro.y >= 0) & (ro.y < r), k2 = (ro.z >= 0) & (ro.z < r), k3 = (ro.w >= 0) & (ro.w < r);
            t0 += (k0 ? a.x : 0) + (k1 ? a.y : 0) + (k2 ? a.z : 0) + (k3 ? a.w : 0);
            t1 += (k0 ? b.x : 0) + (k1 ? b.y : 0) + (k2 ? b.z : 0) + (k3 ? b.w : 0);
        }
        plan[kPlanExpert + r] = wt;
        plan[kPlanStart + r] = st;
        plan[kPlanCount + r] = c;
        plan[kPlanTiles0 + r] = t0;
        plan[kPlanTiles1 + r] = t1;
    }
    if (e == 0) {
        int n = 0, t0 = 0, t1 = 0;
        long long rows = 0;
        const int4* cnt4 = reinterpret_cast<const int4*>(cnt);
        const int4* tl0 = reinterpret_cast<const int4*>(tiles0);
        const int4* tl1 = reinterpret_cast<const int4*>(tiles1);
        for (int q = 0; q < E4; ++q) {
            const int4 co = cnt4[q], a = tl0[q], b = tl1[q];
            n += (co.x > 0) + (co.y > 0) + (co.z > 0) + (co.w > 0);
            rows += (long long)co.x + co.y + co.z + co.w;
            t0 += a.x + a.y + a.z + a.w;
            t1 += b.x + b.y + b.z + b.w;
        }
        plan[0] = n;
        plan[1] = t0;
        plan[2] = t1;
        plan[3] = choice >= 0 ? choice : (rows >= (long long)kLargeBucketRows * n ? 0 : 1);
        plan[kPlanTiles0 + n] = t0;
        plan[kPlanTiles1 + n] = t1;
    }
}

int launch_ffn_plan(const int32_t* counts, const int32_t* starts, const int32_t* placement, int local_gpu,
                    const int32_t* group_expert, int n_weights, int E, int N, int bm0, int bm1, int choice, int32_t* plan,
                    hipStream_t s) {
    LaunchTimer timer(MOE_K_FFN_PLAN, s);
    hipLaunchKernelGGL(ffn_plan_kernel, dim3(1), dim3(256), 0, s, counts, starts, placement, local_gpu, group_expert, n_weights, E, N, bm0, bm1, choice, plan);
    return check_launch("moe_expert_ffn_grouped plan launch");
}

}  // namespace moe
