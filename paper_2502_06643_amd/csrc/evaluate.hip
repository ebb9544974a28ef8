// Placement evaluators: the quantities the paper's two ILPs are built from,
// computed on the GPU from the profiled statistics and a given expert->GPU map
// (the solve itself is not here).
//   moe_accumulate_counts : P_{e,l} += expert_counts of one batch      (ILP 1 input)
//   moe_placement_loads   : T_{c,l} = sum_e P_{e,l} x_{c,e,l}          (Eq. 2)
//                           sum_c |T_{c,l} - mean_l|, mean_l = sum_e P_{e,l} / G   (Eq. 1, Eq. 3)
//   moe_placement_traffic : C_{c1,c2,l} = sum R_{e1,e2,l} x_{c1,e1,l} x_{c2,e2,l+1}   (Eq. 9)
//                           max over GPU pairs of C / B                 (Eq. 8, one layer's term)
// The tables are tiny (E <= 256, G <= 256), so each call is one workgroup.
#include "common.h"

namespace moe {

__global__ __launch_bounds__(256) void accumulate_counts_kernel(const int32_t* __restrict__ counts, int E, long long* __restrict__ P) {
    const int e = threadIdx.x;
    if (e < E) P[e] += (long long)counts[e];
}

__global__ __launch_bounds__(256) void placement_loads_kernel(const long long* __restrict__ P, const int32_t* __restrict__ placement,
                                                              int E, int G, long long* __restrict__ T_c, double* __restrict__ imbalance) {
    __shared__ long long load[MOE_MAX_GPUS];
    __shared__ double dev[MOE_MAX_GPUS];
    const int g = threadIdx.x;
    long long mine = 0, total = 0;
    for (int e = 0; e < E; ++e) {                        // every thread walks the E experts: E <= 256
        const long long p = P[e];
        total += p;
        if (placement[e] == g) mine += p;
    }
    if (g < G) {
        load[g] = mine;
        T_c[g] = mine;
        dev[g] = fabs((double)mine - (double)total / (double)G);
    }
    __syncthreads();
    if (g == 0 && imbalance) {
        double s = 0.0;
        for (int c = 0; c < G; ++c) s += dev[c];         // fixed order
        *imbalance = s;
    }
}

__global__ __launch_bounds__(256) void placement_traffic_kernel(const long long* __restrict__ R, const int32_t* __restrict__ pl_l,
                                                                const int32_t* __restrict__ pl_l1, int E_l, int E_l1, int G,
                                                                long long* __restrict__ C, const double* __restrict__ B,
                                                                double* __restrict__ max_cost) {
    __shared__ double best[256];
    // thread t owns the GPU pairs p = t, t + 256, ...; for each it walks the whole R table (<= 65536 entries)
    double local_max = 0.0;
    for (int p = threadIdx.x; p < G * G; p += 256) {
        const int g1 = p / G, g2 = p - g1 * G;
        long long s = 0;
        for (int e1 = 0; e1 < E_l; ++e1) {
            if (pl_l[e1] != g1) continue;
            for (int e2 = 0; e2 < E_l1; ++e2)
                if (pl_l1[e2] == g2) s += R[(size_t)e1 * E_l1 + e2];
        }
        C[p] = s;
        const double cost = B ? (double)s / B[p] : (double)s;
        local_max = cost > local_max ? cost : local_max;
    }
    best[threadIdx.x] = local_max;
    __syncthreads();
    if (threadIdx.x == 0 && max_cost) {
        double m = 0.0;
        for (int i = 0; i < 256; ++i) m = best[i] > m ? best[i] : m;
        *max_cost = m;
    }
}

int launch_accumulate_counts(const int32_t* counts, int E, int64_t* P, hipStream_t s) {
    hipLaunchKernelGGL(accumulate_counts_kernel, dim3(1), dim3(256), 0, s, counts, E, (long long*)P);
    return check_launch("moe_accumulate_counts launch");
}

int launch_placement_loads(const int64_t* P, const int32_t* placement, int E, int G, int64_t* T_c, double* imbalance, hipStream_t s) {
    hipLaunchKernelGGL(placement_loads_kernel, dim3(1), dim3(256), 0, s, (const long long*)P, placement, E, G, (long long*)T_c, imbalance);
    return check_launch("moe_placement_loads launch");
}

int launch_placement_traffic(const int64_t* R, const int32_t* pl_l, const int32_t* pl_l1, int E_l, int E_l1, int G, int64_t* C,
                             const double* B, double* max_cost, hipStream_t s) {
    hipLaunchKernelGGL(placement_traffic_kernel, dim3(1), dim3(256), 0, s, (const long long*)R, pl_l, pl_l1, E_l, E_l1, G,
                       (long long*)C, B, max_cost);
    return check_launch("moe_placement_traffic launch");
}

}  // namespace moe
