// fp32 path of moe_expert_ffn_grouped (paper Section 2.2 / Fig. 2b, "FFN
// computations" of the resident experts).  A plain LDS-tiled SGEMM pair:
//   up  : H = silu(A W1_e) * (A W3_e)     (both products in one pass over A)
//   down: out = H W2_e
// 64x64 output tile per workgroup, 16-deep k steps, 4x4 outputs per thread,
// fp32 fused multiply-adds.  This path exists for exactness checks on small
// layers; the throughput path is the bf16 MFMA kernel.
#include "ffn_plan.h"

namespace moe {

constexpr int FBM = 64, FBN = 64, FBK = 16;

size_t packed_bytes_f32(int E, int d, int f) { return (size_t)E * 3 * d * f * sizeof(float); }

int launch_pack_f32(const float* w1, const float* w3, const float* w2, int E, int d, int f, float* packed, hipStream_t s) {
    // per expert: [W1 d*f | W3 d*f | W2 f*d], each matrix row-major as given
    const size_t m = (size_t)d * f * sizeof(float);
    const float* src[3] = {w1, w3, w2};
    for (int i = 0; i < 3; ++i) {
        hipError_t e = hipMemcpy2DAsync((char*)packed + i * m, 3 * m, src[i], m, m, E, hipMemcpyDeviceToDevice, s);
        if (e != hipSuccess) return hip_fail(e, "moe_pack_weights copy");
    }
    return MOE_OK;
}

template <bool UP>
__global__ __launch_bounds__(256) void ffn_f32_kernel(const float* __restrict__ A, const float* __restrict__ packed,
                                                      int d, int f, float* __restrict__ C, const int32_t* __restrict__ plan) {
    const int K = UP ? d : f;          // reduction length
    const int NC = UP ? f : d;         // output columns
    RowTile rt;
    if (!find_row_tile(plan, plan + kPlanTiles0, blockIdx.y, FBM, rt)) return;
    const float* We = packed + (size_t)rt.expert * 3 * d * f;
    const float* B0 = UP ? We : We + (size_t)2 * d * f;       // W1 or W2
    const float* B1 = We + (size_t)d * f;                     // W3 (UP only)
    const int n0 = blockIdx.x * FBN;

    __shared__ float As[FBK][FBM + 4];
    __shared__ float Bs0[FBK][FBN];
    __shared__ float Bs1[UP ? FBK : 1][FBN];

    const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
    float acc0[4][4] = {}, acc1[4][4] = {};

    for (int k0 = 0; k0 < K; k0 += FBK) {
        // A tile: 64 rows x 16 k, one float4 along k per thread
        {
            const int r = threadIdx.x / 4, kc = (threadIdx.x % 4) * 4;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (r < rt.rows && k0 + kc < K)      // K % 4 == 0, so a float4 never straddles the end
                v = *reinterpret_cast<const float4*>(A + (size_t)(rt.row0 + r) * K + k0 + kc);
            As[kc + 0][r] = v.x; As[kc + 1][r] = v.y; As[kc + 2][r] = v.z; As[kc + 3][r] = v.w;
        }
        // B tile(s): 16 k x 64 columns, one float4 along the columns per thread
        {
            const int kr = threadIdx.x / 16, c = (threadIdx.x % 16) * 4;
            float4 v0 = make_float4(0.f, 0.f, 0.f, 0.f), v1 = v0;
            if (k0 + kr < K && n0 + c < NC) {    // NC % 4 == 0
                v0 = *reinterpret_cast<const float4*>(B0 + (size_t)(k0 + kr) * NC + n0 + c);
                if (UP) v1 = *reinterpret_cast<const float4*>(B1 + (size_t)(k0 + kr) * NC + n0 + c);
            }
            *reinterpret_cast<float4*>(&Bs0[kr][c]) = v0;
            if (UP) *reinterpret_cast<float4*>(&Bs1[kr][c]) = v1;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < FBK; ++kk) {
            float a[4], b0[4], b1[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                b0[j] = Bs0[kk][tx * 4 + j];
                b1[j] = UP ? Bs1[kk][tx * 4 + j] : 0.f;
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    acc0[i][j] = fmaf(a[i], b0[j], acc0[i][j]);
                    if (UP) acc1[i][j] = fmaf(a[i], b1[j], acc1[i][j]);
                }
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = ty * 4 + i;
        if (r >= rt.rows) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int c = n0 + tx * 4 + j;
            if (c >= NC) continue;
            float v = acc0[i][j];
            if (UP) v = v / (1.0f + expf(-v)) * acc1[i][j];
            C[(size_t)(rt.row0 + r) * NC + c] = v;
        }
    }
}

int launch_ffn_f32(const float* a, int N, int d, int f, int E, const float* packed, const int32_t* counts,
                   const int32_t* starts, const int32_t* placement, int local_gpu, const int32_t* group_expert,
                   int n_weights, float* out, int32_t* plan, float* H, hipStream_t s) {
    int rc = launch_ffn_plan(counts, starts, placement, local_gpu, group_expert, n_weights, E, N, FBM, FBM, 0, plan, s);
    if (rc != MOE_OK) return rc;
    const int mt_max = (N + FBM - 1) / FBM + (E < N ? E : N);     // sum of ceil(n_e/BM) never exceeds this
    if (mt_max > 65535) return fail(MOE_ERR_UNSUPPORTED, "moe_expert_ffn_grouped: fp32 path supports at most %d routes", (65535 - 256) * FBM);
    {
        LaunchTimer timer(MOE_K_FFN_UP, s);
        hipLaunchKernelGGL(ffn_f32_kernel<true>, dim3((f + FBN - 1) / FBN, mt_max), dim3(256), 0, s, a, packed, d, f, H, plan);
        if ((rc = check_launch("moe_expert_ffn_grouped up launch")) != MOE_OK) return rc;
    }
    {
        LaunchTimer timer(MOE_K_FFN_DOWN, s);
        hipLaunchKernelGGL(ffn_f32_kernel<false>, dim3((d + FBN - 1) / FBN, mt_max), dim3(256), 0, s, (const float*)H, packed, d, f, out, plan);
        if ((rc = check_launch("moe_expert_ffn_grouped down launch")) != MOE_OK) return rc;
    }
    return MOE_OK;
}

}  // namespace moe
