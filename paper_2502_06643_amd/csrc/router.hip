// moe_router_gate: the linear router in front of the top-k gate (paper Section
// 2.1): logits = x . W_g + bias, then moe_topk_gate's selection on them.
//
// bf16: a skinny GEMM on the matrix cores that is bound by reading x once.  A
// workgroup owns 32 tokens; its 4 wavefronts split the reduction into four
// contiguous quarters, each feeding v_mfma_f32_32x32x16_bf16 with the activation
// fragment straight from memory (lane l: token l % 32, 8 consecutive k) and the
// weight fragments from the pre-packed router matrix (moe_pack_router: for every
// 16 reduction steps and every 32 experts one 1 KB block in B-fragment order, so
// a fragment is one coalesced 16-byte load per lane).  The four partial sums are
// added through LDS in wavefront order, so results are reproducible.
// fp32: one workgroup per token, one thread per expert, sequential fp32 sum.
// The logits are written to memory and the gate kernel runs on them.
#include "common.h"

namespace moe {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

static inline int padded_experts(int E) { return (E + 31) / 32 * 32; }

size_t router_packed_bytes(int d, int E, moe_dtype_t dt) {
    return dt == MOE_BF16 ? (size_t)padded_experts(E) * d * 2 : (size_t)d * E * sizeof(float);
}

// unit o = (kb * panels + panel) * 64 + lane holds 8 consecutive k of one expert column
__global__ __launch_bounds__(256) void pack_router_bf16_kernel(const uint16_t* __restrict__ w_g, int d, int E, int panels,
                                                               long long total, uint4* __restrict__ packed) {
    const long long o = (long long)blockIdx.x * 256 + threadIdx.x;
    if (o >= total) return;
    const int lane = (int)(o & 63);
    const long long blk = o >> 6;
    const int panel = (int)(blk % panels);
    const int kb = (int)(blk / panels);
    const int e = panel * 32 + (lane & 31);
    const int k0 = kb * 16 + 8 * (lane >> 5);
    uint16_t v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = (e < E) ? w_g[(size_t)(k0 + i) * E + e] : (uint16_t)0;
    uint4 q;
    q.x = v[0] | ((uint32_t)v[1] << 16); q.y = v[2] | ((uint32_t)v[3] << 16);
    q.z = v[4] | ((uint32_t)v[5] << 16); q.w = v[6] | ((uint32_t)v[7] << 16);
    packed[o] = q;
}

int launch_pack_router(const void* w_g, int d, int E, moe_dtype_t dt, void* packed, hipStream_t s) {
    if (dt == MOE_F32) {
        hipError_t e = hipMemcpyAsync(packed, w_g, (size_t)d * E * sizeof(float), hipMemcpyDeviceToDevice, s);
        return e == hipSuccess ? MOE_OK : hip_fail(e, "moe_pack_router copy");
    }
    const int panels = padded_experts(E) / 32;
    const long long total = (long long)(d / 16) * panels * 64;
    hipLaunchKernelGGL(pack_router_bf16_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, (const uint16_t*)w_g, d, E,
                       panels, total, (uint4*)packed);
    return check_launch("moe_pack_router launch");
}

template <int PANELS>
__global__ __launch_bounds__(256) void router_proj_bf16_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ packed,
                                                               const float* __restrict__ bias, int T, int d, int E,
                                                               float* __restrict__ logits) {
    extern __shared__ float red[];                       // [PANELS][16][64] partial sums
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const long long t0 = (long long)blockIdx.x * 32;
    const long long tr = min(t0 + (lane & 31), (long long)T - 1);        // tokens past the end re-read the last one
    const uint16_t* xrow = x + tr * d + 8 * (lane >> 5);
    const uint16_t* wlane = packed + (size_t)lane * 8;
    f32x16 acc[PANELS];
#pragma unroll
    for (int p = 0; p < PANELS; ++p)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[p][v] = 0.f;
    const int KS = d / 16;
    // each wavefront owns a contiguous quarter of the reduction, so that consecutive k-steps of a lane
    // fall into the same 128-byte line of its token's row; U k-steps have their loads in flight together
    constexpr int U = (PANELS <= 2) ? 8 : 4;
    const int KSW = KS / 4;                              // d % 64 == 0
    int ks = wave * KSW;
    const int ks_end = ks + KSW;
    for (; ks + U <= ks_end; ks += U) {
        bf16x8 a[U], b[U][PANELS];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            a[u] = *reinterpret_cast<const bf16x8*>(xrow + (ks + u) * 16);
#pragma unroll
            for (int p = 0; p < PANELS; ++p)
                b[u][p] = *reinterpret_cast<const bf16x8*>(wlane + ((size_t)(ks + u) * PANELS + p) * 512);
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int p = 0; p < PANELS; ++p) acc[p] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[u], b[u][p], acc[p], 0, 0, 0);
    }
    for (; ks < ks_end; ++ks) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(xrow + ks * 16);
#pragma unroll
        for (int p = 0; p < PANELS; ++p) {
            const bf16x8 b = *reinterpret_cast<const bf16x8*>(wlane + ((size_t)ks * PANELS + p) * 512);
            acc[p] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[p], 0, 0, 0);
        }
    }
    // add the four partial sums in wavefront order
    for (int w = 0; w < 4; ++w) {
        if (wave == w && w < 3) {
#pragma unroll
            for (int p = 0; p < PANELS; ++p)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    float* slot = &red[(p * 16 + v) * 64 + lane];
                    *slot = (w == 0) ? acc[p][v] : *slot + acc[p][v];
                }
        }
        if (w < 3) __syncthreads();
    }
    if (wave != 3) return;
    // accumulator v: token 8*(v/4) + 4*(lane/32) + v%4 of this workgroup, expert panel*32 + lane%32
#pragma unroll
    for (int p = 0; p < PANELS; ++p) {
        const int e = p * 32 + (lane & 31);
        const float b = (bias != nullptr && e < E) ? bias[e] : 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const long long t = t0 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
            if (t < T && e < E) logits[t * E + e] = red[(p * 16 + v) * 64 + lane] + acc[p][v] + b;
        }
    }
}

__global__ __launch_bounds__(256) void router_proj_f32_kernel(const float* __restrict__ x, const float* __restrict__ w_g,
                                                              const float* __restrict__ bias, int d, int E,
                                                              float* __restrict__ logits) {
    const long long t = blockIdx.x;
    const int e = threadIdx.x;
    if (e >= E) return;
    float s = 0.f;
    for (int i = 0; i < d; ++i) s = fmaf(x[t * d + i], w_g[(size_t)i * E + e], s);
    logits[t * E + e] = s + (bias ? bias[e] : 0.f);
}

template <int PANELS>
static void launch_proj(const uint16_t* x, const uint16_t* packed, const float* bias, int T, int d, int E, float* logits, hipStream_t s) {
    hipLaunchKernelGGL(router_proj_bf16_kernel<PANELS>, dim3((unsigned)((T + 31) / 32)), dim3(256), PANELS * 16 * 64 * sizeof(float), s,
                       x, packed, bias, T, d, E, logits);
}

int launch_router_gate(const void* x, moe_dtype_t dt, const void* packed, const float* bias, int T, int d, int E, int k,
                       float* logits, int32_t* idx, float* w, hipStream_t s) {
    {
        LaunchTimer timer(MOE_K_ROUTER, s);
        if (dt == MOE_BF16) {
            const uint16_t* xs = (const uint16_t*)x;
            const uint16_t* ps = (const uint16_t*)packed;
            switch (padded_experts(E) / 32) {
                case 1: launch_proj<1>(xs, ps, bias, T, d, E, logits, s); break;
                case 2: launch_proj<2>(xs, ps, bias, T, d, E, logits, s); break;
                case 3: launch_proj<3>(xs, ps, bias, T, d, E, logits, s); break;
                case 4: launch_proj<4>(xs, ps, bias, T, d, E, logits, s); break;
                case 5: launch_proj<5>(xs, ps, bias, T, d, E, logits, s); break;
                case 6: launch_proj<6>(xs, ps, bias, T, d, E, logits, s); break;
                case 7: launch_proj<7>(xs, ps, bias, T, d, E, logits, s); break;
                default: launch_proj<8>(xs, ps, bias, T, d, E, logits, s); break;
            }
        } else {
            hipLaunchKernelGGL(router_proj_f32_kernel, dim3((unsigned)T), dim3(256), 0, s, (const float*)x, (const float*)packed, bias,
                               d, E, logits);
        }
        int rc = check_launch("moe_router_gate projection launch");
        if (rc != MOE_OK) return rc;
    }
    return launch_gate(logits, T, E, k, false, idx, w, s);
}

}  // namespace moe
