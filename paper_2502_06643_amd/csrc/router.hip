// moe_router_gate: the linear router in front of the top-k gate (paper Section
// 2.1): logits = x . W_g + bias and moe_topk_gate's selection on them, in ONE
// kernel: the logits of a workgroup's tokens never leave the compute unit
// (writing them to memory is optional).
//
// bf16: a skinny GEMM on the matrix cores that is bound by reading x once.  A
// workgroup owns 32 tokens; its 4 wavefronts split the reduction into four
// contiguous quarters, each feeding v_mfma_f32_32x32x16_bf16 with the activation
// fragment (lane l: token l % 32, 8 consecutive k; fetched as whole lines and
// re-ordered through a staging tile in LDS, see the kernel) and the
// weight fragments from the pre-packed router matrix (moe_pack_router: for every
// 16 reduction steps and every 32 experts one 1 KB block in B-fragment order, so
// a fragment is one coalesced 16-byte load per lane).  The four partial sums are
// added through LDS in wavefront order, so results are reproducible; the last
// wavefront leaves the 32 x E logits in LDS (and in memory when asked to) and
// all 256 threads run the gate's selection on them, 8 lanes per token.
// fp32: one workgroup per token, one thread per expert, sequential fp32 sum,
// then 16 lanes select from the row in LDS.
#include "gate_select.h"

namespace moe {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

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

// LDS of the bf16 kernel, in floats: four staging tiles of 32 tokens x 64 k (bf16), then the partial sums
// [PANELS][16][64], then the logits [32 tokens][32 * PANELS + 4] (rows padded by 16 bytes), one after the other in
// the same memory
constexpr int router_lds_floats(int panels) { return 32 * (32 * panels + 4) > 4 * 32 * 64 / 2 ? 32 * (32 * panels + 4) : 4 * 32 * 64 / 2; }

template <int PANELS, int KMAX>
__global__ __launch_bounds__(256) void router_gate_bf16_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ packed,
                                                               const float* __restrict__ bias, int T, int d, int E, int k,
                                                               float* __restrict__ logits, int32_t* __restrict__ topk_idx,
                                                               float* __restrict__ topk_w) {
    extern __shared__ __attribute__((aligned(16))) float red[];      // activation staging, then [PANELS][16][64] partial sums, then the logits
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const long long t0 = (long long)blockIdx.x * 32;
    const uint16_t* wlane = packed + (size_t)lane * 8;
    f32x16 acc[PANELS];
#pragma unroll
    for (int p = 0; p < PANELS; ++p)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[p][v] = 0.f;
    // Each wavefront owns a contiguous quarter of the reduction and streams it in stages of 64 k: 32 tokens x
    // 128 bytes, fetched as four fully coalesced 16-byte loads per lane (lane l: token 8 j + l / 8, 16-byte chunk
    // l % 8: whole 128-byte lines) into registers one stage ahead, written to a staging tile of its own in LDS
    // (no barrier: a wavefront's LDS accesses execute in order) whose eight 16-byte slots per row are XOR-swizzled
    // by (row >> 1) & 7, and read back as the A operand of the matrix instruction (lane l: token l % 32, the 8
    // consecutive k that start at 8 * (l / 32) of every 16): conflict-free both ways.  Loading the operand
    // straight from memory instead costs four partly used lines per instruction.
    constexpr int KSTAGE = 64;
    uint16_t* stage = reinterpret_cast<uint16_t*>(red) + wave * (32 * KSTAGE);
    const int KSW = d / 4;                               // k of this wavefront; d % 64 == 0 ...
    const int n_stage = KSW / KSTAGE;                    // ... but KSW % 64 may be 0, 16, 32 or 48: the rest goes the direct way
    const int kw0 = wave * KSW;
    u32x4 cur[4], nxt[4];                                // the stage being multiplied and the next one, in flight (two ahead measured the same)
    const int lr = lane >> 3, lc = lane & 7;
    auto fetch = [&](int st, u32x4 (&r)[4]) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const long long t = min(t0 + 8 * j + lr, (long long)T - 1);          // tokens past the end re-read the last one
            r[j] = *reinterpret_cast<const u32x4*>(x + t * d + kw0 + st * KSTAGE + lc * 8);
        }
    };
    if (n_stage > 0) fetch(0, cur);
    for (int st = 0; st < n_stage; ++st) {
        if (st + 1 < n_stage) fetch(st + 1, nxt);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int row = 8 * j + lr;
            *reinterpret_cast<u32x4*>(stage + row * KSTAGE + ((lc ^ ((row >> 1) & 7)) * 8)) = cur[j];
        }
        const int ks0 = (kw0 + st * KSTAGE) / 16;
#pragma unroll
        for (int u = 0; u < KSTAGE / 16; ++u) {
            const int row = lane & 31;
            const bf16x8 a = *reinterpret_cast<const bf16x8*>(stage + row * KSTAGE + (((2 * u + (lane >> 5)) ^ ((row >> 1) & 7)) * 8));
#pragma unroll
            for (int p = 0; p < PANELS; ++p) {
                const bf16x8 b = *reinterpret_cast<const bf16x8*>(wlane + ((size_t)(ks0 + u) * PANELS + p) * 512);
                acc[p] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[p], 0, 0, 0);
            }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) cur[j] = nxt[j];
    }
    {
        const long long tr = min(t0 + (lane & 31), (long long)T - 1);
        const uint16_t* xrow = x + tr * d + 8 * (lane >> 5);
        for (int ks = (kw0 + n_stage * KSTAGE) / 16; ks < (kw0 + KSW) / 16; ++ks) {
            const bf16x8 a = *reinterpret_cast<const bf16x8*>(xrow + ks * 16);
#pragma unroll
            for (int p = 0; p < PANELS; ++p) {
                const bf16x8 b = *reinterpret_cast<const bf16x8*>(wlane + ((size_t)ks * PANELS + p) * 512);
                acc[p] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[p], 0, 0, 0);
            }
        }
    }
    __syncthreads();                                     // every wavefront is done with its staging tile: the partial sums overwrite them
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
    constexpr int RS = 32 * PANELS + 4;                   // row stride of the logits in LDS
    if (wave == 3) {
        // accumulator v: token 8*(v/4) + 4*(lane/32) + v%4 of this workgroup, expert panel*32 + lane%32.
        // First every partial sum is read (the logits overwrite the same LDS), then the logits are written.
#pragma unroll
        for (int p = 0; p < PANELS; ++p) {
            const int e = p * 32 + (lane & 31);
            const float b = (bias != nullptr && e < E) ? bias[e] : 0.f;
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[p][v] = red[(p * 16 + v) * 64 + lane] + acc[p][v] + b;
        }
        // (a wavefront's LDS accesses execute in program order, so these reads precede the writes below)
#pragma unroll
        for (int p = 0; p < PANELS; ++p) {
            const int e = p * 32 + (lane & 31);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int tl = 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                red[tl * RS + e] = acc[p][v];
                if (logits != nullptr && t0 + tl < T && e < E) logits[(t0 + tl) * E + e] = acc[p][v];
            }
        }
    }
    __syncthreads();
    // the gate: 8 lanes per token, 4 * PANELS logits per lane
    const int tl = threadIdx.x >> 3;
    gate_select<8, 4 * PANELS, KMAX, false>(red + tl * RS, true, threadIdx.x & 7, t0 + tl < T, t0 + tl, E, k, topk_idx, topk_w);
}

template <int KMAX>
__global__ __launch_bounds__(256) void router_gate_f32_kernel(const float* __restrict__ x, const float* __restrict__ w_g,
                                                              const float* __restrict__ bias, int d, int E, int k,
                                                              float* __restrict__ logits, int32_t* __restrict__ topk_idx,
                                                              float* __restrict__ topk_w) {
    __shared__ __attribute__((aligned(16))) float row[MOE_MAX_EXPERTS];
    const long long t = blockIdx.x;
    const int e = threadIdx.x;
    if (e < E) {
        float s = 0.f;
        for (int i = 0; i < d; ++i) s = fmaf(x[t * d + i], w_g[(size_t)i * E + e], s);
        s += bias ? bias[e] : 0.f;
        row[e] = s;
        if (logits != nullptr) logits[t * E + e] = s;
    }
    __syncthreads();
    gate_select<16, MOE_MAX_EXPERTS / 16, KMAX, false>(row, true, threadIdx.x & 15, threadIdx.x < 16, t, E, k, topk_idx, topk_w);
}

template <int PANELS>
static void launch_fused(const uint16_t* x, const uint16_t* packed, const float* bias, int T, int d, int E, int k, float* logits,
                         int32_t* idx, float* w, hipStream_t s) {
    const dim3 grid((unsigned)((T + 31) / 32)), block(256);
    const size_t lds = router_lds_floats(PANELS) * sizeof(float);
    if (k <= 2) hipLaunchKernelGGL((router_gate_bf16_kernel<PANELS, 2>), grid, block, lds, s, x, packed, bias, T, d, E, k, logits, idx, w);
    else if (k <= 8) hipLaunchKernelGGL((router_gate_bf16_kernel<PANELS, 8>), grid, block, lds, s, x, packed, bias, T, d, E, k, logits, idx, w);
    else hipLaunchKernelGGL((router_gate_bf16_kernel<PANELS, MOE_MAX_TOPK>), grid, block, lds, s, x, packed, bias, T, d, E, k, logits, idx, w);
}

int launch_router_gate(const void* x, moe_dtype_t dt, const void* packed, const float* bias, int T, int d, int E, int k,
                       float* logits, int32_t* idx, float* w, hipStream_t s) {
    LaunchTimer timer(MOE_K_ROUTER, s);
    if (dt == MOE_BF16) {
        const uint16_t* xs = (const uint16_t*)x;
        const uint16_t* ps = (const uint16_t*)packed;
        switch (padded_experts(E) / 32) {
            case 1: launch_fused<1>(xs, ps, bias, T, d, E, k, logits, idx, w, s); break;
            case 2: launch_fused<2>(xs, ps, bias, T, d, E, k, logits, idx, w, s); break;
            case 3: launch_fused<3>(xs, ps, bias, T, d, E, k, logits, idx, w, s); break;
            case 4: launch_fused<4>(xs, ps, bias, T, d, E, k, logits, idx, w, s); break;
            case 5: launch_fused<5>(xs, ps, bias, T, d, E, k, logits, idx, w, s); break;
            case 6: launch_fused<6>(xs, ps, bias, T, d, E, k, logits, idx, w, s); break;
            case 7: launch_fused<7>(xs, ps, bias, T, d, E, k, logits, idx, w, s); break;
            default: launch_fused<8>(xs, ps, bias, T, d, E, k, logits, idx, w, s); break;
        }
    } else {
        const float* xf = (const float*)x;
        const float* wf = (const float*)packed;
        if (k <= 2) hipLaunchKernelGGL(router_gate_f32_kernel<2>, dim3((unsigned)T), dim3(256), 0, s, xf, wf, bias, d, E, k, logits, idx, w);
        else if (k <= 8) hipLaunchKernelGGL(router_gate_f32_kernel<8>, dim3((unsigned)T), dim3(256), 0, s, xf, wf, bias, d, E, k, logits, idx, w);
        else hipLaunchKernelGGL(router_gate_f32_kernel<MOE_MAX_TOPK>, dim3((unsigned)T), dim3(256), 0, s, xf, wf, bias, d, E, k, logits, idx, w);
    }
    return check_launch("moe_router_gate launch");
}

}  // namespace moe
