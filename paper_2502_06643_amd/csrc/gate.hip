// moe_topk_gate: top-k router (paper Section 2.1).
//
// A token's E logits are spread over L neighbouring lanes of a wavefront, four
// consecutive logits per lane (one 16-byte load when E % 4 == 0), so a
// wavefront reads 64/L whole rows as one contiguous block.  Each logit becomes
// a 64-bit key  (order-preserving bits of the float) << 32 | ~expert , for
// which "larger key" is exactly "larger logit, ties to the lower expert".  k
// rounds of (best of my four) -> (xor-butterfly max over the L lanes) select
// the experts in descending order; the winner's key is retired by its owner.
// Weights are the softmax over the k selected logits in fp32.
#include "common.h"

namespace moe {

__device__ __forceinline__ uint32_t orderable(float v) {
    if (v == 0.0f) v = 0.0f;                       // -0.0 and +0.0 tie
    uint32_t u = __float_as_uint(v);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ float from_orderable(uint32_t o) {
    uint32_t u = (o & 0x80000000u) ? (o & 0x7FFFFFFFu) : ~o;
    return __uint_as_float(u);
}

__device__ __forceinline__ unsigned long long shfl_xor_u64(unsigned long long v, int m) {
    uint32_t lo = (uint32_t)v, hi = (uint32_t)(v >> 32);
    lo = __shfl_xor(lo, m, 64);
    hi = __shfl_xor(hi, m, 64);
    return ((unsigned long long)hi << 32) | lo;
}

template <int L>
__global__ __launch_bounds__(256) void gate_kernel(const float* __restrict__ logits, int T, int E, int k,
                                                   int32_t* __restrict__ topk_idx, float* __restrict__ topk_w) {
    constexpr int TOK_PER_BLOCK = 256 / L;
    const int sub = threadIdx.x % L;
    const long long t = (long long)blockIdx.x * TOK_PER_BLOCK + threadIdx.x / L;
    const bool live = t < T;
    const int e0 = sub * 4;

    unsigned long long key[4] = {0ull, 0ull, 0ull, 0ull};      // 0 = "no candidate"
    if (live && e0 < E) {
        const float* row = logits + t * E;
        float v[4];
        if ((E & 3) == 0) {
            const float4 q = *reinterpret_cast<const float4*>(row + e0);
            v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) v[i] = (e0 + i < E) ? row[e0 + i] : 0.f;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (e0 + i < E)
                key[i] = ((unsigned long long)orderable(v[i]) << 32) | (uint32_t)(~(uint32_t)(e0 + i));
    }

    float top = 0.f, denom = 0.f;
    for (int j = 0; j < k; ++j) {
        unsigned long long best = key[0];
#pragma unroll
        for (int i = 1; i < 4; ++i) best = key[i] > best ? key[i] : best;
#pragma unroll
        for (int m = 1; m < L; m <<= 1) {
            const unsigned long long o = shfl_xor_u64(best, m);
            best = o > best ? o : best;
        }
        const uint32_t e_win = ~(uint32_t)best;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if ((uint32_t)(e0 + i) == e_win) key[i] = 0ull;
        const float lj = from_orderable((uint32_t)(best >> 32));
        if (j == 0) top = lj;
        const float p = expf(lj - top);              // exp(0) = 1 for the top-1 expert
        denom += p;
        if (live && sub == 0) {
            topk_idx[t * k + j] = (int32_t)e_win;
            topk_w[t * k + j] = p;                   // normalised below by the same lane
        }
    }
    if (live && sub == 0)
        for (int j = 0; j < k; ++j) topk_w[t * k + j] = topk_w[t * k + j] / denom;
}

template <int L>
static void launch_l(const float* logits, int T, int E, int k, int32_t* idx, float* w, hipStream_t s) {
    constexpr int TOK_PER_BLOCK = 256 / L;
    const unsigned grid = (unsigned)(((long long)T + TOK_PER_BLOCK - 1) / TOK_PER_BLOCK);
    hipLaunchKernelGGL(gate_kernel<L>, dim3(grid), dim3(256), 0, s, logits, T, E, k, idx, w);
}

int launch_gate(const float* logits, int T, int E, int k, int32_t* idx, float* w, hipStream_t s) {
    LaunchTimer timer(MOE_K_GATE, s);
    const int lanes = (E + 3) / 4;
    if (lanes <= 2) launch_l<2>(logits, T, E, k, idx, w, s);
    else if (lanes <= 4) launch_l<4>(logits, T, E, k, idx, w, s);
    else if (lanes <= 8) launch_l<8>(logits, T, E, k, idx, w, s);
    else if (lanes <= 16) launch_l<16>(logits, T, E, k, idx, w, s);
    else if (lanes <= 32) launch_l<32>(logits, T, E, k, idx, w, s);
    else launch_l<64>(logits, T, E, k, idx, w, s);
    return check_launch("moe_topk_gate launch");
}

}  // namespace moe
