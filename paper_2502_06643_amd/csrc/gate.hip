// moe_topk_gate: top-k router (paper Section 2.1).
//
// A token's E logits are spread over L neighbouring lanes of a wavefront, VPL
// consecutive logits per lane (16-byte loads when E % 4 == 0), so a wavefront
// reads 64/L whole rows.  Each logit is mapped to an order-preserving unsigned
// key (-0.0 is folded onto +0.0 first, so the two tie); key 0 is below every
// finite logit and marks "no candidate".  One round = scan my VPL keys with a
// strict '>' (ascending index, so the lowest index wins a tie), then an
// xor-butterfly over the L lanes on (key, index) with the same tie rule, then
// the owner retires the winner.  k rounds give the experts in descending logit
// order.  Weights are the softmax over the k selected logits in fp32, or (ALL)
// the softmax over all E logits read at the selected experts: then every lane
// adds exp(logit - top) over its own logits after the first round and a
// butterfly sum over the L lanes gives the denominator.
#include "common.h"

namespace moe {

__device__ __forceinline__ uint32_t orderable(float v) {
    if (v == 0.0f) v = 0.0f;                       // -0.0 and +0.0 tie
    const uint32_t u = __float_as_uint(v);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ float from_orderable(uint32_t o) {
    const uint32_t u = (o & 0x80000000u) ? (o & 0x7FFFFFFFu) : ~o;
    return __uint_as_float(u);
}

template <int L, int VPL, int KMAX, bool ALL>
__global__ __launch_bounds__(256) void gate_kernel(const float* __restrict__ logits, int T, int E, int k,
                                                   int32_t* __restrict__ topk_idx, float* __restrict__ topk_w) {
    constexpr int TOK_PER_BLOCK = 256 / L;
    const int sub = threadIdx.x % L;
    const long long t = (long long)blockIdx.x * TOK_PER_BLOCK + threadIdx.x / L;
    const bool live = t < T;
    const int e0 = sub * VPL;

    uint32_t key[VPL];
#pragma unroll
    for (int i = 0; i < VPL; ++i) key[i] = 0u;
    if (live) {
        const float* row = logits + t * E;
        if ((E & 3) == 0) {
#pragma unroll
            for (int c = 0; c < VPL / 4; ++c) {
                if (e0 + 4 * c < E) {
                    const float4 q = *reinterpret_cast<const float4*>(row + e0 + 4 * c);
                    key[4 * c] = orderable(q.x); key[4 * c + 1] = orderable(q.y);
                    key[4 * c + 2] = orderable(q.z); key[4 * c + 3] = orderable(q.w);
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < VPL; ++i)
                if (e0 + i < E) key[i] = orderable(row[e0 + i]);
        }
    }

    // KMAX >= k is a compile-time bound so that the selected experts and weights stay in registers
    // and are written once
    float top = 0.f, denom = 0.f;
    float p_sel[KMAX];
    int e_sel[KMAX];
#pragma unroll
    for (int j = 0; j < KMAX; ++j) {
        p_sel[j] = 0.f;
        e_sel[j] = 0;
        if (j < k) {
            uint32_t best = key[0];
            int bi = 0;
#pragma unroll
            for (int i = 1; i < VPL; ++i)
                if (key[i] > best) { best = key[i]; bi = i; }
            int be = e0 + bi;
#pragma unroll
            for (int m = 1; m < L; m <<= 1) {
                const uint32_t ok = __shfl_xor(best, m, 64);
                const int oe = __shfl_xor(be, m, 64);
                if (ok > best || (ok == best && oe < be)) { best = ok; be = oe; }
            }
            if (ALL && j == 0) {                    // before the winner is retired: every logit still has its key
                const float t0 = from_orderable(best);
                float sum = 0.f;
#pragma unroll
                for (int i = 0; i < VPL; ++i)
                    if (key[i] != 0u) sum += expf(from_orderable(key[i]) - t0);
#pragma unroll
                for (int m = 1; m < L; m <<= 1) sum += __shfl_xor(sum, m, 64);
                denom = sum;
            }
            const int mine = be - e0;               // in [0,VPL) only for the owner lane
#pragma unroll
            for (int i = 0; i < VPL; ++i)
                if (i == mine) key[i] = 0u;
            const float lj = from_orderable(best);
            if (j == 0) top = lj;
            const float p = expf(lj - top);         // exp(0) = 1 for the top-1 expert
            if (!ALL) denom += p;
            p_sel[j] = p;
            e_sel[j] = be;
        }
    }
    if (live && sub == 0) {
        if (KMAX == 2 && k == 2) {                  // the common top-2 case: one 8-byte store each
            *reinterpret_cast<int2*>(topk_idx + t * 2) = make_int2(e_sel[0], e_sel[1]);
            *reinterpret_cast<float2*>(topk_w + t * 2) = make_float2(p_sel[0] / denom, p_sel[1] / denom);
        } else {
#pragma unroll
            for (int j = 0; j < KMAX; ++j)
                if (j < k) {
                    topk_idx[t * k + j] = e_sel[j];
                    topk_w[t * k + j] = p_sel[j] / denom;
                }
        }
    }
}

template <int L, int VPL, bool ALL>
static void launch_l(const float* logits, int T, int E, int k, int32_t* idx, float* w, hipStream_t s) {
    constexpr int TOK_PER_BLOCK = 256 / L;
    const unsigned grid = (unsigned)(((long long)T + TOK_PER_BLOCK - 1) / TOK_PER_BLOCK);
    if (k <= 2) hipLaunchKernelGGL((gate_kernel<L, VPL, 2, ALL>), dim3(grid), dim3(256), 0, s, logits, T, E, k, idx, w);
    else if (k <= 8) hipLaunchKernelGGL((gate_kernel<L, VPL, 8, ALL>), dim3(grid), dim3(256), 0, s, logits, T, E, k, idx, w);
    else hipLaunchKernelGGL((gate_kernel<L, VPL, MOE_MAX_TOPK, ALL>), dim3(grid), dim3(256), 0, s, logits, T, E, k, idx, w);
}

template <bool ALL>
static void launch_e(const float* logits, int T, int E, int k, int32_t* idx, float* w, hipStream_t s) {
    if (E <= 4) launch_l<1, 4, ALL>(logits, T, E, k, idx, w, s);
    else if (E <= 8) launch_l<1, 8, ALL>(logits, T, E, k, idx, w, s);
    else if (E <= 16) launch_l<2, 8, ALL>(logits, T, E, k, idx, w, s);
    else if (E <= 32) launch_l<4, 8, ALL>(logits, T, E, k, idx, w, s);
    else if (E <= 64) launch_l<4, 16, ALL>(logits, T, E, k, idx, w, s);
    else if (E <= 128) launch_l<8, 16, ALL>(logits, T, E, k, idx, w, s);
    else launch_l<16, 16, ALL>(logits, T, E, k, idx, w, s);
}

int launch_gate(const float* logits, int T, int E, int k, bool all_norm, int32_t* idx, float* w, hipStream_t s) {
    LaunchTimer timer(MOE_K_GATE, s);
    if (all_norm) launch_e<true>(logits, T, E, k, idx, w, s);
    else launch_e<false>(logits, T, E, k, idx, w, s);
    return check_launch("moe_topk_gate launch");
}

}  // namespace moe
