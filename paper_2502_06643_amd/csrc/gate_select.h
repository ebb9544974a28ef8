// The top-k selection of moe_topk_gate (paper Section 2.1) for one token whose E logits are spread over L
// neighbouring lanes of a wavefront, VPL consecutive logits per lane: shared by the gate kernel (logits
// from memory) and by the fused router (logits from LDS, where the projection left them).
#pragma once
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

// row: the token's E logits (global memory or LDS; 16-byte aligned when E % 4 == 0 or `padded`); sub = this lane's
// index among the token's L lanes; live = the token exists.  `padded`: the row holds L * VPL readable floats and the
// ones from E on are ignored (the fused router's LDS rows).  Every lane of the L-lane group must call this (shuffles);
// lane sub == 0 of a live token writes topk_idx[t][0..k) and topk_w[t][0..k).
template <int L, int VPL, int KMAX, bool ALL>
__device__ __forceinline__ void gate_select(const float* row, bool padded, int sub, bool live, long long t, int E, int k,
                                            int32_t* __restrict__ topk_idx, float* __restrict__ topk_w) {
    const int e0 = sub * VPL;
    uint32_t key[VPL];
#pragma unroll
    for (int i = 0; i < VPL; ++i) key[i] = 0u;
    if (live) {
        if (padded || (E & 3) == 0) {
#pragma unroll
            for (int c = 0; c < VPL / 4; ++c) {
                if (e0 + 4 * c < E) {
                    const float4 q = *reinterpret_cast<const float4*>(row + e0 + 4 * c);
                    key[4 * c] = orderable(q.x);
                    if (!padded || e0 + 4 * c + 1 < E) key[4 * c + 1] = orderable(q.y);
                    if (!padded || e0 + 4 * c + 2 < E) key[4 * c + 2] = orderable(q.z);
                    if (!padded || e0 + 4 * c + 3 < E) key[4 * c + 3] = orderable(q.w);
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

}  // namespace moe
