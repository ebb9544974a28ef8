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
#include "gate_select.h"

namespace moe {

template <int L, int VPL, int KMAX, bool ALL>
__global__ __launch_bounds__(256) void gate_kernel(const float* __restrict__ logits, int T, int E, int k,
                                                   int32_t* __restrict__ topk_idx, float* __restrict__ topk_w) {
    constexpr int TOK_PER_BLOCK = 256 / L;
    const int sub = threadIdx.x % L;
    const long long t = (long long)blockIdx.x * TOK_PER_BLOCK + threadIdx.x / L;
    const bool live = t < T;
    gate_select<L, VPL, KMAX, ALL>(logits + (live ? t : 0) * E, false, sub, live, t, E, k, topk_idx, topk_w);
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
