// moe_combine: gate-weighted un-permute of the expert outputs (the step after
// the second all-to-all in the paper's Fig. 2b).
//
// Gather form: one thread owns one 16-byte unit of an output row y[t] and walks
// the token's k routes in ascending j, so the fp32 sum has a fixed order and no
// atomics are needed.  Routes whose expert is not on local_gpu are skipped;
// a token with no local route writes zeros.
#include "common.h"

namespace moe {

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xFFFF0000u); }

// two fp32 -> packed bf16 pair, round to nearest even (finite inputs)
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
    uint32_t ua = __float_as_uint(a), ub = __float_as_uint(b);
    ua += 0x7FFFu + ((ua >> 16) & 1u);
    ub += 0x7FFFu + ((ub >> 16) & 1u);
    return (ua >> 16) | (ub & 0xFFFF0000u);
}

template <bool BF16>
__global__ __launch_bounds__(256) void combine_kernel(const uint4* __restrict__ ffn_out, const int32_t* __restrict__ inv_perm,
                                                      const int32_t* __restrict__ topk_idx, const float* __restrict__ topk_w,
                                                      const int32_t* __restrict__ placement, int local_gpu,
                                                      long long total_units, int units_per_row, int E, int k, int N,
                                                      uint4* __restrict__ y) {
    const long long u = (long long)blockIdx.x * 256 + threadIdx.x;
    if (u >= total_units) return;
    const long long t = u / units_per_row;
    const int c = (int)(u - t * units_per_row);
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int j = 0; j < k; ++j) {
        const long long r = t * k + j;
        if (local_gpu >= 0) {
            const int e = topk_idx[r];
            if ((unsigned)e >= (unsigned)E || placement[e] != local_gpu) continue;
        }
        const int p = inv_perm[r];
        if ((unsigned)p >= (unsigned)N) continue;
        const float w = topk_w[r];
        const uint4 v = ffn_out[(long long)p * units_per_row + c];
        if (BF16) {
            acc[0] = fmaf(w, bf16_lo(v.x), acc[0]); acc[1] = fmaf(w, bf16_hi(v.x), acc[1]);
            acc[2] = fmaf(w, bf16_lo(v.y), acc[2]); acc[3] = fmaf(w, bf16_hi(v.y), acc[3]);
            acc[4] = fmaf(w, bf16_lo(v.z), acc[4]); acc[5] = fmaf(w, bf16_hi(v.z), acc[5]);
            acc[6] = fmaf(w, bf16_lo(v.w), acc[6]); acc[7] = fmaf(w, bf16_hi(v.w), acc[7]);
        } else {
            acc[0] = fmaf(w, __uint_as_float(v.x), acc[0]); acc[1] = fmaf(w, __uint_as_float(v.y), acc[1]);
            acc[2] = fmaf(w, __uint_as_float(v.z), acc[2]); acc[3] = fmaf(w, __uint_as_float(v.w), acc[3]);
        }
    }
    uint4 o;
    if (BF16) {
        o.x = pack_bf16(acc[0], acc[1]); o.y = pack_bf16(acc[2], acc[3]);
        o.z = pack_bf16(acc[4], acc[5]); o.w = pack_bf16(acc[6], acc[7]);
    } else {
        o.x = __float_as_uint(acc[0]); o.y = __float_as_uint(acc[1]);
        o.z = __float_as_uint(acc[2]); o.w = __float_as_uint(acc[3]);
    }
    y[u] = o;
}

// Wide rows: one workgroup per token (four tokens per workgroup, one per wavefront, when a row is at most
// 4 KB).  The token's k routes (expert, sorted position, weight) are wave-uniform, so they are read once with
// scalar loads, and every thread then has its k row gathers in flight at the same time.
template <bool BF16, int UNITS_PER_THREAD, int TOKENS_PER_GROUP>
__global__ __launch_bounds__(256) void combine_token_kernel(const uint4* __restrict__ ffn_out, const int32_t* __restrict__ inv_perm,
                                                            const int32_t* __restrict__ topk_idx, const float* __restrict__ topk_w,
                                                            const int32_t* __restrict__ placement, int local_gpu,
                                                            int units_per_row, int E, int k, int N, int T,
                                                            uint4* __restrict__ y) {
    // TOKENS_PER_GROUP tokens per workgroup, each on 256 / TOKENS_PER_GROUP threads (whole wavefronts, so the
    // token stays wave-uniform): short rows would otherwise make workgroups of one 4 KB row each, and the
    // rate at which workgroups start then bounds the kernel
    constexpr int TPT = 256 / TOKENS_PER_GROUP;
    static_assert(TPT % 64 == 0, "a token owns whole wavefronts");
    const long long t = (long long)blockIdx.x * TOKENS_PER_GROUP + __builtin_amdgcn_readfirstlane(threadIdx.x / TPT);
    if (t >= T) return;
    const int c0 = threadIdx.x % TPT;
    float acc[UNITS_PER_THREAD][8];
#pragma unroll
    for (int i = 0; i < UNITS_PER_THREAD; ++i)
#pragma unroll
        for (int q = 0; q < 8; ++q) acc[i][q] = 0.f;
    auto add_row = [&](int p, float w) {
        const uint4* row = ffn_out + (long long)p * units_per_row;
        uint4 v[UNITS_PER_THREAD];
#pragma unroll
        for (int i = 0; i < UNITS_PER_THREAD; ++i) {
            const int c = c0 + i * TPT;
            v[i] = (c < units_per_row) ? row[c] : make_uint4(0u, 0u, 0u, 0u);
        }
#pragma unroll
        for (int i = 0; i < UNITS_PER_THREAD; ++i) {
            if (BF16) {
                acc[i][0] = fmaf(w, bf16_lo(v[i].x), acc[i][0]); acc[i][1] = fmaf(w, bf16_hi(v[i].x), acc[i][1]);
                acc[i][2] = fmaf(w, bf16_lo(v[i].y), acc[i][2]); acc[i][3] = fmaf(w, bf16_hi(v[i].y), acc[i][3]);
                acc[i][4] = fmaf(w, bf16_lo(v[i].z), acc[i][4]); acc[i][5] = fmaf(w, bf16_hi(v[i].z), acc[i][5]);
                acc[i][6] = fmaf(w, bf16_lo(v[i].w), acc[i][6]); acc[i][7] = fmaf(w, bf16_hi(v[i].w), acc[i][7]);
            } else {
                acc[i][0] = fmaf(w, __uint_as_float(v[i].x), acc[i][0]); acc[i][1] = fmaf(w, __uint_as_float(v[i].y), acc[i][1]);
                acc[i][2] = fmaf(w, __uint_as_float(v[i].z), acc[i][2]); acc[i][3] = fmaf(w, __uint_as_float(v[i].w), acc[i][3]);
            }
        }
    };
    if (k <= 8 && local_gpu < 0) {
        // every expert resident: the token's positions and weights are all fetched before any is used
        // (independent wave-uniform loads instead of a dependent chain per route)
        int p[8];
        float w[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            p[j] = (j < k) ? inv_perm[t * k + j] : -1;
            w[j] = (j < k) ? topk_w[t * k + j] : 0.f;
        }
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if ((unsigned)p[j] < (unsigned)N) add_row(p[j], w[j]);
    } else if (k <= 8) {
        // a resident subset of the experts: the token's k expert ids, positions and weights, then the k
        // owners, are fetched as two rounds of independent wave-uniform loads; only the routes that turn out
        // to be local (one in G on average) go on to their row
        int ex[8], owner[8], p[8];
        float w[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            ex[j] = (j < k) ? topk_idx[t * k + j] : -1;
            p[j] = (j < k) ? inv_perm[t * k + j] : -1;
            w[j] = (j < k) ? topk_w[t * k + j] : 0.f;
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) owner[j] = ((unsigned)ex[j] < (unsigned)E) ? placement[ex[j]] : -1;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if (j >= k || owner[j] != local_gpu) continue;
            if ((unsigned)p[j] >= (unsigned)N) continue;
            add_row(p[j], w[j]);
        }
    } else {
        for (int j = 0; j < k; ++j) {
            const long long r = t * k + j;
            if (local_gpu >= 0) {
                const int ex = topk_idx[r];
                if ((unsigned)ex >= (unsigned)E || placement[ex] != local_gpu) continue;
            }
            const int p = inv_perm[r];
            if ((unsigned)p >= (unsigned)N) continue;
            add_row(p, topk_w[r]);
        }
    }
#pragma unroll
    for (int i = 0; i < UNITS_PER_THREAD; ++i) {
        const int c = c0 + i * TPT;
        if (c >= units_per_row) break;
        uint4 o;
        if (BF16) {
            o.x = pack_bf16(acc[i][0], acc[i][1]); o.y = pack_bf16(acc[i][2], acc[i][3]);
            o.z = pack_bf16(acc[i][4], acc[i][5]); o.w = pack_bf16(acc[i][6], acc[i][7]);
        } else {
            o.x = __float_as_uint(acc[i][0]); o.y = __float_as_uint(acc[i][1]);
            o.z = __float_as_uint(acc[i][2]); o.w = __float_as_uint(acc[i][3]);
        }
        y[t * units_per_row + c] = o;
    }
}

int launch_combine(const void* ffn_out, moe_dtype_t dt, const int32_t* inv_perm, const int32_t* topk_idx,
                   const float* topk_w, const int32_t* placement, int local_gpu, int T, int d, int E, int k,
                   void* y, hipStream_t s) {
    const int units_per_row = d * elt_bytes(dt) / 16;
    const long long total_units = (long long)T * units_per_row;
    const long long grid = (total_units + 255) / 256;
    if (grid > 0x7FFFFFFFll) return fail(MOE_ERR_UNSUPPORTED, "moe_combine: T*d too large for one launch");
    LaunchTimer timer(MOE_K_COMBINE, s);
    const bool bf = dt == MOE_BF16;
#define MOE_LAUNCH_TOKEN(BF, UPT, TPG)                                                                                  \
    hipLaunchKernelGGL((combine_token_kernel<BF, UPT, TPG>), dim3((unsigned)((T + TPG - 1) / TPG)), dim3(256), 0, s,      \
                       (const uint4*)ffn_out, inv_perm, topk_idx, topk_w, placement, local_gpu, units_per_row, E, k, T * k, T, \
                       (uint4*)y)
    if (units_per_row >= 192 && units_per_row <= 256) {
        if (bf) MOE_LAUNCH_TOKEN(true, 4, 4); else MOE_LAUNCH_TOKEN(false, 4, 4);
    } else if (units_per_row > 256 && units_per_row <= 512) {
        if (bf) MOE_LAUNCH_TOKEN(true, 2, 1); else MOE_LAUNCH_TOKEN(false, 2, 1);
    } else if (units_per_row > 512 && units_per_row <= 1024) {
        if (bf) MOE_LAUNCH_TOKEN(true, 4, 1); else MOE_LAUNCH_TOKEN(false, 4, 1);
    } else if (bf) {
        hipLaunchKernelGGL(combine_kernel<true>, dim3((unsigned)grid), dim3(256), 0, s, (const uint4*)ffn_out, inv_perm, topk_idx,
                           topk_w, placement, local_gpu, total_units, units_per_row, E, k, T * k, (uint4*)y);
    } else {
        hipLaunchKernelGGL(combine_kernel<false>, dim3((unsigned)grid), dim3(256), 0, s, (const uint4*)ffn_out, inv_perm, topk_idx,
                           topk_w, placement, local_gpu, total_units, units_per_row, E, k, T * k, (uint4*)y);
    }
#undef MOE_LAUNCH_TOKEN
    return check_launch("moe_combine launch");
}

}  // namespace moe
