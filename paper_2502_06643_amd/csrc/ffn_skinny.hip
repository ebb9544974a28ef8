// Decode-sized batches of moe_expert_ffn_grouped (paper Section 2.2 / Fig. 2b,
// the expert FFN), bf16: a handful of rows per expert, so the two GEMMs read
// every weight once and do almost no arithmetic per byte.  The job is to keep
// HBM busy, not the matrix cores.
//
// The packed weights (moe_pack_weights) are already in matrix-instruction
// fragment order: a block of 256 columns x 64 reduction steps is 32 KB of
// sixteen 16-column panels x two 32-step halves of 1 KB, and the blocks of one
// column tile follow each other along k.  A workgroup of four wavefronts takes
// one (expert, column tile) and streams that contiguous run; each wavefront
// owns four panels (8 KB per k tile) which it loads straight into registers
// with 16-byte loads, one k tile ahead of the matrix instructions.  There is no
// LDS and no barrier: nothing ever waits for another wavefront, and the eight
// wavefronts a compute unit holds keep 64 KB of weights in flight.  The few
// activation rows are read as A fragments from global memory as well (they stay
// in L1/L2: every workgroup of an expert reads the same rows).
//
// Up projection: a wavefront's panels alternate W1/W3 (as packed), so the two
// SwiGLU factors meet in the same lane and accumulator index; H is written
// row-major as bf16.  Down projection: one column tile of one expert is 7 MB of
// weights at the Mixtral shape and there are only E * d / 256 of them, too few
// to fill the chip, so the reduction is cut into `parts` k ranges that run as
// separate workgroups and write fp32 partial sums; a small kernel adds the
// parts in a fixed order (bitwise reproducible) and rounds to bf16.
// Buckets of more than 64 rows are walked in passes of 64 rows.
#include "ffn_plan.h"

namespace moe {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kSkinnyThreads = 256;
constexpr int kSkinnyRows = 64;          // rows per pass (four 16-row fragments)
constexpr int kSkinnyMaxParts = 16;
constexpr int kSkinnyDownTasks = 512;    // workgroups the down projection is cut into

__device__ __forceinline__ bf16x8 as_frag(const uint4& q) { return __builtin_bit_cast(bf16x8, q); }

// one pass over MF * 16 rows starting at bucket row `row0`, k tiles [kt0, kt1)
template <bool UP, int MF>
__device__ __forceinline__ void skinny_pass(const uint16_t* __restrict__ A, int K, const uint4* __restrict__ Bp, int start, int n,
                                            int row0, int kt0, int kt1, int nt, int wave, int lane, int ldc,
                                            uint16_t* __restrict__ H, float* __restrict__ partial) {
    f32x4 acc[MF][4];
#pragma unroll
    for (int m = 0; m < MF; ++m)
#pragma unroll
        for (int p = 0; p < 4; ++p)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[m][p][v] = 0.f;

    // A fragment of row block m: lane l holds row l % 16 and the 8 consecutive k that start at 8 * (l / 16);
    // rows past the bucket's end re-read its last row (their results are never stored)
    const uint4* Ap[MF];
#pragma unroll
    for (int m = 0; m < MF; ++m) {
        const int r = min(row0 + m * 16 + (lane & 15), n - 1);
        Ap[m] = reinterpret_cast<const uint4*>(A + (size_t)(start + r) * K) + (lane >> 4);
    }
    uint4 a[2][MF * 2], b[2][8];
    auto load = [&](int kt, int buf) {
        const uint4* bp = Bp + (size_t)kt * 2048;                  // 32 KB block of this k tile, in 16-byte units
#pragma unroll
        for (int i = 0; i < 8; ++i) b[buf][i] = bp[i * 64];        // panel i / 2, half i % 2
#pragma unroll
        for (int m = 0; m < MF; ++m) {
            a[buf][m * 2] = Ap[m][kt * 8];
            a[buf][m * 2 + 1] = Ap[m][kt * 8 + 4];
        }
    };
    auto multiply = [&](int buf) {
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int p = 0; p < 4; ++p)
#pragma unroll
                for (int m = 0; m < MF; ++m)
                    acc[m][p] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_frag(a[buf][m * 2 + ks]), as_frag(b[buf][p * 2 + ks]),
                                                                        acc[m][p], 0, 0, 0);
    };
    load(kt0, 0);
    int kt = kt0;
    for (; kt + 2 <= kt1; kt += 2) {
        load(kt + 1, 1);
        multiply(0);
        if (kt + 2 < kt1) load(kt + 2, 0);
        multiply(1);
    }
    if (kt < kt1) multiply(0);

    // accumulator v of a fragment: row 4 * (lane / 16) + v, column lane % 16
#pragma unroll
    for (int m = 0; m < MF; ++m)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int r = row0 + m * 16 + 4 * (lane >> 4) + v;
            if (r >= n) continue;
            if (UP) {
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const int col = nt * 128 + wave * 32 + j * 16 + (lane & 15);
                    const float u = acc[m][2 * j][v], g = acc[m][2 * j + 1][v];
                    const float hv = u * __builtin_amdgcn_rcpf(1.0f + __expf(-u)) * g;    // silu(u) * g
                    if (col < ldc) H[(size_t)(start + r) * ldc + col] = __builtin_bit_cast(uint16_t, (__bf16)hv);
                }
            } else {
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    const int col = nt * 256 + wave * 64 + p * 16 + (lane & 15);
                    if (col < ldc) partial[(size_t)(start + r) * ldc + col] = acc[m][p][v];
                }
            }
        }
}

// UP:   task = (listed expert, column tile);            writes H [N, f] bf16
// DOWN: task = (listed expert, column tile, k part);    writes partial [parts][N, d] fp32
template <bool UP>
__global__ __launch_bounds__(kSkinnyThreads, 2) void ffn_skinny_kernel(const uint16_t* __restrict__ A, const uint16_t* __restrict__ Wp,
                                                                    size_t expert_stride, int K, int NT, int ldc,
                                                                    const int32_t* __restrict__ plan, uint16_t* __restrict__ H,
                                                                    float* __restrict__ partial, int parts, int N) {
    int task = blockIdx.x;
    const int part = UP ? 0 : task % parts;
    if (!UP) task /= parts;
    const int nt = task % NT, i = task / NT;
    if (i >= plan[0]) return;
    const int e = plan[kPlanExpert + i], start = plan[kPlanStart + i], n = plan[kPlanCount + i];
    const int KT = K / 64;
    const int kt0 = UP ? 0 : (int)((long long)part * KT / parts), kt1 = UP ? KT : (int)((long long)(part + 1) * KT / parts);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // this wavefront's four panels (8 pieces of 1 KB) of k tile 0 of the column tile
    const uint4* Bp = reinterpret_cast<const uint4*>(Wp + (size_t)e * expert_stride + (size_t)nt * ((size_t)K * 256)) + wave * 512 + lane;
    float* my_partial = UP ? nullptr : partial + (size_t)part * N * ldc;
    for (int row0 = 0; row0 < n; row0 += kSkinnyRows) {
        const int mf = (min(kSkinnyRows, n - row0) + 15) >> 4;
        if (mf == 1) skinny_pass<UP, 1>(A, K, Bp, start, n, row0, kt0, kt1, nt, wave, lane, ldc, H, my_partial);
        else if (mf == 2) skinny_pass<UP, 2>(A, K, Bp, start, n, row0, kt0, kt1, nt, wave, lane, ldc, H, my_partial);
        else if (mf == 3) skinny_pass<UP, 3>(A, K, Bp, start, n, row0, kt0, kt1, nt, wave, lane, ldc, H, my_partial);
        else skinny_pass<UP, 4>(A, K, Bp, start, n, row0, kt0, kt1, nt, wave, lane, ldc, H, my_partial);
    }
}

// out[row] = bf16(sum over parts, in part order) for the rows of the listed buckets; one workgroup per row
__global__ __launch_bounds__(256) void ffn_skinny_reduce_kernel(const float* __restrict__ partial, int parts, int N, int d,
                                                                const int32_t* __restrict__ plan, uint16_t* __restrict__ out) {
    const int row = blockIdx.x;
    const int n_listed = plan[0];
    bool listed = false;
    for (int i = 0; i < n_listed; ++i) {
        const int st = plan[kPlanStart + i];
        listed |= row >= st && row < st + plan[kPlanCount + i];
    }
    if (!listed) return;
    for (int c = threadIdx.x * 4; c < d; c += 1024) {
        float4 s = *reinterpret_cast<const float4*>(partial + (size_t)row * d + c);
        for (int p = 1; p < parts; ++p) {
            const float4 t = *reinterpret_cast<const float4*>(partial + ((size_t)p * N + row) * d + c);
            s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
        }
        ushort4 o;
        o.x = __builtin_bit_cast(uint16_t, (__bf16)s.x); o.y = __builtin_bit_cast(uint16_t, (__bf16)s.y);
        o.z = __builtin_bit_cast(uint16_t, (__bf16)s.z); o.w = __builtin_bit_cast(uint16_t, (__bf16)s.w);
        *reinterpret_cast<ushort4*>(out + (size_t)row * d + c) = o;
    }
}


// E row groups; plan has been built.  H [N, f] bf16 and the fp32 partial area (scratch_bytes) come from the workspace.
int launch_ffn_skinny(const void* a, int N, int d, int f, int E, const void* packed, size_t s13, size_t expert_stride,
                      const int32_t* plan, void* H, float* partial, size_t scratch_bytes, void* out, hipStream_t s) {
    const int nt_up = (int)(round_up((size_t)2 * f, 256) / 256), nt_down = (int)(round_up((size_t)d, 256) / 256);
    const uint16_t* Wp = (const uint16_t*)packed;
    int rc;
    {
        LaunchTimer timer(MOE_K_FFN_UP, s);
        hipLaunchKernelGGL(ffn_skinny_kernel<true>, dim3((unsigned)(E * nt_up)), dim3(kSkinnyThreads), 0, s, (const uint16_t*)a, Wp,
                           expert_stride, d, nt_up, f, plan, (uint16_t*)H, (float*)nullptr, 1, N);
        if ((rc = check_launch("moe_expert_ffn_grouped up launch (small batch)")) != MOE_OK) return rc;
    }
    // k parts of the down projection: two workgroups per compute unit (more, shorter parts were slower), at least 8 k tiles each
    int parts = (kSkinnyDownTasks + E * nt_down - 1) / (E * nt_down);
    parts = parts < 1 ? 1 : (parts > kSkinnyMaxParts ? kSkinnyMaxParts : parts);
    while (parts > 1 && ((f / 64) / parts < 8 || (size_t)parts * N * d * sizeof(float) > scratch_bytes)) --parts;
    if ((size_t)parts * N * d * sizeof(float) > scratch_bytes)
        return fail(MOE_ERR_WORKSPACE, "moe_expert_ffn_grouped: partial sums of %d rows x %d do not fit the workspace", N, d);
    {
        LaunchTimer timer(MOE_K_FFN_DOWN, s);
        hipLaunchKernelGGL(ffn_skinny_kernel<false>, dim3((unsigned)(E * nt_down * parts)), dim3(kSkinnyThreads), 0, s,
                           (const uint16_t*)H, Wp + s13, expert_stride, f, nt_down, d, plan, (uint16_t*)nullptr, partial, parts, N);
        if ((rc = check_launch("moe_expert_ffn_grouped down launch (small batch)")) != MOE_OK) return rc;
        hipLaunchKernelGGL(ffn_skinny_reduce_kernel, dim3((unsigned)N), dim3(256), 0, s, partial, parts, N, d, plan, (uint16_t*)out);
        if ((rc = check_launch("moe_expert_ffn_grouped reduce launch (small batch)")) != MOE_OK) return rc;
    }
    return MOE_OK;
}

}  // namespace moe
