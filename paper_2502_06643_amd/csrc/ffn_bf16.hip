// bf16 path of moe_expert_ffn_grouped (paper Section 2.2 / Fig. 2b: the expert
// FFN, whose per-GPU cost is what the placement ILP 1 balances) as two grouped
// GEMMs on the gfx950 matrix cores:
//   up  : H   = silu(A W1_e) * (A W3_e)   [rows, f]  bf16, fp32 accumulate
//   down: out = H W2_e                    [rows, d]  bf16, fp32 accumulate
//
// Weights are pre-packed (moe_pack_weights) in MFMA fragment order: the matrix
// is cut into panels of 32 output columns; a panel is stored k-block after
// k-block, one k-block being 16 reduction steps x 32 columns = 1 KB, inside
// which lane l of a wavefront owns 8 consecutive k of column l % 32 starting at
// k = 8 * (l / 32).  That is exactly the B operand of
// v_mfma_f32_32x32x16_bf16, so a tile of weights is a straight 16-byte-per-lane
// copy from memory to LDS to registers.  For the up projection the panels of
// W1 and W3 alternate (W1 cols 0-31, W3 cols 0-31, W1 cols 32-63, ...), so the
// two factors of the SwiGLU product sit in the same lane and register index.
//
// Activations stay row-major; their LDS tile is [rows][64 k] with the 16-byte
// chunks of a row XOR-swizzled by (row >> 1) & 7, which makes both the
// row-contiguous stores and the column-of-rows fragment loads conflict-free.
//
// Work decomposition: a workgroup (4 wavefronts, 2 x 2) owns one BM x BN output
// tile of one expert; the (expert, row tile) list comes from the device-side
// plan.  Tile ids are dealt to the 8 XCDs in contiguous ranges (workgroup ids
// round-robin over XCDs), ordered expert -> column tile -> row tile, so that
// workgroups sharing an L2 share weight panels and activation rows.
#include "ffn_plan.h"

namespace moe {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int BK = 64;                 // reduction steps per LDS tile
constexpr int kPanelCols = 32;
constexpr int kNPad = 256;             // packed column count is padded to this

static inline size_t npad13(int f) { return round_up((size_t)2 * f, kNPad); }
static inline size_t npad2(int d) { return round_up((size_t)d, kNPad); }

size_t packed_bytes_bf16(int E, int d, int f) {
    return (size_t)E * (npad13(f) * d + npad2(d) * f) * 2;
}

// One thread per 16-byte unit of the packed buffer.
__global__ __launch_bounds__(256) void pack_bf16_kernel(const uint16_t* __restrict__ w1, const uint16_t* __restrict__ w3,
                                                        const uint16_t* __restrict__ w2, int d, int f,
                                                        long long units13, long long units2, long long total,
                                                        uint4* __restrict__ packed) {
    const long long o = (long long)blockIdx.x * 256 + threadIdx.x;
    if (o >= total) return;
    const long long per_e = units13 + units2;
    const long long e = o / per_e;
    long long r = o - e * per_e;
    const uint16_t* src;
    int K, ncols, col;
    if (r < units13) {
        K = d; ncols = f;
        const long long panel = r / ((long long)K * 4);
        const int lane = (int)(r % 64);
        col = (int)(panel / 2) * kPanelCols + lane % 32;
        src = ((panel & 1) ? w3 : w1) + (size_t)e * d * f;
    } else {
        r -= units13;
        K = f; ncols = d;
        const long long panel = r / ((long long)K * 4);
        const int lane = (int)(r % 64);
        col = (int)panel * kPanelCols + lane % 32;
        src = w2 + (size_t)e * d * f;
    }
    const int kb = (int)((r % ((long long)K * 4)) / 64);
    const int lane = (int)(r % 64);
    const int k0 = kb * 16 + 8 * (lane / 32);
    uint16_t v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = (col < ncols) ? src[(size_t)(k0 + i) * ncols + col] : (uint16_t)0;
    uint4 q;
    q.x = v[0] | ((uint32_t)v[1] << 16); q.y = v[2] | ((uint32_t)v[3] << 16);
    q.z = v[4] | ((uint32_t)v[5] << 16); q.w = v[6] | ((uint32_t)v[7] << 16);
    packed[o] = q;
}

int launch_pack_bf16(const void* w1, const void* w3, const void* w2, int E, int d, int f, void* packed, hipStream_t s) {
    const long long units13 = (long long)npad13(f) * d / 8, units2 = (long long)npad2(d) * f / 8;
    const long long total = (units13 + units2) * E;
    const long long grid = (total + 255) / 256;
    if (grid > 0x7FFFFFFFll) return fail(MOE_ERR_UNSUPPORTED, "moe_pack_weights: weights too large for one launch");
    hipLaunchKernelGGL(pack_bf16_kernel, dim3((unsigned)grid), dim3(256), 0, s, (const uint16_t*)w1, (const uint16_t*)w3,
                       (const uint16_t*)w2, d, f, units13, units2, total, (uint4*)packed);
    return check_launch("moe_pack_weights launch");
}

__device__ __forceinline__ int swz(int row, int chunk) { return chunk ^ ((row >> 1) & 7); }

template <int BM, int BN, bool UP>
__global__ __launch_bounds__(256) void ffn_bf16_kernel(const uint16_t* __restrict__ A, const uint16_t* __restrict__ Wp,
                                                       size_t expert_stride, int K, int npad, uint16_t* __restrict__ C,
                                                       int ldc, const int32_t* __restrict__ plan) {
    constexpr int WTM = BM / 2, WTN = BN / 2, FM = WTM / 32, FN = WTN / 32;
    constexpr int PA = BM / 32, PB = BN / 32;       // 16-byte loads per thread and k tile
    static_assert(!UP || (FN % 2 == 0), "SwiGLU pairs need an even number of column fragments per wavefront");
    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
    uint16_t* As = smem;                 // [BM][64]
    uint16_t* Bs = smem + BM * BK;       // [PB panels][4 k-blocks][64 lanes][8]

    // ---- which tile --------------------------------------------------------
    const int32_t* prefix = plan + (UP ? kPlanTiles0 : kPlanTiles1);
    const int n_exp = plan[0];
    const int NT = npad / BN;
    const long long total = (long long)prefix[n_exp] * NT;
    const long long chunk = (total + 7) / 8;
    const long long slot = blockIdx.x / 8;
    if (slot >= chunk) return;
    const long long tile = (long long)(blockIdx.x % 8) * chunk + slot;
    if (tile >= total) return;
    int i = 0;
    while (i + 1 < n_exp && (long long)prefix[i + 1] * NT <= tile) ++i;
    const int mt_e = prefix[i + 1] - prefix[i];
    const int rem = (int)(tile - (long long)prefix[i] * NT);
    const int nt = rem / mt_e, mt = rem - nt * mt_e;
    const int expert = plan[kPlanExpert + i];
    const int row0 = plan[kPlanStart + i] + mt * BM;
    const int rows = min(BM, plan[kPlanCount + i] - mt * BM);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_m = wave >> 1, wave_n = wave & 1;

    const uint16_t* Bt = Wp + (size_t)expert * expert_stride + (size_t)nt * PB * ((size_t)K * kPanelCols);
    const size_t panel_stride = (size_t)K * kPanelCols;

    // ---- staging registers ---------------------------------------------------
    u32x4 ra[PA], rb[PB];
    const int a_row = tid >> 3, a_chunk = tid & 7;
    size_t a_off[PA];
#pragma unroll
    for (int p = 0; p < PA; ++p) {
        const int r = min(p * 32 + a_row, rows - 1);            // rows past the bucket re-read its last row
        a_off[p] = (size_t)(row0 + r) * K + a_chunk * 8;
    }
#define MOE_GLOAD(kt)                                                                                         \
    {                                                                                                         \
        _Pragma("unroll") for (int p = 0; p < PA; ++p)                                                        \
            ra[p] = *reinterpret_cast<const u32x4*>(A + a_off[p] + (size_t)(kt) * BK);                        \
        _Pragma("unroll") for (int p = 0; p < PB; ++p)                                                        \
            rb[p] = *reinterpret_cast<const u32x4*>(Bt + p * panel_stride + (size_t)(kt) * (BK * kPanelCols) + tid * 8); \
    }
#define MOE_LSTORE()                                                                                          \
    {                                                                                                         \
        _Pragma("unroll") for (int p = 0; p < PA; ++p) {                                                      \
            const int r = p * 32 + a_row;                                                                     \
            *reinterpret_cast<u32x4*>(As + r * BK + swz(r, a_chunk) * 8) = ra[p];                             \
        }                                                                                                     \
        _Pragma("unroll") for (int p = 0; p < PB; ++p)                                                        \
            *reinterpret_cast<u32x4*>(Bs + p * (BK * kPanelCols) + tid * 8) = rb[p];                          \
    }

    f32x16 acc[FM][FN];
#pragma unroll
    for (int a = 0; a < FM; ++a)
#pragma unroll
        for (int b = 0; b < FN; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    const int KT = K / BK;
    MOE_GLOAD(0)
    for (int kt = 0; kt < KT; ++kt) {
        __syncthreads();                 // everyone is done reading the previous tile
        MOE_LSTORE()
        __syncthreads();
        if (kt + 1 < KT) MOE_GLOAD(kt + 1)   // in flight while the matrix cores work
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 af[FM], bfr[FN];
#pragma unroll
            for (int a = 0; a < FM; ++a) {
                const int r = wave_m * WTM + a * 32 + (lane & 31);
                af[a] = *reinterpret_cast<const bf16x8*>(As + r * BK + swz(r, ks * 2 + (lane >> 5)) * 8);
            }
#pragma unroll
            for (int b = 0; b < FN; ++b)
                bfr[b] = *reinterpret_cast<const bf16x8*>(Bs + (wave_n * FN + b) * (BK * kPanelCols) + ks * 512 + lane * 8);
#pragma unroll
            for (int a = 0; a < FM; ++a)
#pragma unroll
                for (int b = 0; b < FN; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[a], bfr[b], acc[a][b], 0, 0, 0);
        }
    }

#undef MOE_GLOAD
#undef MOE_LSTORE

    // ---- epilogue ------------------------------------------------------------
    // accumulator v of a 32x32 fragment: row 8*(v/4) + 4*(lane/32) + v%4, column lane%32
    const int panel0 = nt * PB + wave_n * FN;
#pragma unroll
    for (int a = 0; a < FM; ++a) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int r = wave_m * WTM + a * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
            if (r >= rows) continue;
            uint16_t* crow = C + (size_t)(row0 + r) * ldc;
            if (UP) {
#pragma unroll
                for (int b = 0; b < FN; b += 2) {
                    const int col = ((panel0 + b) >> 1) * kPanelCols + (lane & 31);
                    if (col < ldc) {
                        const float u = acc[a][b][v], g = acc[a][b + 1][v];
                        const float h = u / (1.0f + __expf(-u)) * g;
                        crow[col] = __builtin_bit_cast(uint16_t, (__bf16)h);
                    }
                }
            } else {
#pragma unroll
                for (int b = 0; b < FN; ++b) {
                    const int col = (panel0 + b) * kPanelCols + (lane & 31);
                    if (col < ldc) crow[col] = __builtin_bit_cast(uint16_t, (__bf16)acc[a][b][v]);
                }
            }
        }
    }
}

template <int BM, int BN, bool UP>
static int launch_gemm(const uint16_t* A, const uint16_t* Wp, size_t expert_stride, int K, int npad, uint16_t* C, int ldc,
                       const int32_t* plan, int mt_max, hipStream_t s) {
    constexpr int smem = (BM + BN) * BK * 2;
    static bool configured = false;
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&ffn_bf16_kernel<BM, BN, UP>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        if (e != hipSuccess) return hip_fail(e, "hipFuncSetAttribute");
        configured = true;
    }
    const long long tiles = (long long)mt_max * (npad / BN);
    const long long grid = (tiles + 7) / 8 * 8;
    if (grid > 0x7FFFFFFFll) return fail(MOE_ERR_UNSUPPORTED, "moe_expert_ffn_grouped: too many tiles for one launch");
    hipLaunchKernelGGL((ffn_bf16_kernel<BM, BN, UP>), dim3((unsigned)grid), dim3(256), smem, s, A, Wp, expert_stride, K, npad, C, ldc, plan);
    return check_launch("moe_expert_ffn_grouped gemm launch");
}

int launch_ffn_bf16(const void* a, int N, int d, int f, int E, const void* packed, const int32_t* counts,
                    const int32_t* starts, const int32_t* placement, int local_gpu, void* out,
                    int32_t* plan, void* H, hipStream_t s) {
    constexpr int BM = 128, BN = 128;
    int rc = launch_ffn_plan(counts, starts, placement, local_gpu, E, N, BM, BM, plan, s);
    if (rc != MOE_OK) return rc;
    const int mt_max = (N + BM - 1) / BM + (E < N ? E : N);
    const size_t s13 = npad13(f) * d, s2 = npad2(d) * f, stride = s13 + s2;
    const uint16_t* Wp = (const uint16_t*)packed;
    {
        LaunchTimer timer(MOE_K_FFN_UP, s);
        rc = launch_gemm<BM, BN, true>((const uint16_t*)a, Wp, stride, d, (int)npad13(f), (uint16_t*)H, f, plan, mt_max, s);
        if (rc != MOE_OK) return rc;
    }
    {
        LaunchTimer timer(MOE_K_FFN_DOWN, s);
        rc = launch_gemm<BM, BN, false>((const uint16_t*)H, Wp + s13, stride, f, (int)npad2(d), (uint16_t*)out, d, plan, mt_max, s);
        if (rc != MOE_OK) return rc;
    }
    return MOE_OK;
}

}  // namespace moe
