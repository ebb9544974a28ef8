// bf16 path of moe_expert_ffn_grouped (paper Section 2.2 / Fig. 2b: the expert
// FFN, whose per-GPU cost is what the placement ILP 1 balances) as two grouped
// GEMMs on the gfx950 matrix cores:
//   up  : H   = silu(A W1_e) * (A W3_e)   [rows, f]  bf16, fp32 accumulate
//   down: out = H W2_e                    [rows, d]  bf16, fp32 accumulate
//
// Work decomposition.  A workgroup of 8 wavefronts (4 along rows x 2 along
// columns, two wavefronts per SIMD) owns one 256 x 256 output tile of one
// expert, or 384 x 256 when the resident buckets are large on average (the
// host decides when it knows them all, else the device-side plan does; one
// launch holds the code of both heights and branches on the plan's header);
// the (expert, row tile) list comes from that plan, so no bucket size ever
// reaches the host.  Workgroup ids are dealt round-robin to the 8 XCDs by the hardware;
// every XCD owns an eighth of the column tiles of every expert (a weight panel
// passes through one L2 only, and all XCDs see the same mix of experts) and
// walks them expert -> chunk of row tiles -> column tile -> row tile:
// workgroups that share an L2 share weight panels and activation rows.
// Within a tile the rows are dealt to the four wavefront rows in blocks of 32, and a wavefront skips the blocks that lie
// past the end of a ragged bucket: such a tile costs ceil(rows / 128) blocks
// per wavefront, every SIMD staying equally loaded.  Tiles of at most 128
// rows (up projection) run a three-stage loop of their own, see mainloop_small.
//
// Matrix instruction.  v_mfma_f32_16x16x32_bf16: with both operands coming from
// registers it accumulates 32 k per pass over a 16 x 16 accumulator, half the
// accumulator traffic per flop of the 32x32x16 form; under the chip's power
// limit it sustains about 10 % more flops (measured with random operands) and
// this kernel gained 4-7 % from the switch.
//
// Weights are pre-packed (moe_pack_weights) in fragment order.  The packed
// matrix is cut into blocks of 256 columns x 64 reduction steps = 32 KB, stored
// column tile after column tile, k tile after k tile, so the 32 KB a workgroup
// needs per step are contiguous.  A block holds 16 panels (16 columns) x 2
// k-blocks (32 steps) of 1 KB, in which lane l of a wavefront owns the 8
// consecutive k of column l % 16 that start at k = 8 * (l / 16): exactly the B
// operand of the instruction.  For the up projection the panels of W1 and W3
// alternate, so both factors of the SwiGLU product sit in the same lane and
// accumulator index.  Activations stay row-major; their LDS tile is
// [rows][64 k] with the eight 16-byte slots of a row XOR-swizzled by
// (row >> 1) & 7, conflict-free for the fills and for the fragment reads.
//
// Data movement.  global_load_lds_dwordx4 copies 16 bytes per lane from memory
// straight into LDS (destination = M0 + 16 * lane, one wavefront instruction
// fills 1 KB), so a tile needs no staging registers and no LDS store
// instructions; the swizzle is applied by choosing which global chunk each lane
// fetches.  Two LDS stages: the loads of k tile kt+1 are in flight while tile kt
// is multiplied, and one barrier per k tile both publishes tile kt and retires
// the stage that tile kt+1 overwrites.  With 256-row tiles the 160 KB of LDS
// hold a third weight stage: the weights (streamed from memory, the
// long-latency operand) are then fetched two k tiles ahead, the activations
// one (+4-9 % on every batch size that uses these tiles).  The loads are issued from inline
// assembly: the compiler then does not treat them as LDS writes that every
// later LDS read must wait for, and the wait is explicit (s_waitcnt vmcnt
// before the barrier).  They are issued by four of the eight wavefronts (the
// older one of each SIMD), spread between its matrix instructions, and the LDS
// fragment reads run one column ahead of the matrix instructions.  The k tile
// holds no branch: after the last k tile the loaders fetch that tile once more
// into the idle stage instead of skipping the loads.
//
// Tail balancing (down projection).  The tiles of the last, partly filled round
// on an XCD are each split along k into s parts that run as separate workgroups
// and write fp32 partial accumulators, s chosen so that the parts fill the
// compute units in the fewest, shortest rounds; a small fix-up kernel adds the
// parts in a fixed order and runs the normal epilogue.  Results stay bitwise
// reproducible.
//
// Epilogue.  Accumulators are converted to bf16 (round to nearest even),
// transposed through a per-wavefront LDS staging tile and written with
// 16-byte stores that cover whole 128-byte lines.
#include "ffn_tiles.h"
#include <mutex>

namespace moe {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;

// The workgroup tile is (128 * FM) x 256 with FM = 2 or 3 fragment rows per wavefront (template parameter).
constexpr int BN = 256, BK = 64;                // tile width and k depth of one LDS stage
constexpr int WM = 4, WN = 2, NW = WM * WN;     // wavefront grid
constexpr int WTN = BN / WN;                    // 128 columns per wavefront
constexpr int FN = WTN / 16;                    // 8 column fragments of 16
constexpr int NS = 2;                           // LDS stages
constexpr int kDmaEvery = 4;                    // matrix instructions between two direct-to-LDS loads of the next k tile
constexpr int KB = BK / 32;                     // k steps of one matrix instruction per stage
constexpr int B_CHUNKS = BN / 8;                // 1 KB pieces of the weight tile per stage
constexpr int B_PER_WAVE = B_CHUNKS / NW;
constexpr int kThreads = NW * 64;
template <int FM> struct Tile {
    static constexpr int WTM = 32 * FM, BM = WM * WTM;
    // LDS of the main loop: NS activation stages, then NSB weight stages.  With 256-row tiles a third weight
    // stage fits (64 + 96 KB): the weights, which come from memory and are the long-latency operand, are then
    // fetched two k tiles ahead and the activations one
    static constexpr int NSB = FM == 2 ? 3 : 2;
    static constexpr int A_STAGE = BM * BK, B_STAGE = BN * BK;           // elements
    static constexpr int LOOP_ELEMS = NS * A_STAGE + NSB * B_STAGE;
    static constexpr int A_CHUNKS = BM / 8, A_PER_WAVE = A_CHUNKS / NW;
    static constexpr size_t kPartialFloats = (size_t)BM * BN;
};
constexpr int kPanelCols = 16;
constexpr size_t kMaxPartialFloats = (size_t)384 * BN;          // one fp32 partial tile of the largest tile

static inline size_t npad13(int f) { return round_up((size_t)2 * f, BN); }
static inline size_t npad2(int d) { return round_up((size_t)d, BN); }

size_t packed_bytes_bf16(int E, int d, int f) {
    return (size_t)E * (npad13(f) * d + npad2(d) * f) * 2;
}

// fp32 partial tiles for the split tail of the down projection: two slots per compute unit
size_t ffn_bf16_scratch_bytes() { return (size_t)kXcds * 2 * kMaxCusPerXcd * kMaxPartialFloats * sizeof(float); }

// One thread per 16-byte unit of the packed buffer.  Unit index within one matrix of one expert:
// (((nt * KT + kt) * 16 + panel) * 2 + kb) * 64 + lane.
__global__ __launch_bounds__(256) void pack_bf16_kernel(const uint16_t* __restrict__ w1, const uint16_t* __restrict__ w3,
                                                        const uint16_t* __restrict__ w2, int d, int f,
                                                        long long units13, long long units2, long long total,
                                                        uint4* __restrict__ packed) {
    const long long o = (long long)blockIdx.x * 256 + threadIdx.x;
    if (o >= total) return;
    const long long per_e = units13 + units2;
    const long long e = o / per_e;
    long long r = o - e * per_e;
    const bool up = r < units13;
    if (!up) r -= units13;
    const int K = up ? d : f, ncols = up ? f : d;
    const int KT = K / BK;
    const int lane = (int)(r & 63);
    const int kb = (int)((r >> 6) & 1);
    const int p = (int)((r >> 7) & 15);
    const long long tile = r >> 11;                 // nt * KT + kt
    const int kt = (int)(tile % KT);
    const long long panel = (tile / KT) * 16 + p;   // 16-column panel of the (interleaved) matrix
    const uint16_t* src;
    int col;
    if (up) {
        col = (int)(panel / 2) * kPanelCols + lane % 16;
        src = ((panel & 1) ? w3 : w1) + (size_t)e * d * f;
    } else {
        col = (int)panel * kPanelCols + lane % 16;
        src = w2 + (size_t)e * d * f;
    }
    const int k0 = kt * BK + kb * 32 + 8 * (lane / 16);
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

// ---------------------------------------------------------------------------
// pieces of the GEMM
// ---------------------------------------------------------------------------
// M0 (the LDS destination) is written here without being declared clobbered: the compiler reserves M0, never
// keeps a value of its own in it across statements and rejects it on a clobber list; it writes M0 itself only
// right in front of an instruction that reads it implicitly (indirect register indexing, which these kernels
// avoid: every register-array index is a compile-time constant).
__device__ __forceinline__ void dma16(uint32_t voff, const void* sbase, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1\n"
                 :: "v"(voff), "s"(sbase), "s"(lds_addr) : "memory");
}

__device__ __forceinline__ int swz(int row, int chunk) { return chunk ^ ((row >> 1) & 7); }

// Rows of a tile are dealt to the four wavefront rows in blocks of 32 (two 16-row fragments): block j of
// wavefront row m covers tile rows 32 * (4j + m) .. +31.  A ragged tile of r rows then keeps every SIMD
// equally busy and costs ceil(r / 128) blocks of matrix work per wavefront instead of the whole tile.
__device__ __forceinline__ int block_row(int j, int wave_m) { return (j * WM + wave_m) * 32; }
__device__ __forceinline__ int active_blocks(int rows, int wave_m, int fm) {
    const int n = (rows - wave_m * 32 + 32 * WM - 1) / (32 * WM);
    return n < 0 ? 0 : (n > fm ? fm : n);
}

// What a loading wavefront needs to fetch its share of a k tile: per-lane byte offsets of its 1 KB
// pieces (the k tile moves the scalar base) and the LDS address of its first piece in stage 0.
// Only the first NL wavefronts of a workgroup (one per SIMD, the older of its two) issue the loads.  The
// SIMD gives its older wavefront the issue slot whenever both are ready, so the younger one runs its
// matrix instructions late in the k tile; loads placed in its instruction stream start late too, and a
// wavefront waiting to issue a load holds back its own matrix instructions.  With all twenty pieces of a
// k tile in the older wavefronts' streams both projections gained 2-3 %; the younger four as loaders
// lost 10 %, two loaders instead of four 25 %.
// A loader's activation pieces are 8-row chunks NL * 8 rows apart: their per-lane offsets differ by a
// constant (the swizzle term of a row depends on the chunk's parity only, which NL = 4 preserves), so one
// offset register serves all of them; offsets past the bucket's last row are clamped into that row.
constexpr int NL = 4;
template <int FM>
struct Loader {
    static constexpr int A_PER_L = Tile<FM>::A_CHUNKS / NL, B_PER_L = B_CHUNKS / NL;
    uint32_t a_voff0, a_vmax, a_step, b_voff0;
    const uint16_t* Abase;
    const uint16_t* Bbase;
    uint32_t lds;
    static constexpr int N_DMA = A_PER_L + B_PER_L;
    // piece j of a k tile: an activation piece of tile kta into activation stage sa, or a weight piece of
    // tile ktb into weight stage sb
    __device__ __forceinline__ void issue(int j, int kta, int ktb, int sa, int sb) const {
        if (j < A_PER_L)
            dma16(min(a_voff0 + (uint32_t)j * a_step, a_vmax), Abase + (size_t)kta * BK,
                  lds + (uint32_t)sa * (Tile<FM>::A_STAGE * 2) + j * NL * 1024);
        else
            dma16(b_voff0, Bbase + (size_t)ktb * (BK * BN) + (size_t)(j - A_PER_L) * (NL * 512),
                  lds + (uint32_t)(NS * Tile<FM>::A_STAGE * 2) + (uint32_t)sb * (Tile<FM>::B_STAGE * 2) + (j - A_PER_L) * NL * 1024);
    }
};

// One k tile of matrix instructions for a wavefront with NF active 32-row blocks (2 NF fragment rows
// of v_mfma_f32_16x16x32_bf16).  With `load`, the pieces of the next k tile are issued one at a time
// between groups of kDmaEvery matrix instructions: the memory pipeline takes 16 cycles per 1 KB piece,
// and a wavefront that issues its pieces back to back sits in the issue stage for that long while its
// matrix instructions wait behind them.  Pieces that find no slot (few active blocks) go first.
//
// Fragments are streamed: the weight fragment of the next column is read while the current column
// multiplies, and each activation fragment of the next 32 k is read into place right after its last
// use, so that a matrix instruction rarely waits for LDS.  The schedule is pinned.
template <int FM, int NF, bool LOADER>
__device__ __forceinline__ void ktile(f32x4 (&acc)[2 * FM][FN], const uint16_t* As, const uint16_t* Bs, const Loader<FM>& ld,
                                      int kta, int ktb, int sa, int sb, int wave_m, int wave_n, int lane) {
    constexpr int N_DMA = Loader<FM>::N_DMA, NR = 2 * NF;
    constexpr int SLOTS = KB * NR * FN / kDmaEvery;
    constexpr int UPFRONT = N_DMA > SLOTS ? N_DMA - SLOTS : 0;
    // kta / ktb are the k tiles to fetch (into stages sa / sb), clamped to the last one: near the end the
    // last tile is fetched again into an idle stage, so the stream of matrix instructions holds no branch at
    // all, which is worth more than the redundant pieces cost
    if (LOADER && UPFRONT > 0) {
#pragma unroll
        for (int j = 0; j < UPFRONT; ++j) ld.issue(j, kta, ktb, sa, sb);
    }
    // A operand: lane l holds row l % 16 and the 8 consecutive k that start at 8 * (l / 16)
    auto read_a = [&](int a, int ks) {
        const int r = block_row(a >> 1, wave_m) + (a & 1) * 16 + (lane & 15);
        return *reinterpret_cast<const bf16x8*>(As + r * BK + swz(r, ks * 4 + (lane >> 4)) * 8);
    };
    auto read_b = [&](int b, int ks) {
        return *reinterpret_cast<const bf16x8*>(Bs + ((wave_n * FN + b) * KB + ks) * 512 + lane * 8);
    };
    bf16x8 af[NR], bq[2];
    bq[0] = read_b(0, 0);                                    // the first matrix instruction needs only bq[0] and af[0]
#pragma unroll
    for (int a = 0; a < NR; ++a) {
        af[a] = read_a(a, 0);
        __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int ks = 0; ks < KB; ++ks) {
#pragma unroll
        for (int b = 0; b < FN; ++b) {
            const int c = ks * FN + b;
            if (b + 1 < FN) bq[(c + 1) & 1] = read_b(b + 1, ks);
            else if (ks + 1 < KB) bq[(c + 1) & 1] = read_b(0, ks + 1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int a = 0; a < NR; ++a) {
                acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[a], bq[c & 1], acc[a][b], 0, 0, 0);
                if (b == FN - 1 && ks + 1 < KB) af[a] = read_a(a, ks + 1);
                const int m = c * NR + a;
                __builtin_amdgcn_sched_barrier(0);
                if (LOADER && m % kDmaEvery == kDmaEvery - 1 && UPFRONT + m / kDmaEvery < N_DMA) {
                    ld.issue(UPFRONT + m / kDmaEvery, kta, ktb, sa, sb);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
    }
}

// the k loop of a wavefront with NF active 32-row blocks (NF = 0: it only fetches its share of the tiles)
template <int FM, int NF, bool LOADER>
__device__ __forceinline__ void kloop(f32x4 (&acc)[2 * FM][FN], const uint16_t* smem, const Loader<FM>& ld, const WorkItem& w,
                                      int wave_m, int wave_n, int lane) {
    constexpr int NSB = Tile<FM>::NSB, A_STAGE = Tile<FM>::A_STAGE, B_STAGE = Tile<FM>::B_STAGE, N_DMA = Loader<FM>::N_DMA;
    static_assert(Loader<FM>::B_PER_L == 8, "the wait below leaves eight weight pieces in flight");
    const uint16_t* smem_b = smem + NS * A_STAGE;
    const int last = w.kt1 - 1;
    int sa = 0, sb = 0;
    for (int kt = w.kt0; kt < w.kt1; ++kt) {
        // this wavefront's pieces of tile kt have landed; with three weight stages its (in-order) weight
        // pieces of tile kt+1, issued last, may still be in flight
        if (NSB == 3) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();                                     // everyone's have, and tile kt-1 has been consumed
        const int kta = min(kt + 1, last), ktb = min(kt + NSB - 1, last);
        const int sa_next = sa ^ 1, sb_next = sb == 0 ? NSB - 1 : sb - 1;      // (sb + NSB - 1) % NSB: the stage of tile kt-1
        if (NF > 0) {
            ktile<FM, (NF > 0 ? NF : 1), LOADER>(acc, smem + sa * A_STAGE, smem_b + sb * B_STAGE, ld, kta, ktb, sa_next, sb_next,
                                                 wave_m, wave_n, lane);
        } else if (LOADER) {
#pragma unroll
            for (int j = 0; j < N_DMA; ++j) ld.issue(j, kta, ktb, sa_next, sb_next);
        }
        sa = sa_next;
        sb = sb + 1 == NSB ? 0 : sb + 1;
    }
}

// acc += A[row0 .. row0+rows, k tiles kt0..kt1) * B(tile), everything through LDS
template <int FM>
__device__ __forceinline__ void mainloop(f32x4 (&acc)[2 * FM][FN], uint16_t* smem, const uint16_t* __restrict__ A,
                                         const uint16_t* __restrict__ Bbase, int K, const WorkItem& w, int wave, int lane,
                                         int nfrag) {
    constexpr int N_DMA = Loader<FM>::N_DMA;
    const int wave_m = wave / WN, wave_n = wave % WN;
    Loader<FM> ld;
    ld.Abase = A + (size_t)w.row0 * K;
    ld.Bbase = Bbase + (size_t)(wave % NL) * 512;
    ld.lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)smem + (uint32_t)(wave % NL) * 1024u;
    {
        const int r = (wave % NL) * 8 + (lane >> 3);
        ld.a_voff0 = (uint32_t)r * (uint32_t)K * 2u + (uint32_t)swz(r, lane & 7) * 16u;
        ld.a_vmax = (uint32_t)(w.rows - 1) * (uint32_t)K * 2u + 112u;   // rows past the bucket re-read the end of its last row
        ld.a_step = (uint32_t)(NL * 8) * (uint32_t)K * 2u;
        ld.b_voff0 = (uint32_t)lane * 16u;
    }
    const bool loader = wave < NL;
    if (loader) {
#pragma unroll
        for (int j = 0; j < N_DMA; ++j) ld.issue(j, w.kt0, w.kt0, 0, 0);
        if (Tile<FM>::NSB == 3) {
#pragma unroll
            for (int j = Loader<FM>::A_PER_L; j < N_DMA; ++j) ld.issue(j, w.kt0, min(w.kt0 + 1, w.kt1 - 1), 0, 1);
        }
    }
#define KLOOP(NFV)                                                              \
    do {                                                                        \
        if (loader) kloop<FM, NFV, true>(acc, smem, ld, w, wave_m, wave_n, lane); \
        else kloop<FM, NFV, false>(acc, smem, ld, w, wave_m, wave_n, lane);       \
    } while (0)
    if (nfrag == FM) KLOOP(FM);
    else if (FM >= 2 && nfrag == FM - 1) KLOOP((FM >= 2 ? FM - 1 : 0));
    else if (FM >= 3 && nfrag == FM - 2) KLOOP((FM >= 3 ? FM - 2 : 0));
    else KLOOP(0);
#undef KLOOP
}

// Tiles of at most kSmallRows rows (the ragged last tile of a bucket, small buckets): there is next to no
// matrix work to hide the loads behind, so with two stages every k tile costs a full memory round trip
// (measured: an 18-row tile takes 93 us where a full one takes 137).  Such a tile needs only a third of the
// activation space, so its stages are 48 KB and three of them fit: two k tiles are in flight while one is
// multiplied.  Row block 0 of every wavefront row covers the tile (rows 32 * wave_m .. +31).  Used by the
// up projection only: in the down projection it gained at some batch sizes and lost at others (the small
// tiles then take bandwidth from the large bucket's tiles, which finish last).
constexpr int kSmallRows = 128, kSmallStages = 3;
constexpr int kSmallAChunks = kSmallRows / 8, kSmallAPerWave = kSmallAChunks / NW;
constexpr int kSmallStage = (kSmallRows + BN) * BK;                     // elements per stage
constexpr int kSmallDma = kSmallAPerWave + B_PER_WAVE;                   // pieces per wavefront and k tile
static_assert(kSmallDma == 6, "the wait below counts six pieces per k tile");

template <int FM>
__device__ __forceinline__ void mainloop_small(f32x4 (&acc)[2 * FM][FN], uint16_t* smem, const uint16_t* __restrict__ A,
                                               const uint16_t* __restrict__ Bbase, int K, const WorkItem& w, int wave, int lane,
                                               bool has_rows) {
    const int wave_m = wave / WN, wave_n = wave % WN;
    uint32_t a_voff[kSmallAPerWave], b_voff[B_PER_WAVE];
#pragma unroll
    for (int j = 0; j < kSmallAPerWave; ++j) {
        const int r = (wave + j * NW) * 8 + (lane >> 3);
        a_voff[j] = (uint32_t)min(r, w.rows - 1) * (uint32_t)K * 2u + (uint32_t)swz(r, lane & 7) * 16u;
    }
#pragma unroll
    for (int j = 0; j < B_PER_WAVE; ++j) b_voff[j] = (uint32_t)(wave + j * NW) * 1024u + (uint32_t)lane * 16u;
    const uint16_t* Abase = A + (size_t)w.row0 * K;
    const uint32_t lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)smem + (uint32_t)wave * 1024u;
    auto issue_tile = [&](int kt, int st) {
        const uint32_t l = lds + (uint32_t)st * (kSmallStage * 2);
#pragma unroll
        for (int j = 0; j < kSmallAPerWave; ++j) dma16(a_voff[j], Abase + (size_t)kt * BK, l + j * NW * 1024);
#pragma unroll
        for (int j = 0; j < B_PER_WAVE; ++j) dma16(b_voff[j], Bbase + (size_t)kt * (BK * BN), l + (kSmallAChunks + j * NW) * 1024);
    };
    const int n = w.kt1 - w.kt0;
    issue_tile(w.kt0, 0);
    if (n > 1) issue_tile(w.kt0 + 1, 1);
    int st = 0;
    for (int i = 0; i < n; ++i) {
        // tile i has landed (the pieces of tile i+1 may still be in flight: six per wavefront, in order)
        if (i + 1 < n) asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();                                     // everyone's pieces have, and tile i-1 has been consumed
        if (i + 2 < n) issue_tile(w.kt0 + i + 2, st == 0 ? 2 : st - 1);      // into the stage of tile i-1
        if (has_rows) {
            const uint16_t* As = smem + st * kSmallStage;
            const uint16_t* Bs = As + kSmallRows * BK;
            // all fragments of the k tile are read before the first matrix instruction (registers are plentiful
            // on this path): one LDS round trip per k tile instead of one per column
            bf16x8 af[KB][2], bq[KB][FN];
#pragma unroll
            for (int ks = 0; ks < KB; ++ks) {
#pragma unroll
                for (int a = 0; a < 2; ++a) {
                    const int r = wave_m * 32 + a * 16 + (lane & 15);
                    af[ks][a] = *reinterpret_cast<const bf16x8*>(As + r * BK + swz(r, ks * 4 + (lane >> 4)) * 8);
                }
#pragma unroll
                for (int b = 0; b < FN; ++b)
                    bq[ks][b] = *reinterpret_cast<const bf16x8*>(Bs + ((wave_n * FN + b) * KB + ks) * 512 + lane * 8);
            }
#pragma unroll
            for (int ks = 0; ks < KB; ++ks)
#pragma unroll
                for (int b = 0; b < FN; ++b) {
                    acc[0][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[ks][0], bq[ks][b], acc[0][b], 0, 0, 0);
                    acc[1][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[ks][1], bq[ks][b], acc[1][b], 0, 0, 0);
                }
        }
        st = st == 2 ? 0 : st + 1;
    }
}

// accumulators -> bf16 -> per-wavefront LDS staging tile (32 rows at a time) -> 16-byte stores of
// whole lines.  accumulator v of a 16x16 fragment: row 4 * (lane / 16) + v, column lane % 16.
// One 32-row block (two fragment rows, blk[0] and blk[1]) whose first tile row is row_base:
template <bool UP>
__device__ __forceinline__ void epilogue_block(const f32x4 (&blk0)[FN], const f32x4 (&blk1)[FN], int row_base, uint16_t* smem,
                                               uint16_t* __restrict__ C, int ldc, const WorkItem& w, int wave, int lane) {
    constexpr int OUTC = UP ? WTN / 2 : WTN;          // output columns of this wavefront
    constexpr int RS = OUTC + 8;                      // staging row stride (elements); the pad staggers the banks
    constexpr int CPR = OUTC / 8;                     // 16-byte chunks per row
    constexpr int RPI = 64 / CPR;                     // rows covered by one wavefront-wide 16-byte access
    const int wave_n = wave % WN;
    uint16_t* stg = smem + wave * (32 * RS);
    const int col = (UP ? w.nt * (BN / 2) : w.nt * BN) + wave_n * OUTC + (lane % CPR) * 8;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const f32x4 (&fr)[FN] = h ? blk1 : blk0;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int r = h * 16 + 4 * (lane >> 4) + v;
            if (UP) {
#pragma unroll
                for (int b = 0; b < FN; b += 2) {
                    const float u = fr[b][v], g = fr[b + 1][v];
                    const float hv = u * __builtin_amdgcn_rcpf(1.0f + __expf(-u)) * g;   // silu(u) * g; rcp is good to 1 ulp, the result is rounded to bf16
                    stg[r * RS + (b >> 1) * 16 + (lane & 15)] = __builtin_bit_cast(uint16_t, (__bf16)hv);
                }
            } else {
#pragma unroll
                for (int b = 0; b < FN; ++b)
                    stg[r * RS + b * 16 + (lane & 15)] = __builtin_bit_cast(uint16_t, (__bf16)fr[b][v]);
            }
        }
    }
#pragma unroll
    for (int it = 0; it < 32 / RPI; ++it) {
        const int r = it * RPI + lane / CPR;
        const int gr = row_base + r;
        if (gr < w.rows && col < ldc)
            *reinterpret_cast<u32x4*>(C + (size_t)(w.row0 + gr) * ldc + col) =
                *reinterpret_cast<const u32x4*>(stg + r * RS + (lane % CPR) * 8);
    }
}

template <bool UP, int FM>
__device__ __forceinline__ void epilogue(const f32x4 (&acc)[2 * FM][FN], uint16_t* smem, uint16_t* __restrict__ C, int ldc,
                                         const WorkItem& w, int wave, int lane, int nfrag) {
#pragma unroll
    for (int j = 0; j < FM; ++j)
        if (j < nfrag) epilogue_block<UP>(acc[2 * j], acc[2 * j + 1], block_row(j, wave / WN), smem, C, ldc, w, wave, lane);
}

template <bool UP>
constexpr int epilogue_bytes() { return NW * 32 * ((UP ? WTN / 2 : WTN) + 8) * 2; }

template <bool UP, int FM>
constexpr int smem_bytes() {
    constexpr int stage_bytes = Tile<FM>::LOOP_ELEMS * 2, small_bytes = kSmallStages * kSmallStage * 2;
    constexpr int loop_bytes = stage_bytes > small_bytes ? stage_bytes : small_bytes;
    return loop_bytes > epilogue_bytes<UP>() ? loop_bytes : epilogue_bytes<UP>();
}

// one workgroup's tile (or k part of a tile) on row tiles of 128 * FM rows
template <bool UP, bool SPLIT, int FM>
__device__ __forceinline__ void ffn_tile(uint16_t* smem, const uint16_t* __restrict__ A, const uint16_t* __restrict__ Wp,
                                         size_t expert_stride, int K, int npad, uint16_t* __restrict__ C, int ldc,
                                         const int32_t* __restrict__ plan, float* __restrict__ partials, int cus_per_xcd,
                                         int row_chunk) {
    constexpr int BM = Tile<FM>::BM;
    const int32_t* prefix = plan + (FM == 3 ? kPlanTiles0 : kPlanTiles1);
    const int NT = npad / BN, KT = K / BK;
    WorkItem w;
    if (!workgroup_item(plan, prefix, NT, KT, BM, blockIdx.x, cus_per_xcd, row_chunk, SPLIT, w)) return;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nfrag = active_blocks(w.rows, wave / WN, FM);   // 32-row blocks of this wavefront that hold rows of the bucket
    const uint16_t* Bbase = Wp + (size_t)w.expert * expert_stride + (size_t)w.nt * ((size_t)K * BN);

    f32x4 acc[2 * FM][FN];
#pragma unroll
    for (int a = 0; a < 2 * FM; ++a)
#pragma unroll
        for (int b = 0; b < FN; ++b)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[a][b][v] = 0.f;

    if (UP && w.rows <= kSmallRows) {
        mainloop_small<FM>(acc, smem, A, Bbase, K, w, wave, lane, nfrag > 0);
    } else if (UP && FM == 3 && w.rows <= Tile<2>::BM) {
        // a ragged tile of at most 256 rows: no wavefront has a third block, so it runs the loop of the
        // 256-row tiles (same row dealing) with its third weight stage and without the clamped loads of
        // the missing rows (up projection only, like the small tiles: the down projection lost 1.5 % with it)
        mainloop<2>(reinterpret_cast<f32x4(&)[4][FN]>(acc), smem, A, Bbase, K, w, wave, lane, nfrag);
    } else {
        mainloop<FM>(acc, smem, A, Bbase, K, w, wave, lane, nfrag);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the pieces fetched during the last k tile land in LDS: nothing may follow them there

    if (SPLIT && w.partial >= 0) {
        if (nfrag > 0) {
            // 16 bytes per lane and store: [fragment][thread]; fragments past the bucket's end hold zeros
            f32x4* dst = reinterpret_cast<f32x4*>(partials + (size_t)w.partial * Tile<FM>::kPartialFloats) + tid;
#pragma unroll
            for (int a = 0; a < 2 * FM; ++a)
#pragma unroll
                for (int b = 0; b < FN; ++b) dst[(size_t)(a * FN + b) * kThreads] = acc[a][b];
        }
        return;
    }
    __syncthreads();                                  // the last tile's fragments have been read by everyone
    epilogue<UP, FM>(acc, smem, C, ldc, w, wave, lane, nfrag);
}

// One launch serves both tile heights: the plan's header says which one this call uses (the host's
// choice, or the plan kernel's own when only the device knows the bucket sizes), and every workgroup
// takes that branch.  Registers and LDS are those of the larger tile either way; one workgroup fits a
// compute unit with both.
template <bool UP, bool SPLIT>
__global__ __launch_bounds__(kThreads) void ffn_bf16_kernel(const uint16_t* __restrict__ A, const uint16_t* __restrict__ Wp,
                                                            size_t expert_stride, int K, int npad, uint16_t* __restrict__ C,
                                                            int ldc, const int32_t* __restrict__ plan, float* __restrict__ partials,
                                                            int cus_per_xcd, int row_chunk) {
    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
    if (plan[3] == 0) ffn_tile<UP, SPLIT, 3>(smem, A, Wp, expert_stride, K, npad, C, ldc, plan, partials, cus_per_xcd, row_chunk);
    else ffn_tile<UP, SPLIT, 2>(smem, A, Wp, expert_stride, K, npad, C, ldc, plan, partials, cus_per_xcd, row_chunk);
}

// adds the k parts of the split tail tiles in part order and writes the tiles; a workgroup handles
// the j-th 32-row block of every wavefront of one tile (fm = 3 or 2 such blocks, by the plan's tile height)
__global__ __launch_bounds__(kThreads) void ffn_bf16_fixup_kernel(int K, int npad, uint16_t* __restrict__ C, int ldc,
                                                                  const int32_t* __restrict__ plan,
                                                                  const float* __restrict__ partials, int cus_per_xcd, int row_chunk) {
    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
    const bool tall = plan[3] == 0;
    const int fm = tall ? 3 : 2, BM = 128 * fm;
    const size_t partial_floats = (size_t)BM * BN;
    const int32_t* prefix = plan + (tall ? kPlanTiles0 : kPlanTiles1);
    const int NT = npad / BN, KT = K / BK;
    const int x = blockIdx.x % kXcds, q = (blockIdx.x / kXcds) / fm, j = (blockIdx.x / kXcds) % fm;
    WorkItem w;
    int first_partial, parts;
    if (!fixup_item(plan, prefix, NT, KT, BM, x, q, cus_per_xcd, row_chunk, w, first_partial, parts)) return;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    if (j >= active_blocks(w.rows, wave / WN, fm)) return;
    f32x4 blk[2][FN];
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int b = 0; b < FN; ++b)
#pragma unroll
            for (int v = 0; v < 4; ++v) blk[h][b][v] = 0.f;
    for (int part = 0; part < parts; ++part) {
        const f32x4* src = reinterpret_cast<const f32x4*>(partials + (size_t)(first_partial + part) * partial_floats) + tid;
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int b = 0; b < FN; ++b) {
                const f32x4 t = src[(size_t)((2 * j + h) * FN + b) * kThreads];
                blk[h][b][0] += t[0]; blk[h][b][1] += t[1]; blk[h][b][2] += t[2]; blk[h][b][3] += t[3];
            }
    }
    epilogue_block<false>(blk[0], blk[1], block_row(j, wave / WN), smem, C, ldc, w, wave, lane);
}

template <typename Kernel>
static int set_smem(Kernel k, int bytes) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    return e == hipSuccess ? MOE_OK : hip_fail(e, "hipFuncSetAttribute");
}

struct FfnCall {
    const void* a; int N, d, f, E; const void* packed; void* out; int32_t* plan; void* H; hipStream_t s;
    int cpx, chunk_up, chunk_down;
    size_t s13, stride;
    float* partials;
    long long grid_for(size_t npad, int bm, bool split) const { return ffn_grid(N, E, (long long)(npad / BN), bm, split, cpx); }
};

template <bool UP>
constexpr int launch_smem() { return smem_bytes<UP, 3>() > smem_bytes<UP, 2>() ? smem_bytes<UP, 3>() : smem_bytes<UP, 2>(); }

// Per-device set-up, done on the first call on each device (not during a stream capture: it calls
// hipFuncSetAttribute): the LDS sizes of the three kernels are raised and the compute units per XCD are read.
// A failure is reported and tried again by the next call rather than remembered.
static int device_setup(int* cus_per_xcd) {
    constexpr int kMaxDevices = 64;
    struct Setup { bool done; int cpx; };
    static std::mutex mutex;
    static Setup setup[kMaxDevices] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return fail(MOE_ERR_UNSUPPORTED, "moe_expert_ffn_grouped: device %d outside [0,%d)", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(mutex);
    Setup& st = setup[dev];
    if (!st.done) {
        int r, cus = 0;
        if ((r = set_smem(&ffn_bf16_kernel<true, false>, launch_smem<true>())) != MOE_OK) return r;
        if ((r = set_smem(&ffn_bf16_kernel<false, true>, launch_smem<false>())) != MOE_OK) return r;
        if ((r = set_smem(&ffn_bf16_fixup_kernel, epilogue_bytes<false>())) != MOE_OK) return r;
        e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess) return hip_fail(e, "hipDeviceGetAttribute");
        st.cpx = cus >= kXcds ? (cus / kXcds < kMaxCusPerXcd ? cus / kXcds : kMaxCusPerXcd) : 32;
        st.done = true;
    }
    *cus_per_xcd = st.cpx;
    return MOE_OK;
}

// the two projections; bm = the smallest tile height the plan may choose (it sizes the grid)
static int run_up(const FfnCall& c, int bm) {
    const long long grid = c.grid_for(npad13(c.f), bm, false);
    if (grid > 0x7FFFFFFFll) return fail(MOE_ERR_UNSUPPORTED, "moe_expert_ffn_grouped: too many tiles for one launch");
    hipLaunchKernelGGL((ffn_bf16_kernel<true, false>), dim3((unsigned)grid), dim3(kThreads), (launch_smem<true>()), c.s,
                       (const uint16_t*)c.a, (const uint16_t*)c.packed, c.stride, c.d, (int)npad13(c.f), (uint16_t*)c.H, c.f, c.plan,
                       c.partials, c.cpx, c.chunk_up);
    return check_launch("moe_expert_ffn_grouped up launch");
}

static int run_down(const FfnCall& c, int bm, int fm_max) {
    const long long grid = c.grid_for(npad2(c.d), bm, true);
    if (grid > 0x7FFFFFFFll) return fail(MOE_ERR_UNSUPPORTED, "moe_expert_ffn_grouped: too many tiles for one launch");
    const uint16_t* W2 = (const uint16_t*)c.packed + c.s13;
    hipLaunchKernelGGL((ffn_bf16_kernel<false, true>), dim3((unsigned)grid), dim3(kThreads), (launch_smem<false>()), c.s,
                       (const uint16_t*)c.H, W2, c.stride, c.f, (int)npad2(c.d), (uint16_t*)c.out, c.d, c.plan, c.partials, c.cpx,
                       c.chunk_down);
    int rc = check_launch("moe_expert_ffn_grouped down launch");
    if (rc != MOE_OK) return rc;
    hipLaunchKernelGGL(ffn_bf16_fixup_kernel, dim3(kXcds * c.cpx * fm_max), dim3(kThreads), (epilogue_bytes<false>()), c.s, c.f,
                       (int)npad2(c.d), (uint16_t*)c.out, c.d, c.plan, c.partials, c.cpx, c.chunk_down);
    return check_launch("moe_expert_ffn_grouped fix-up launch");
}

int launch_ffn_bf16(const void* a, int N, int d, int f, int E, const void* packed, const int32_t* counts,
                    const int32_t* starts, const int32_t* placement, int local_gpu, const int32_t* group_expert,
                    int n_weights, void* out, int32_t* plan, void* H, hipStream_t s) {
    int rc;
    if (N <= kFfnSkinnyMaxRows) {
        // decode-sized batch: every weight is read once and hardly used; stream them without LDS or barriers
        rc = launch_ffn_plan(counts, starts, placement, local_gpu, group_expert, n_weights, E, N, 256, 256, 0, plan, s);
        if (rc != MOE_OK) return rc;
        const size_t s13 = npad13(f) * d, s2 = npad2(d) * f;
        float* partials = (float*)((char*)H + round_up((size_t)N * f * 2, 256));
        return launch_ffn_skinny(a, N, d, f, E, packed, s13, s13 + s2, plan, H, partials, ffn_bf16_scratch_bytes(), out, s);
    }
    // Row tiles of 384 move about a sixth fewer bytes per flop than tiles of 256, but waste more on
    // ragged buckets and leave compute units idle when there are few tiles: 384 when the resident buckets
    // hold kLargeBucketRows rows or more on average.  When every row is in a resident bucket the host
    // knows that average; otherwise only the device does and the plan decides.  Either way the choice
    // reaches the kernels through the plan's header.
    int cpx = 0;
    if ((rc = device_setup(&cpx)) != MOE_OK) return rc;
    const bool every_row_resident = local_gpu < 0 && group_expert == nullptr;
    const int choice = every_row_resident ? ((long long)N >= (long long)kLargeBucketRows * E ? 0 : 1) : -1;
    rc = launch_ffn_plan(counts, starts, placement, local_gpu, group_expert, n_weights, E, N, Tile<3>::BM, Tile<2>::BM, choice, plan, s);
    if (rc != MOE_OK) return rc;
    FfnCall c;
    c.a = a; c.N = N; c.d = d; c.f = f; c.E = E; c.packed = packed; c.out = out; c.plan = plan; c.H = H; c.s = s;
    c.cpx = cpx;
    c.chunk_up = row_chunk_for((size_t)N * d * 2);
    c.chunk_down = row_chunk_for((size_t)N * f * 2);
    c.s13 = npad13(f) * d;
    c.stride = c.s13 + npad2(d) * f;
    c.partials = (float*)((char*)H + round_up((size_t)N * f * 2, 256));     // partial tiles live behind H in the workspace
    const int bm_grid = choice == 0 ? Tile<3>::BM : Tile<2>::BM;     // the grid covers the shorter tiles unless the host chose the tall ones
    const int fm_max = choice == 1 ? 2 : 3;
    {
        LaunchTimer timer(MOE_K_FFN_UP, s);
        if ((rc = run_up(c, bm_grid)) != MOE_OK) return rc;
    }
    {
        LaunchTimer timer(MOE_K_FFN_DOWN, s);
        if ((rc = run_down(c, bm_grid, fm_max)) != MOE_OK) return rc;
    }
    return MOE_OK;
}

}  // namespace moe
