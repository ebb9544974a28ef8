// moe_dispatch: placement-aware token dispatch (paper Section 1, Section 2.2,
// Section 3.1) as a stable counting sort of the N = T*k routes by the key
// (placement[expert], expert), followed by the row copy into the send buffer.
//
//   count : each workgroup histograms its contiguous chunk of routes by expert
//   scan  : one workgroup turns the per-chunk histograms into exclusive
//           per-expert prefixes, sums them to expert_counts (= P_{e,l}), ranks
//           the experts by (gpu, expert) to get expert_start, and derives
//           gpu_counts / gpu_offsets
//   rank  : each workgroup recomputes, wavefront by wavefront, the stable rank
//           of every route among the routes of the same expert (ballot match +
//           popcount of the lower lanes) and writes perm / inv_perm
//   rows  : every 16-byte piece of x[t] is read once and written to the k
//           sorted positions of token t
//
// The result does not depend on how workgroups are scheduled: every position
// is a pure function of the route id.
#include <mutex>
#include "common.h"

namespace moe {

constexpr int kWaves = kDispatchBlock / 64;
constexpr int kMaxChunks = 1024;     // the scan walks this many per-chunk histograms at most

// Routes per thread: 4 for ordinary batches, more for very large ones so that the number of chunks
// (and with it the scan) stays bounded.
void dispatch_geometry(long long N, int* items, int* nblocks) {
    long long it = (N + (long long)kMaxChunks * kDispatchBlock - 1) / ((long long)kMaxChunks * kDispatchBlock);
    if (it < kDispatchItems) it = kDispatchItems;
    it = (it + 3) / 4 * 4;
    *items = (int)it;
    *nblocks = (int)((N + it * kDispatchBlock - 1) / (it * kDispatchBlock));
}

__global__ __launch_bounds__(kDispatchBlock) void dispatch_count_kernel(const int32_t* __restrict__ topk_idx, int N, int E, int items,
                                                                        int32_t* __restrict__ block_counts) {
    __shared__ int hist[MOE_MAX_EXPERTS];
    for (int e = threadIdx.x; e < E; e += kDispatchBlock) hist[e] = 0;
    __syncthreads();
    const long long base = (long long)blockIdx.x * kDispatchBlock * items;
    for (int i = 0; i < items; ++i) {
        const long long r = base + i * kDispatchBlock + threadIdx.x;
        if (r < N) {
            const int e = topk_idx[r];
            if ((unsigned)e < (unsigned)E) atomicAdd(&hist[e], 1);
        }
    }
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += kDispatchBlock) block_counts[(size_t)blockIdx.x * E + e] = hist[e];
}

constexpr int kScanThreads = 1024;

__global__ __launch_bounds__(kScanThreads) void dispatch_scan_kernel(int32_t* __restrict__ block_counts, int nblocks, int E, int EP,
                                                            const int32_t* __restrict__ placement, int G,
                                                            int32_t* __restrict__ expert_counts,
                                                            int32_t* __restrict__ expert_start,
                                                            int32_t* __restrict__ gpu_counts,
                                                            int32_t* __restrict__ gpu_offsets) {
    // EP = E rounded up to a power of two; the threads form kScanThreads/EP slices of the chunk range,
    // each thread owning one expert in one slice
    __shared__ int pl[MOE_MAX_EXPERTS];
    __shared__ int tot[MOE_MAX_EXPERTS];
    __shared__ int slice_tot[kScanThreads];
    const int e = threadIdx.x % EP, sl = threadIdx.x / EP, S = kScanThreads / EP;
    const int per = (nblocks + S - 1) / S;
    const int b0 = sl * per, b1 = min(nblocks, b0 + per);
    int sum = 0;
    if (e < E)
        for (int b = b0; b < b1; ++b) sum += block_counts[(size_t)b * E + e];
    slice_tot[threadIdx.x] = sum;
    if ((int)threadIdx.x < E) pl[threadIdx.x] = placement[threadIdx.x];
    __syncthreads();
    if (e < E) {
        int run = 0;
        for (int s2 = 0; s2 < sl; ++s2) run += slice_tot[s2 * EP + e];
        if (sl == S - 1) {
            tot[e] = run + sum;
            expert_counts[e] = run + sum;
        }
        for (int b = b0; b < b1; ++b) {
            const int c = block_counts[(size_t)b * E + e];
            block_counts[(size_t)b * E + e] = run;      // exclusive prefix over chunks, per expert
            run += c;
        }
    }
    __syncthreads();
    if ((int)threadIdx.x < E) {
        const int me = threadIdx.x;
        int start = 0;
        const int ge = pl[me];
#pragma unroll 8
        for (int o = 0; o < E; ++o) {
            const int go = pl[o];
            start += ((go < ge) | ((go == ge) & (o < me))) ? tot[o] : 0;
        }
        expert_start[me] = start;
    }
    for (int g = threadIdx.x; g < G; g += kScanThreads) {
        int cnt = 0, off = 0;
#pragma unroll 8
        for (int o = 0; o < E; ++o) {
            const int go = pl[o], to = tot[o];
            cnt += (go == g) ? to : 0;
            off += ((go >= 0) & (go < g)) ? to : 0;
        }
        gpu_counts[g] = cnt;
        gpu_offsets[g] = off;
        if (g == G - 1) gpu_offsets[G] = off + cnt;
    }
}

// lanes of this wavefront that hold the same expert as the calling lane
__device__ __forceinline__ unsigned long long match_expert(int e, bool valid, int ebits) {
    unsigned long long m = __ballot(valid);
    for (int b = 0; b < ebits; ++b) {
        const bool bit = (e >> b) & 1;
        const unsigned long long v = __ballot(bit);
        m &= bit ? v : ~v;
    }
    return m;
}

__global__ __launch_bounds__(kDispatchBlock) void dispatch_rank_kernel(const int32_t* __restrict__ topk_idx, int N, int E, int ebits, int items,
                                                                       const int32_t* __restrict__ block_counts,
                                                                       const int32_t* __restrict__ expert_start,
                                                                       int32_t* __restrict__ perm, int32_t* __restrict__ inv_perm) {
    // per wavefront: first the number of routes of each expert in its slice,
    // then (after the prefix over wavefronts) the running write offset
    __shared__ int woff[kWaves][MOE_MAX_EXPERTS];
    const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
    for (int i = threadIdx.x; i < kWaves * MOE_MAX_EXPERTS; i += kDispatchBlock) (&woff[0][0])[i] = 0;
    __syncthreads();

    const long long wbase = ((long long)blockIdx.x * kWaves + wave) * 64 * items;
    const unsigned long long lower = (1ull << lane) - 1ull;
    for (int i = 0; i < items; ++i) {
        const long long r = wbase + i * 64 + lane;
        const int ex = (r < N) ? topk_idx[r] : -1;
        const bool ok = (unsigned)ex < (unsigned)E;
        const unsigned long long m = match_expert(ex, ok, ebits);
        if (ok && (m & lower) == 0ull) atomicAdd(&woff[wave][ex], __popcll(m));   // first lane of the group
    }
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += kDispatchBlock) {
        int run = expert_start[e] + block_counts[(size_t)blockIdx.x * E + e];
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const int c = woff[w][e];
            woff[w][e] = run;
            run += c;
        }
    }
    __syncthreads();
    volatile int* my = woff[wave];
    for (int i = 0; i < items; ++i) {
        const long long r = wbase + i * 64 + lane;
        const int ex = (r < N) ? topk_idx[r] : -1;
        const bool ok = (unsigned)ex < (unsigned)E;
        const unsigned long long m = match_expert(ex, ok, ebits);
        int pos = 0;
        if (ok) pos = my[ex] + __popcll(m & lower);
        __builtin_amdgcn_wave_barrier();
        if (ok && (m & lower) == 0ull) my[ex] += __popcll(m);
        __builtin_amdgcn_wave_barrier();
        if (ok) {
            perm[pos] = (int32_t)r;
            inv_perm[r] = pos;
        }
    }
}

// Batches of up to kFusedMaxRoutes routes: count, scan and rank in ONE workgroup of 16 wavefronts, each
// owning a contiguous slice of the routes.  Three launches become one, which is what matters at these
// sizes (every launch costs more than the work it does).  A thread keeps its ITEMS expert ids in
// registers: they are loaded once, all loads in flight together, and serve both passes.  Same
// results: positions are a pure function of the route id.
constexpr int kFusedThreads = 1024, kFusedWaves = kFusedThreads / 64, kFusedMaxItems = 16;
constexpr int kFusedMaxRoutes = kFusedThreads * kFusedMaxItems;

template <int ITEMS>
__global__ __launch_bounds__(kFusedThreads) void dispatch_index_kernel(const int32_t* __restrict__ topk_idx, int N, int E, int ebits,
                                                                       const int32_t* __restrict__ placement, int G,
                                                                       int32_t* __restrict__ expert_counts,
                                                                       int32_t* __restrict__ expert_start,
                                                                       int32_t* __restrict__ gpu_counts,
                                                                       int32_t* __restrict__ gpu_offsets,
                                                                       int32_t* __restrict__ perm, int32_t* __restrict__ inv_perm) {
    // per wavefront: first the number of routes of each expert in its slice, then its running write offset
    __shared__ int woff[kFusedWaves][MOE_MAX_EXPERTS];
    __shared__ int pl[MOE_MAX_EXPERTS];
    __shared__ int tot[MOE_MAX_EXPERTS];
    const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
    for (int i = threadIdx.x; i < kFusedWaves * MOE_MAX_EXPERTS; i += kFusedThreads) (&woff[0][0])[i] = 0;
    if ((int)threadIdx.x < E) pl[threadIdx.x] = placement[threadIdx.x];
    __syncthreads();

    const int wbase = wave * ITEMS * 64;                                // ITEMS 64-route steps per wavefront
    const unsigned long long lower = (1ull << lane) - 1ull;
    volatile int* my = woff[wave];
    int exs[ITEMS];
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        const int r = wbase + i * 64 + lane;
        exs[i] = (r < N) ? topk_idx[r] : -1;
    }
#pragma unroll
    for (int i = 0; i < ITEMS; ++i)
        if ((unsigned)exs[i] < (unsigned)E) atomicAdd(&woff[wave][exs[i]], 1);   // LDS atomics: counts need no order
    __syncthreads();
    if ((int)threadIdx.x < E) {
        int t = 0;
#pragma unroll
        for (int w = 0; w < kFusedWaves; ++w) t += woff[w][threadIdx.x];
        tot[threadIdx.x] = t;
        expert_counts[threadIdx.x] = t;
    }
    __syncthreads();
    if ((int)threadIdx.x < E) {
        const int me = threadIdx.x, ge = pl[me];
        int start = 0;
#pragma unroll 8
        for (int o = 0; o < E; ++o) {
            const int go = pl[o];
            start += ((go < ge) | ((go == ge) & (o < me))) ? tot[o] : 0;
        }
        expert_start[me] = start;
        int run = start;
#pragma unroll
        for (int w = 0; w < kFusedWaves; ++w) {
            const int c = woff[w][me];
            woff[w][me] = run;
            run += c;
        }
    }
    for (int g = threadIdx.x; g < G; g += kFusedThreads) {
        int cnt = 0, off = 0;
#pragma unroll 8
        for (int o = 0; o < E; ++o) {
            const int go = pl[o], to = tot[o];
            cnt += (go == g) ? to : 0;
            off += ((go >= 0) & (go < g)) ? to : 0;
        }
        gpu_counts[g] = cnt;
        gpu_offsets[g] = off;
        if (g == G - 1) gpu_offsets[G] = off + cnt;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        const int r = wbase + i * 64 + lane;
        const int ex = exs[i];
        const bool ok = (unsigned)ex < (unsigned)E;
        const unsigned long long m = match_expert(ex, ok, ebits);
        int pos = 0;
        if (ok) pos = my[ex] + __popcll(m & lower);
        __builtin_amdgcn_wave_barrier();
        if (ok && (m & lower) == 0ull) my[ex] += __popcll(m);
        __builtin_amdgcn_wave_barrier();
        if (ok) {
            perm[pos] = (int32_t)r;
            inv_perm[r] = pos;
        }
    }
}

// One thread per 16-byte unit of a source row: read once, write k times.
__global__ __launch_bounds__(256) void dispatch_rows_kernel(const uint4* __restrict__ x, long long total_units, int units_per_row,
                                                            int k, int N, const int32_t* __restrict__ inv_perm,
                                                            uint4* __restrict__ send_buf) {
    const long long u = (long long)blockIdx.x * 256 + threadIdx.x;
    if (u >= total_units) return;
    const long long t = u / units_per_row;
    const int c = (int)(u - t * units_per_row);
    const uint4 v = x[u];
    for (int j = 0; j < k; ++j) {
        const int p = inv_perm[t * k + j];
        if ((unsigned)p < (unsigned)N) send_buf[(long long)p * units_per_row + c] = v;
    }
}

// Scratch of moe_dispatch_noalloc: the per-chunk expert histograms (count -> scan -> rank) in device memory
// that exists from the moment the library is loaded, so that the call allocates nothing.  Every GPU the
// library runs on holds its own copy at its own address; in host code the array's name is only a handle
// for hipGetSymbolAddress, never a pointer to pass to a kernel.  The count kernel writes every entry the
// scan and rank kernels read, so nothing has to be cleared between calls; calls that overlap on one GPU
// share the array and race.
static __device__ __align__(256) unsigned char dispatch_scratch[kDispatchStaticScratchBytes];

constexpr int kMaxDevices = 64;

int dispatch_static_scratch(int32_t** scratch) {
    static std::mutex mu;
    static void* addr[kMaxDevices] = {};
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "moe_dispatch_noalloc: hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return fail(MOE_ERR_UNSUPPORTED, "moe_dispatch_noalloc: device %d outside [0,%d)", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(mu);
    if (addr[dev] == nullptr) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(dispatch_scratch));     // this device's copy (dev is current)
        if (e != hipSuccess) return hip_fail(e, "moe_dispatch_noalloc: hipGetSymbolAddress");
        if (p == nullptr) return fail(MOE_ERR_HIP, "moe_dispatch_noalloc: no device address for the scratch array");
        addr[dev] = p;
    }
    *scratch = static_cast<int32_t*>(addr[dev]);
    return MOE_OK;
}

int launch_dispatch(const void* x, int row_bytes, const int32_t* topk_idx, int T, int E, int k,
                    const int32_t* placement, int G, void* send_buf, int32_t* perm, int32_t* inv_perm,
                    int32_t* expert_counts, int32_t* expert_start, int32_t* gpu_counts,
                    int32_t* gpu_offsets, int32_t* block_counts, hipStream_t s) {
    const int N = T * k;
    int items, nblocks;
    dispatch_geometry(N, &items, &nblocks);
    int ebits = 0;
    while ((1 << ebits) < E) ++ebits;
    const int EP = 1 << ebits;
    int rc;
    if (N <= kFusedMaxRoutes) {
        LaunchTimer timer(MOE_K_DISPATCH_RANK, s);
#define MOE_LAUNCH_INDEX(ITEMS)                                                                                          \
    hipLaunchKernelGGL(dispatch_index_kernel<ITEMS>, dim3(1), dim3(kFusedThreads), 0, s, topk_idx, N, E, ebits, placement, G, \
                       expert_counts, expert_start, gpu_counts, gpu_offsets, perm, inv_perm)
        if (N <= kFusedThreads) MOE_LAUNCH_INDEX(1);
        else if (N <= 2 * kFusedThreads) MOE_LAUNCH_INDEX(2);
        else if (N <= 4 * kFusedThreads) MOE_LAUNCH_INDEX(4);
        else if (N <= 8 * kFusedThreads) MOE_LAUNCH_INDEX(8);
        else MOE_LAUNCH_INDEX(kFusedMaxItems);
#undef MOE_LAUNCH_INDEX
        if ((rc = check_launch("moe_dispatch index launch")) != MOE_OK) return rc;
    } else {
        if (nblocks > 0) {
            LaunchTimer timer(MOE_K_DISPATCH_COUNT, s);
            hipLaunchKernelGGL(dispatch_count_kernel, dim3(nblocks), dim3(kDispatchBlock), 0, s, topk_idx, N, E, items, block_counts);
            if ((rc = check_launch("moe_dispatch count launch")) != MOE_OK) return rc;
        }
        {
            LaunchTimer timer(MOE_K_DISPATCH_SCAN, s);
            hipLaunchKernelGGL(dispatch_scan_kernel, dim3(1), dim3(kScanThreads), 0, s, block_counts, nblocks, E, EP, placement, G,
                               expert_counts, expert_start, gpu_counts, gpu_offsets);
            if ((rc = check_launch("moe_dispatch scan launch")) != MOE_OK) return rc;
        }
        if (nblocks > 0) {
            LaunchTimer timer(MOE_K_DISPATCH_RANK, s);
            hipLaunchKernelGGL(dispatch_rank_kernel, dim3(nblocks), dim3(kDispatchBlock), 0, s, topk_idx, N, E, ebits, items,
                               block_counts, expert_start, perm, inv_perm);
            if ((rc = check_launch("moe_dispatch rank launch")) != MOE_OK) return rc;
        }
    }
    if (x != nullptr && N > 0) {
        const int units_per_row = row_bytes / 16;
        const long long total_units = (long long)T * units_per_row;
        const long long grid = (total_units + 255) / 256;
        if (grid > 0x7FFFFFFFll) return fail(MOE_ERR_UNSUPPORTED, "moe_dispatch: T*d too large for one launch");
        LaunchTimer timer(MOE_K_DISPATCH_ROWS, s);
        hipLaunchKernelGGL(dispatch_rows_kernel, dim3((unsigned)grid), dim3(256), 0, s, (const uint4*)x, total_units,
                           units_per_row, k, N, inv_perm, (uint4*)send_buf);
        if ((rc = check_launch("moe_dispatch rows launch")) != MOE_OK) return rc;
    }
    return MOE_OK;
}

}  // namespace moe
