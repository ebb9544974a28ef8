// moe_receive_segments: the segment table of the buffer a GPU receives from the first all-to-all of an
// expert-parallel layer (paper Section 2.2 / Fig. 2b), built on the device from the ranks' gathered
// expert_counts so that no bucket size has to visit the host between dispatch and the expert FFN.
//
// Source rank s sends GPU `dest` its bucket for dest, already sorted by expert; the receive buffer is the
// concatenation of those buckets in source order.  Its segments are therefore, source after source, one run
// of rows per expert that lives on dest, experts ascending: segment (s, i-th expert of dest) holds
// expert_counts[s][e] rows.  The table feeds moe_expert_ffn_segments directly.
// The tables are tiny (at most 256 segments), so the call is one workgroup.
#include "common.h"

namespace moe {

__global__ __launch_bounds__(MOE_MAX_EXPERTS) void receive_segments_kernel(const int32_t* __restrict__ counts_all,
                                                                          const int32_t* __restrict__ placement, int E, int G, int dest,
                                                                          int max_seg, int32_t* __restrict__ seg_expert,
                                                                          int32_t* __restrict__ seg_counts, int32_t* __restrict__ seg_start,
                                                                          int32_t* __restrict__ src_offset, int32_t* __restrict__ n_seg_out) {
    __shared__ int is_local[MOE_MAX_EXPERTS];
    __shared__ int local_expert[MOE_MAX_EXPERTS];        // the experts of dest, ascending
    __shared__ int cnt[MOE_MAX_EXPERTS];                 // rows of segment i
    const int i = threadIdx.x;
    is_local[i] = (i < E && placement[i] == dest) ? 1 : 0;
    __syncthreads();
    int rank = 0, n_local = 0;
    for (int e = 0; e < E; ++e) {
        rank += (e < i) ? is_local[e] : 0;
        n_local += is_local[e];
    }
    if (is_local[i]) local_expert[rank] = i;
    __syncthreads();
    const long long wanted = (long long)G * n_local;
    const int n_seg = (int)(wanted < max_seg ? wanted : max_seg);
    int e = 0, c = 0;
    if (i < n_seg) {
        const int s = i / n_local;
        e = local_expert[i - s * n_local];
        c = counts_all[(size_t)s * E + e];
        if (c < 0) c = 0;
    }
    cnt[i] = c;
    __syncthreads();
    int start = 0, total = 0;
    for (int j = 0; j < n_seg; ++j) {
        start += (j < i) ? cnt[j] : 0;
        total += cnt[j];
    }
    if (i < max_seg) {                                   // entries past the last segment are empty segments at the end of the buffer
        seg_expert[i] = e;
        seg_counts[i] = c;
        seg_start[i] = i < n_seg ? start : total;
    }
    if (src_offset != nullptr) {
        // source s begins at its first segment (s * n_local); sources whose segments did not fit, and the end, at the total
        if (i < G) {
            int off = 0;
            const int first = i * n_local;
            for (int j = 0; j < n_seg && j < first; ++j) off += cnt[j];
            src_offset[i] = off;
        }
        if (i == 0) src_offset[G] = total;
    }
    if (i == 0 && n_seg_out != nullptr) *n_seg_out = (int)(wanted < 0x7FFFFFFF ? wanted : 0x7FFFFFFF);
}

int launch_receive_segments(const int32_t* counts_all, const int32_t* placement, int E, int G, int dest, int max_seg,
                            int32_t* seg_expert, int32_t* seg_counts, int32_t* seg_start, int32_t* src_offset, int32_t* n_seg_out,
                            hipStream_t s) {
    hipLaunchKernelGGL(receive_segments_kernel, dim3(1), dim3(MOE_MAX_EXPERTS), 0, s, counts_all, placement, E, G, dest, max_seg,
                       seg_expert, seg_counts, seg_start, src_offset, n_seg_out);
    return check_launch("moe_receive_segments launch");
}

}  // namespace moe
