// Internal helpers shared by the HIP sources of libmoetuner_hip (not part of
// the public interface, which is include/moetuner.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "moetuner.h"

namespace moe {

// printf-style message for moe_last_error(); returns `code` for tail calls.
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
int hip_fail(hipError_t e, const char* what);

// Brackets one kernel launch with a pair of events when a timing session has
// selected this kernel id; otherwise does nothing.
class LaunchTimer {
public:
    LaunchTimer(int kernel_id, hipStream_t stream);
    ~LaunchTimer();
    LaunchTimer(const LaunchTimer&) = delete;
    LaunchTimer& operator=(const LaunchTimer&) = delete;
private:
    int slot_;
    hipStream_t stream_;
    hipEvent_t start_ = nullptr, stop_ = nullptr;
};

inline int check_launch(const char* what) {
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? MOE_OK : hip_fail(e, what);
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline int elt_bytes(moe_dtype_t dt) { return dt == MOE_BF16 ? 2 : 4; }

// ---- launchers implemented in the .hip files --------------------------------
int launch_gate(const float* logits, int T, int E, int k, bool all_norm, int32_t* idx, float* w, hipStream_t s);

constexpr int kDispatchBlock = 256;
constexpr int kDispatchItems = 4;
void dispatch_geometry(long long N, int* items, int* nblocks);      // routes per thread and number of chunks
int launch_dispatch(const void* x, int row_bytes, const int32_t* topk_idx, int T, int E, int k,
                    const int32_t* placement, int G, void* send_buf, int32_t* perm, int32_t* inv_perm,
                    int32_t* expert_counts, int32_t* expert_start, int32_t* gpu_counts,
                    int32_t* gpu_offsets, int32_t* block_counts, hipStream_t s);

// moe_dispatch_noalloc: the per-chunk histograms live in a file-scope device array of this many bytes;
// dispatch_static_scratch returns the current device's copy of it (looked up once per device)
constexpr size_t kDispatchStaticScratchBytes = (size_t)256 << 10;
int dispatch_static_scratch(int32_t** scratch);

int launch_combine(const void* ffn_out, moe_dtype_t dt, const int32_t* inv_perm, const int32_t* topk_idx,
                   const float* topk_w, const int32_t* placement, int local_gpu, int T, int d, int E, int k,
                   void* y, hipStream_t s);

int launch_transition(const int32_t* idx_l, const int32_t* idx_l1, int T, int k_l, int k_l1, int E_l,
                      int E_l1, bool top1_only, int64_t* R, hipStream_t s);

size_t router_packed_bytes(int d, int E, moe_dtype_t dt);
int launch_pack_router(const void* w_g, int d, int E, moe_dtype_t dt, void* packed, hipStream_t s);
int launch_router_gate(const void* x, moe_dtype_t dt, const void* packed, const float* bias, int T, int d, int E, int k,
                       float* logits, int32_t* idx, float* w, hipStream_t s);
int launch_accumulate_counts(const int32_t* counts, int E, int64_t* P, hipStream_t s);
int launch_placement_loads(const int64_t* P, const int32_t* placement, int E, int G, int64_t* T_c, double* imbalance, hipStream_t s);
int launch_placement_traffic(const int64_t* R, const int32_t* pl_l, const int32_t* pl_l1, int E_l, int E_l1, int G, int64_t* C,
                             const double* B, double* max_cost, hipStream_t s);

int launch_receive_segments(const int32_t* counts_all, const int32_t* placement, int E, int G, int dest, int max_seg,
                            int32_t* seg_expert, int32_t* seg_counts, int32_t* seg_start, int32_t* src_offset, int32_t* n_seg_out,
                            hipStream_t s);

// FFN: the workspace starts with a small plan area, followed by H [N,f].
constexpr size_t kPlanBytes = 8192;
size_t packed_bytes_f32(int E, int d, int f);
size_t packed_bytes_bf16(int E, int d, int f);
size_t ffn_bf16_scratch_bytes();      // fp32 partial tiles of the split tail, sized for the largest supported XCD
int launch_pack_f32(const float* w1, const float* w3, const float* w2, int E, int d, int f, float* packed, hipStream_t s);
int launch_pack_bf16(const void* w1, const void* w3, const void* w2, int E, int d, int f, void* packed, hipStream_t s);
// E row groups (counts/starts); group g uses the weights of expert group_expert[g] of n_weights
// (g itself when group_expert is NULL)
int launch_ffn_f32(const float* a, int N, int d, int f, int E, const float* packed, const int32_t* counts,
                   const int32_t* starts, const int32_t* placement, int local_gpu, const int32_t* group_expert,
                   int n_weights, float* out, int32_t* plan, float* H, hipStream_t s);
// bf16, N <= kFfnSkinnyMaxRows: weight-streaming kernels for decode-sized batches (plan already built).
// Measured at the Mixtral shape with skewed top-2 routing: they win up to N = 128 rows (+13 to +18 %) and lose from
// N = 256 on (-7 %), where the largest bucket needs several passes of 64 rows over its weights.
#ifndef MOE_SKINNY_MAX_ROWS
#define MOE_SKINNY_MAX_ROWS 160
#endif
constexpr int kFfnSkinnyMaxRows = MOE_SKINNY_MAX_ROWS;
int launch_ffn_skinny(const void* a, int N, int d, int f, int E, const void* packed, size_t s13, size_t expert_stride,
                      const int32_t* plan, void* H, float* partial, size_t scratch_bytes, void* out, hipStream_t s);
int launch_ffn_bf16(const void* a, int N, int d, int f, int E, const void* packed, const int32_t* counts,
                    const int32_t* starts, const int32_t* placement, int local_gpu, const int32_t* group_expert,
                    int n_weights, void* out, int32_t* plan, void* H, hipStream_t s);

}  // namespace moe
