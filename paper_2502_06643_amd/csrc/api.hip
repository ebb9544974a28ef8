// C ABI of libmoetuner_hip: argument validation, error text, kernel timing.
// The numerical work is in the launchers (gate.hip, dispatch.hip, ffn_*.hip,
// combine.hip, transition.hip).
#include "common.h"
#include <cstdarg>
#include <atomic>
#include <cstdio>
#include <mutex>
#include <vector>

namespace moe {

static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

int hip_fail(hipError_t e, const char* what) {
    return fail(MOE_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

// ---- timing session -----------------------------------------------------------
// One session per process.  The mask is atomic and the record table is guarded, so launches from several
// host threads may run while a session is open; begin and end themselves are for one controlling thread.
struct TimingRecord { int kid; hipEvent_t start, stop; };
static std::atomic<unsigned> g_mask{0};
static std::mutex g_timing_mutex;
static int g_used = 0;
static std::vector<TimingRecord> g_records;

LaunchTimer::LaunchTimer(int kernel_id, hipStream_t stream) : slot_(-1), stream_(stream) {
    if (!(g_mask.load(std::memory_order_acquire) & (1u << kernel_id))) return;
    std::lock_guard<std::mutex> lock(g_timing_mutex);
    if (!(g_mask.load(std::memory_order_relaxed) & (1u << kernel_id)) || g_used >= (int)g_records.size()) return;
    slot_ = g_used++;
    g_records[slot_].kid = kernel_id;
    start_ = g_records[slot_].start;
    stop_ = g_records[slot_].stop;
    (void)hipEventRecord(start_, stream_);
}

LaunchTimer::~LaunchTimer() {
    if (slot_ >= 0) (void)hipEventRecord(stop_, stream_);
}

// caller holds g_timing_mutex
static void destroy_records() {
    g_mask.store(0, std::memory_order_release);
    for (auto& r : g_records) {
        (void)hipEventDestroy(r.start);
        (void)hipEventDestroy(r.stop);
    }
    g_records.clear();
    g_used = 0;
}

}  // namespace moe

using namespace moe;

#define REQUIRE(cond, ...) do { if (!(cond)) return fail(MOE_ERR_INVALID_ARG, __VA_ARGS__); } while (0)

extern "C" {

const char* moe_last_error(void) { return g_err; }

const char* moe_version(void) { return "moetuner-hip 0.1 (gfx950)"; }

int moe_timing_begin(unsigned mask, int max_records) {
    REQUIRE(max_records > 0 && max_records <= (1 << 20), "moe_timing_begin: max_records=%d out of range", max_records);
    std::lock_guard<std::mutex> lock(g_timing_mutex);
    destroy_records();
    g_records.resize(max_records);
    for (int i = 0; i < max_records; ++i) {
        hipError_t e = hipEventCreate(&g_records[i].start);
        if (e == hipSuccess) e = hipEventCreate(&g_records[i].stop);
        if (e != hipSuccess) {
            g_records.resize(i);
            destroy_records();
            return hip_fail(e, "hipEventCreate");
        }
    }
    g_mask.store(mask, std::memory_order_release);
    return MOE_OK;
}

int moe_timing_end(double* sum_ms, int* launches) {
    REQUIRE(sum_ms && launches, "moe_timing_end: NULL output");
    for (int i = 0; i < MOE_K_COUNT; ++i) { sum_ms[i] = 0.0; launches[i] = 0; }
    std::lock_guard<std::mutex> lock(g_timing_mutex);
    g_mask.store(0, std::memory_order_release);          // launches from here on are not timed
    int rc = MOE_OK;
    for (int i = 0; i < g_used; ++i) {
        hipError_t e = hipEventSynchronize(g_records[i].stop);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, g_records[i].start, g_records[i].stop);
        if (e != hipSuccess) { rc = hip_fail(e, "moe_timing_end"); break; }
        sum_ms[g_records[i].kid] += ms;
        launches[g_records[i].kid] += 1;
    }
    destroy_records();
    return rc;
}

int moe_topk_gate_norm(const float* logits, int T, int E, int k, moe_norm_t norm, int32_t* topk_idx, float* topk_w, void* stream) {
    REQUIRE(norm == MOE_NORM_SOFTMAX_SELECTED || norm == MOE_NORM_SOFTMAX_ALL, "moe_topk_gate: unknown norm %d", (int)norm);
    REQUIRE(T >= 0, "moe_topk_gate: T=%d < 0", T);
    REQUIRE(E >= 1 && E <= MOE_MAX_EXPERTS, "moe_topk_gate: E=%d outside [1,%d]", E, MOE_MAX_EXPERTS);
    REQUIRE(k >= 1 && k <= E && k <= MOE_MAX_TOPK, "moe_topk_gate: k=%d outside [1,min(E=%d,%d)]", k, E, MOE_MAX_TOPK);
    REQUIRE((long long)T * E < (1ll << 31) , "moe_topk_gate: T*E too large");
    if (T == 0) return MOE_OK;
    REQUIRE(logits && topk_idx && topk_w, "moe_topk_gate: NULL pointer");
    REQUIRE(aligned16(logits) && aligned16(topk_idx) && aligned16(topk_w), "moe_topk_gate: pointers must be 16-byte aligned");
    return launch_gate(logits, T, E, k, norm == MOE_NORM_SOFTMAX_ALL, topk_idx, topk_w, (hipStream_t)stream);
}

int moe_topk_gate(const float* logits, int T, int E, int k, int32_t* topk_idx, float* topk_w, void* stream) {
    return moe_topk_gate_norm(logits, T, E, k, MOE_NORM_SOFTMAX_SELECTED, topk_idx, topk_w, stream);
}

static int check_router_shape(const char* who, int d, int E, moe_dtype_t dt) {
    REQUIRE(dt == MOE_F32 || dt == MOE_BF16, "%s: unknown dtype %d", who, (int)dt);
    REQUIRE(E >= 1 && E <= MOE_MAX_EXPERTS, "%s: E=%d outside [1,%d]", who, E, MOE_MAX_EXPERTS);
    REQUIRE(d >= 1, "%s: d=%d < 1", who, d);
    if (dt == MOE_BF16 && d % 64) return fail(MOE_ERR_UNSUPPORTED, "%s: bf16 needs d %% 64 == 0 (d=%d)", who, d);
    return MOE_OK;
}

size_t moe_router_packed_bytes(int d, int E, moe_dtype_t dt) {
    if (check_router_shape("moe_router_packed_bytes", d, E, dt) != MOE_OK) return 0;
    return router_packed_bytes(d, E, dt);
}

int moe_pack_router(const void* w_g, int d, int E, moe_dtype_t dt, void* packed, size_t packed_bytes, void* stream) {
    int rc = check_router_shape("moe_pack_router", d, E, dt);
    if (rc != MOE_OK) return rc;
    REQUIRE(w_g && packed, "moe_pack_router: NULL pointer");
    REQUIRE(aligned16(w_g) && aligned16(packed), "moe_pack_router: pointers must be 16-byte aligned");
    if (packed_bytes < router_packed_bytes(d, E, dt))
        return fail(MOE_ERR_WORKSPACE, "moe_pack_router: packed buffer %zu < %zu bytes", packed_bytes, router_packed_bytes(d, E, dt));
    return launch_pack_router(w_g, d, E, dt, packed, (hipStream_t)stream);
}

int moe_router_gate(const void* x, moe_dtype_t dt, const void* packed_router, const float* bias, int T, int d, int E, int k,
                    float* logits, int32_t* topk_idx, float* topk_w, void* stream) {
    int rc = check_router_shape("moe_router_gate", d, E, dt);
    if (rc != MOE_OK) return rc;
    REQUIRE(T >= 0, "moe_router_gate: T=%d < 0", T);
    REQUIRE(k >= 1 && k <= E && k <= MOE_MAX_TOPK, "moe_router_gate: k=%d outside [1,min(E=%d,%d)]", k, E, MOE_MAX_TOPK);
    REQUIRE((long long)T * E < (1ll << 31), "moe_router_gate: T*E too large");
    if (T == 0) return MOE_OK;
    REQUIRE(x && packed_router && topk_idx && topk_w, "moe_router_gate: NULL pointer");
    REQUIRE(aligned16(x) && aligned16(packed_router) && aligned16(logits) && aligned16(topk_idx) && aligned16(topk_w),
            "moe_router_gate: pointers must be 16-byte aligned");
    return launch_router_gate(x, dt, packed_router, bias, T, d, E, k, logits, topk_idx, topk_w, (hipStream_t)stream);
}

size_t moe_dispatch_workspace_bytes(int T, int E, int k) {
    if (T < 0 || E < 1 || k < 1) return 0;
    int items = 0, nb = 0;
    dispatch_geometry((long long)T * k, &items, &nb);
    if (nb == 0) nb = 1;
    return round_up((size_t)nb * (size_t)E * sizeof(int32_t), 256);
}

// scalar and pointer checks shared by the two dispatch entry points; sets row_bytes
static int check_dispatch_args(const char* who, const void* x, moe_dtype_t dt, const int32_t* topk_idx, int T, int d, int E, int k,
                               const int32_t* placement, int G, const void* send_buf, const int32_t* perm, const int32_t* inv_perm,
                               const int32_t* expert_counts, const int32_t* expert_start, const int32_t* gpu_counts,
                               const int32_t* gpu_offsets, int* row_bytes) {
    REQUIRE(dt == MOE_F32 || dt == MOE_BF16, "%s: unknown dtype %d", who, (int)dt);
    REQUIRE(T >= 0, "%s: T=%d < 0", who, T);
    REQUIRE(E >= 1 && E <= MOE_MAX_EXPERTS, "%s: E=%d outside [1,%d]", who, E, MOE_MAX_EXPERTS);
    REQUIRE(k >= 1 && k <= E && k <= MOE_MAX_TOPK, "%s: k=%d outside [1,min(E=%d,%d)]", who, k, E, MOE_MAX_TOPK);
    REQUIRE(G >= 1 && G <= MOE_MAX_GPUS, "%s: G=%d outside [1,%d]", who, G, MOE_MAX_GPUS);
    REQUIRE((long long)T * k < (1ll << 31), "%s: T*k does not fit int32", who);
    REQUIRE(placement && expert_counts && expert_start && gpu_counts && gpu_offsets, "%s: NULL output or placement", who);
    REQUIRE(T == 0 || (topk_idx && perm && inv_perm), "%s: NULL index pointer", who);
    REQUIRE((x == nullptr) == (send_buf == nullptr), "%s: x and send_buf must both be given or both be NULL", who);
    *row_bytes = 0;
    if (x) {
        REQUIRE(d >= 1, "%s: d=%d < 1", who, d);
        REQUIRE(((long long)d * elt_bytes(dt)) % 16 == 0, "%s: a row (d=%d) must be a multiple of 16 bytes", who, d);
        REQUIRE(aligned16(x) && aligned16(send_buf), "%s: x/send_buf must be 16-byte aligned", who);
        *row_bytes = d * elt_bytes(dt);
    }
    return MOE_OK;
}

int moe_dispatch(const void* x, moe_dtype_t dt, const int32_t* topk_idx, int T, int d, int E, int k,
                 const int32_t* placement, int G, void* send_buf, int32_t* perm, int32_t* inv_perm,
                 int32_t* expert_counts, int32_t* expert_start, int32_t* gpu_counts, int32_t* gpu_offsets,
                 void* workspace, size_t workspace_bytes, void* stream) {
    int row_bytes = 0;
    int rc = check_dispatch_args("moe_dispatch", x, dt, topk_idx, T, d, E, k, placement, G, send_buf, perm, inv_perm, expert_counts,
                                 expert_start, gpu_counts, gpu_offsets, &row_bytes);
    if (rc != MOE_OK) return rc;
    REQUIRE(workspace != nullptr, "moe_dispatch: NULL workspace");
    if (workspace_bytes < moe_dispatch_workspace_bytes(T, E, k))
        return fail(MOE_ERR_WORKSPACE, "moe_dispatch: workspace %zu < %zu bytes", workspace_bytes,
                    moe_dispatch_workspace_bytes(T, E, k));
    return launch_dispatch(x, row_bytes, topk_idx, T, E, k, placement, G, send_buf, perm, inv_perm, expert_counts,
                           expert_start, gpu_counts, gpu_offsets, (int32_t*)workspace, (hipStream_t)stream);
}

size_t moe_dispatch_static_scratch_bytes(void) { return kDispatchStaticScratchBytes; }

int moe_dispatch_noalloc(const void* x, moe_dtype_t dt, const int32_t* topk_idx, int T, int d, int E, int k,
                         const int32_t* placement, int G, void* send_buf, int32_t* perm, int32_t* inv_perm,
                         int32_t* expert_counts, int32_t* expert_start, int32_t* gpu_counts, int32_t* gpu_offsets,
                         void* stream) {
    int row_bytes = 0;
    int rc = check_dispatch_args("moe_dispatch_noalloc", x, dt, topk_idx, T, d, E, k, placement, G, send_buf, perm, inv_perm,
                                 expert_counts, expert_start, gpu_counts, gpu_offsets, &row_bytes);
    if (rc != MOE_OK) return rc;
    const size_t need = moe_dispatch_workspace_bytes(T, E, k);
    if (need > kDispatchStaticScratchBytes)
        return fail(MOE_ERR_WORKSPACE, "moe_dispatch_noalloc: T=%d, k=%d, E=%d need %zu bytes of scratch, the built-in buffer holds %zu; "
                    "use moe_dispatch with a caller workspace", T, k, E, need, kDispatchStaticScratchBytes);
    int32_t* scratch = nullptr;
    if ((rc = dispatch_static_scratch(&scratch)) != MOE_OK) return rc;
    return launch_dispatch(x, row_bytes, topk_idx, T, E, k, placement, G, send_buf, perm, inv_perm, expert_counts,
                           expert_start, gpu_counts, gpu_offsets, scratch, (hipStream_t)stream);
}

static int check_ffn_shape(const char* who, int E, int d, int f, moe_dtype_t dt) {
    REQUIRE(dt == MOE_F32 || dt == MOE_BF16, "%s: unknown dtype %d", who, (int)dt);
    REQUIRE(E >= 1 && E <= MOE_MAX_EXPERTS, "%s: E=%d outside [1,%d]", who, E, MOE_MAX_EXPERTS);
    REQUIRE(d >= 1 && f >= 1, "%s: d=%d, f=%d must be positive", who, d, f);
    if (dt == MOE_BF16) {
        if (d % 64 || f % 64) return fail(MOE_ERR_UNSUPPORTED, "%s: bf16 needs d %% 64 == 0 and f %% 64 == 0 (d=%d, f=%d)", who, d, f);
    } else {
        if (d % 4 || f % 4) return fail(MOE_ERR_UNSUPPORTED, "%s: fp32 needs d %% 4 == 0 and f %% 4 == 0 (d=%d, f=%d)", who, d, f);
    }
    return MOE_OK;
}

size_t moe_packed_weights_bytes(int E, int d, int f, moe_dtype_t dt) {
    if (check_ffn_shape("moe_packed_weights_bytes", E, d, f, dt) != MOE_OK) return 0;
    return dt == MOE_BF16 ? packed_bytes_bf16(E, d, f) : packed_bytes_f32(E, d, f);
}

int moe_pack_weights(const void* w1, const void* w3, const void* w2, int E, int d, int f, moe_dtype_t dt,
                     void* packed, size_t packed_bytes, void* stream) {
    int rc = check_ffn_shape("moe_pack_weights", E, d, f, dt);
    if (rc != MOE_OK) return rc;
    REQUIRE(w1 && w3 && w2 && packed, "moe_pack_weights: NULL pointer");
    REQUIRE(aligned16(w1) && aligned16(w3) && aligned16(w2) && aligned16(packed), "moe_pack_weights: pointers must be 16-byte aligned");
    size_t need = moe_packed_weights_bytes(E, d, f, dt);
    if (packed_bytes < need) return fail(MOE_ERR_WORKSPACE, "moe_pack_weights: packed buffer %zu < %zu bytes", packed_bytes, need);
    if (dt == MOE_BF16) return launch_pack_bf16(w1, w3, w2, E, d, f, packed, (hipStream_t)stream);
    return launch_pack_f32((const float*)w1, (const float*)w3, (const float*)w2, E, d, f, (float*)packed, (hipStream_t)stream);
}

size_t moe_ffn_workspace_bytes(int N, int d, int f, int E, moe_dtype_t dt) {
    if (N < 0 || check_ffn_shape("moe_ffn_workspace_bytes", E, d, f, dt) != MOE_OK) return 0;
    return kPlanBytes + round_up((size_t)N * f * elt_bytes(dt), 256) + 256 + (dt == MOE_BF16 ? ffn_bf16_scratch_bytes() : 0);
}

int moe_expert_ffn_grouped(const void* send_buf, moe_dtype_t dt, int N, int d, int f, int E,
                           const void* packed_weights, const int32_t* expert_counts, const int32_t* expert_start,
                           const int32_t* placement, int local_gpu, void* ffn_out,
                           void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_ffn_shape("moe_expert_ffn_grouped", E, d, f, dt);
    if (rc != MOE_OK) return rc;
    REQUIRE(N >= 0, "moe_expert_ffn_grouped: N=%d < 0", N);
    REQUIRE(local_gpu >= -1 && local_gpu < MOE_MAX_GPUS, "moe_expert_ffn_grouped: local_gpu=%d outside [-1,%d)", local_gpu, MOE_MAX_GPUS);
    if (N == 0) return MOE_OK;
    REQUIRE(send_buf && packed_weights && expert_counts && expert_start && placement && ffn_out && workspace,
            "moe_expert_ffn_grouped: NULL pointer");
    REQUIRE(aligned16(send_buf) && aligned16(packed_weights) && aligned16(ffn_out) && aligned16(workspace),
            "moe_expert_ffn_grouped: pointers must be 16-byte aligned");
    size_t need = moe_ffn_workspace_bytes(N, d, f, E, dt);
    if (workspace_bytes < need) return fail(MOE_ERR_WORKSPACE, "moe_expert_ffn_grouped: workspace %zu < %zu bytes", workspace_bytes, need);
    int32_t* plan = (int32_t*)workspace;
    void* H = (char*)workspace + kPlanBytes;
    hipStream_t s = (hipStream_t)stream;
    if (dt == MOE_BF16)
        return launch_ffn_bf16(send_buf, N, d, f, E, packed_weights, expert_counts, expert_start, placement, local_gpu, nullptr, E,
                               ffn_out, plan, H, s);
    return launch_ffn_f32((const float*)send_buf, N, d, f, E, (const float*)packed_weights, expert_counts, expert_start,
                          placement, local_gpu, nullptr, E, (float*)ffn_out, plan, (float*)H, s);
}

int moe_expert_ffn_segments(const void* recv_buf, moe_dtype_t dt, int N, int d, int f, int E,
                            const void* packed_weights, int n_seg, const int32_t* seg_expert, const int32_t* seg_counts,
                            const int32_t* seg_start, void* ffn_out, void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_ffn_shape("moe_expert_ffn_segments", E, d, f, dt);
    if (rc != MOE_OK) return rc;
    REQUIRE(N >= 0, "moe_expert_ffn_segments: N=%d < 0", N);
    REQUIRE(n_seg >= 0 && n_seg <= MOE_MAX_EXPERTS, "moe_expert_ffn_segments: n_seg=%d outside [0,%d]", n_seg, MOE_MAX_EXPERTS);
    if (N == 0 || n_seg == 0) return MOE_OK;
    REQUIRE(recv_buf && packed_weights && seg_expert && seg_counts && seg_start && ffn_out && workspace,
            "moe_expert_ffn_segments: NULL pointer");
    REQUIRE(aligned16(recv_buf) && aligned16(packed_weights) && aligned16(ffn_out) && aligned16(workspace),
            "moe_expert_ffn_segments: pointers must be 16-byte aligned");
    size_t need = moe_ffn_workspace_bytes(N, d, f, E, dt);
    if (workspace_bytes < need) return fail(MOE_ERR_WORKSPACE, "moe_expert_ffn_segments: workspace %zu < %zu bytes", workspace_bytes, need);
    int32_t* plan = (int32_t*)workspace;
    void* H = (char*)workspace + kPlanBytes;
    hipStream_t s = (hipStream_t)stream;
    if (dt == MOE_BF16)
        return launch_ffn_bf16(recv_buf, N, d, f, n_seg, packed_weights, seg_counts, seg_start, nullptr, -1, seg_expert, E, ffn_out, plan, H, s);
    return launch_ffn_f32((const float*)recv_buf, N, d, f, n_seg, (const float*)packed_weights, seg_counts, seg_start, nullptr, -1,
                          seg_expert, E, (float*)ffn_out, plan, (float*)H, s);
}

int moe_receive_segments(const int32_t* expert_counts_all, const int32_t* placement, int E, int G, int dest, int max_seg,
                         int32_t* seg_expert, int32_t* seg_counts, int32_t* seg_start, int32_t* src_offset, int32_t* n_seg,
                         void* stream) {
    REQUIRE(E >= 1 && E <= MOE_MAX_EXPERTS, "moe_receive_segments: E=%d outside [1,%d]", E, MOE_MAX_EXPERTS);
    REQUIRE(G >= 1 && G <= MOE_MAX_GPUS, "moe_receive_segments: G=%d outside [1,%d]", G, MOE_MAX_GPUS);
    REQUIRE(dest >= 0 && dest < G, "moe_receive_segments: dest=%d outside [0,G=%d)", dest, G);
    REQUIRE(max_seg >= 1 && max_seg <= MOE_MAX_EXPERTS, "moe_receive_segments: max_seg=%d outside [1,%d]", max_seg, MOE_MAX_EXPERTS);
    REQUIRE(expert_counts_all && placement && seg_expert && seg_counts && seg_start, "moe_receive_segments: NULL pointer");
    return launch_receive_segments(expert_counts_all, placement, E, G, dest, max_seg, seg_expert, seg_counts, seg_start, src_offset,
                                   n_seg, (hipStream_t)stream);
}

int moe_combine(const void* ffn_out, moe_dtype_t dt, const int32_t* inv_perm, const int32_t* topk_idx,
                const float* topk_w, const int32_t* placement, int local_gpu, int T, int d, int E, int k,
                void* y, void* stream) {
    REQUIRE(dt == MOE_F32 || dt == MOE_BF16, "moe_combine: unknown dtype %d", (int)dt);
    REQUIRE(T >= 0, "moe_combine: T=%d < 0", T);
    REQUIRE(E >= 1 && E <= MOE_MAX_EXPERTS, "moe_combine: E=%d outside [1,%d]", E, MOE_MAX_EXPERTS);
    REQUIRE(k >= 1 && k <= E && k <= MOE_MAX_TOPK, "moe_combine: k=%d outside [1,min(E=%d,%d)]", k, E, MOE_MAX_TOPK);
    REQUIRE(d >= 1 && ((long long)d * elt_bytes(dt)) % 16 == 0, "moe_combine: a row (d=%d) must be a positive multiple of 16 bytes", d);
    REQUIRE(local_gpu >= -1 && local_gpu < MOE_MAX_GPUS, "moe_combine: local_gpu=%d outside [-1,%d)", local_gpu, MOE_MAX_GPUS);
    REQUIRE((long long)T * k < (1ll << 31), "moe_combine: T*k does not fit int32");
    if (T == 0) return MOE_OK;
    REQUIRE(ffn_out && inv_perm && topk_idx && topk_w && y, "moe_combine: NULL pointer");
    REQUIRE(local_gpu < 0 || placement, "moe_combine: placement is required when local_gpu >= 0");
    REQUIRE(aligned16(ffn_out) && aligned16(y), "moe_combine: ffn_out/y must be 16-byte aligned");
    return launch_combine(ffn_out, dt, inv_perm, topk_idx, topk_w, placement, local_gpu, T, d, E, k, y, (hipStream_t)stream);
}

int moe_transition_counts_pairs(const int32_t* idx_l, const int32_t* idx_l1, int T, int k_l, int k_l1, int E_l, int E_l1,
                                moe_pairs_t pairs, int64_t* R, void* stream) {
    REQUIRE(pairs == MOE_PAIRS_ALL || pairs == MOE_PAIRS_TOP1, "moe_transition_counts: unknown pair mode %d", (int)pairs);
    REQUIRE(T >= 0, "moe_transition_counts: T=%d < 0", T);
    REQUIRE(E_l >= 1 && E_l <= MOE_MAX_EXPERTS && E_l1 >= 1 && E_l1 <= MOE_MAX_EXPERTS,
            "moe_transition_counts: E_l=%d, E_l1=%d outside [1,%d]", E_l, E_l1, MOE_MAX_EXPERTS);
    REQUIRE(k_l >= 1 && k_l <= E_l && k_l <= MOE_MAX_TOPK && k_l1 >= 1 && k_l1 <= E_l1 && k_l1 <= MOE_MAX_TOPK,
            "moe_transition_counts: k_l=%d, k_l1=%d out of range", k_l, k_l1);
    REQUIRE((long long)T * k_l < (1ll << 31) && (long long)T * k_l1 < (1ll << 31), "moe_transition_counts: T*k does not fit int32");
    REQUIRE(R != nullptr, "moe_transition_counts: NULL R");
    if (T == 0) return MOE_OK;
    REQUIRE(idx_l && idx_l1, "moe_transition_counts: NULL index pointer");
    return launch_transition(idx_l, idx_l1, T, k_l, k_l1, E_l, E_l1, pairs == MOE_PAIRS_TOP1, R, (hipStream_t)stream);
}

int moe_transition_counts(const int32_t* idx_l, const int32_t* idx_l1, int T, int k_l, int k_l1, int E_l, int E_l1,
                          int64_t* R, void* stream) {
    return moe_transition_counts_pairs(idx_l, idx_l1, T, k_l, k_l1, E_l, E_l1, MOE_PAIRS_ALL, R, stream);
}

int moe_accumulate_counts(const int32_t* expert_counts, int E, int64_t* P, void* stream) {
    REQUIRE(E >= 1 && E <= MOE_MAX_EXPERTS, "moe_accumulate_counts: E=%d outside [1,%d]", E, MOE_MAX_EXPERTS);
    REQUIRE(expert_counts && P, "moe_accumulate_counts: NULL pointer");
    return launch_accumulate_counts(expert_counts, E, P, (hipStream_t)stream);
}

int moe_placement_loads(const int64_t* P, const int32_t* placement, int E, int G, int64_t* T_c, double* imbalance, void* stream) {
    REQUIRE(E >= 1 && E <= MOE_MAX_EXPERTS, "moe_placement_loads: E=%d outside [1,%d]", E, MOE_MAX_EXPERTS);
    REQUIRE(G >= 1 && G <= MOE_MAX_GPUS, "moe_placement_loads: G=%d outside [1,%d]", G, MOE_MAX_GPUS);
    REQUIRE(P && placement && T_c, "moe_placement_loads: NULL pointer");
    return launch_placement_loads(P, placement, E, G, T_c, imbalance, (hipStream_t)stream);
}

int moe_placement_traffic(const int64_t* R, const int32_t* placement_l, const int32_t* placement_l1, int E_l, int E_l1, int G,
                          int64_t* C, const double* B, double* max_cost, void* stream) {
    REQUIRE(E_l >= 1 && E_l <= MOE_MAX_EXPERTS && E_l1 >= 1 && E_l1 <= MOE_MAX_EXPERTS,
            "moe_placement_traffic: E_l=%d, E_l1=%d outside [1,%d]", E_l, E_l1, MOE_MAX_EXPERTS);
    REQUIRE(G >= 1 && G <= MOE_MAX_GPUS, "moe_placement_traffic: G=%d outside [1,%d]", G, MOE_MAX_GPUS);
    REQUIRE(R && placement_l && placement_l1 && C, "moe_placement_traffic: NULL pointer");
    return launch_placement_traffic(R, placement_l, placement_l1, E_l, E_l1, G, C, B, max_cost, (hipStream_t)stream);
}

}  // extern "C"
