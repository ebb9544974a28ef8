/*
 * moetuner.h - C ABI of libmoetuner_hip: the per-GPU hot path of an
 * expert-parallel Mixture-of-Experts layer on AMD MI355X (gfx950).
 *
 * The layer is the one whose per-GPU token load and GPU-to-GPU routing skew the
 * MoETuner paper (arXiv 2502.06643) balances with its expert placement: a
 * sparse top-k router (Section 2.1), token dispatch to the GPU that owns each
 * selected expert under an expert->GPU map that is contiguous by default
 * (Section 1; Section 4.2 "Baseline") or arbitrary and uneven per layer after
 * the placement optimisation (Section 3.1 "Custom Expert Parallelism"), the
 * expert FFN between the two all-to-alls (Section 2.2, Fig. 2b), the weighted
 * combine after the second one, and the two profiled statistics that feed the
 * placement ILPs: P_{e,l}, tokens routed to expert e of layer l (Section 3.2,
 * ILP 1 inputs), and R_{e1,e2,l}, tokens routed from expert e1 of layer l to
 * expert e2 of layer l+1 (Section 2.4; Section 3.2, ILP 2 inputs).
 *
 * Everything here is one GPU's share: the send buffers are laid out but never
 * sent, and only the experts resident on `local_gpu` are evaluated.
 *
 * General conventions
 * -------------------
 *  - Every pointer argument is DEVICE memory owned by the caller unless the
 *    comment says "host".  The library allocates no device memory in these
 *    calls; scratch space comes from caller workspaces sized by the *_bytes
 *    queries.  Buffers must be 16-byte aligned.
 *  - `stream` is a hipStream_t passed as void* (NULL = the null stream).  All
 *    calls are asynchronous: they enqueue kernels and return; none of them
 *    synchronises or copies to the host.  Data-dependent sizes (bucket sizes)
 *    stay on the device and are read there by the next call.
 *  - Return value: MOE_OK or a negative moe_status_t.  Scalar arguments are
 *    validated on the host; on failure nothing is enqueued and
 *    moe_last_error() describes the problem.  Device-side CONTENTS
 *    (placement[e] in [0,G), topk_idx in [0,E)) are the caller's contract:
 *    kernels skip out-of-range entries instead of faulting, but the results
 *    are then unspecified.
 *  - Stream capture: the hot calls record kernels only (no memset, no copy, no
 *    synchronisation), so a caller may capture them into a HIP graph.  The
 *    first bf16 moe_expert_ffn_grouped / _segments call on each device
 *    queries the device and raises its kernels' LDS limits (host-side calls;
 *    the result is kept per device, a failure is reported and tried again by
 *    the next call), and the first moe_dispatch_noalloc call on a device
 *    looks up its scratch buffer: make one call of each entry point you use,
 *    on each device you use, before a capture begins.
 *  - Tokens t in [0,T); experts e in [0,E); a token's j-th choice is route
 *    r = t*k + j (j = 0 is the top-1 expert); N = T*k routes.
 *  - Row-major everywhere.  Activations are MOE_F32 (float) or MOE_BF16
 *    (bfloat16, 2 bytes); a row must be a multiple of 16 bytes.
 */
#ifndef MOETUNER_H
#define MOETUNER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MOE_MAX_EXPERTS 256   /* E <= 256 */
#define MOE_MAX_GPUS    256   /* G <= 256 */
#define MOE_MAX_TOPK    16    /* k <= 16  */

typedef enum {
    MOE_OK = 0,
    MOE_ERR_INVALID_ARG = -1,   /* bad scalar, NULL or misaligned pointer     */
    MOE_ERR_UNSUPPORTED = -2,   /* valid request outside the built kernels    */
    MOE_ERR_WORKSPACE   = -3,   /* workspace too small                        */
    MOE_ERR_HIP         = -4    /* a HIP runtime call failed                  */
} moe_status_t;

typedef enum { MOE_F32 = 0, MOE_BF16 = 1 } moe_dtype_t;

/* Gate weights: softmax over the k selected logits (the default everywhere),
 * or softmax over all E logits read at the selected experts, not renormalised. */
typedef enum { MOE_NORM_SOFTMAX_SELECTED = 0, MOE_NORM_SOFTMAX_ALL = 1 } moe_norm_t;

/* Expert pairs a token contributes to the routing history table: all
 * k_l * k_l1 pairs of its experts in the two layers, or only the pair of its
 * top-1 experts (slot 0 of either index array). */
typedef enum { MOE_PAIRS_ALL = 0, MOE_PAIRS_TOP1 = 1 } moe_pairs_t;

/* Kernels that can be timed with moe_timing_begin / moe_timing_end. */
typedef enum {
    MOE_K_GATE = 0,
    MOE_K_DISPATCH_COUNT = 1,
    MOE_K_DISPATCH_SCAN = 2,
    MOE_K_DISPATCH_RANK = 3,
    MOE_K_DISPATCH_ROWS = 4,
    MOE_K_FFN_PLAN = 5,
    MOE_K_FFN_UP = 6,          /* A.[W1|W3] with the SwiGLU epilogue          */
    MOE_K_FFN_DOWN = 7,        /* H.W2                                        */
    MOE_K_COMBINE = 8,
    MOE_K_TRANSITION = 9,
    MOE_K_ROUTER = 10,         /* x.W_g + bias of moe_router_gate              */
    MOE_K_COUNT = 11
} moe_kernel_id_t;

/* Thread-local description of the last failure on this thread; never NULL. */
const char* moe_last_error(void);

/* Library version string, e.g. "moetuner-hip 0.1 (gfx950)"; host memory owned
 * by the library. */
const char* moe_version(void);

/* ------------------------------------------------------------------------
 * moe_topk_gate - sparse top-k router (Section 2.1; Mixtral routes each token
 * to its two most relevant experts).
 *
 *   logits   [T,E] float   router logits, finite
 *   topk_idx [T,k] int32   out: the k experts with the largest logits, in
 *                          descending logit order; equal logits (including
 *                          -0.0 vs +0.0) go to the lower expert index
 *   topk_w   [T,k] float   out: softmax over the k selected logits
 *
 * Requires 1 <= k <= min(E, MOE_MAX_TOPK), E <= MOE_MAX_EXPERTS, T >= 0.
 * NaN or infinite logits are outside the contract.
 * ---------------------------------------------------------------------- */
int moe_topk_gate(const float* logits, int T, int E, int k,
                  int32_t* topk_idx, float* topk_w, void* stream);

/* moe_topk_gate with the gate-weight rule spelled out (Section 2.1 fixes the
 * top-k selection only).  MOE_NORM_SOFTMAX_SELECTED is moe_topk_gate;
 * MOE_NORM_SOFTMAX_ALL writes topk_w[t][j] = softmax(logits[t])[topk_idx[t][j]],
 * so a token's weights sum to the probability mass of its k experts.  The
 * selection and everything else are the same. */
int moe_topk_gate_norm(const float* logits, int T, int E, int k, moe_norm_t norm,
                       int32_t* topk_idx, float* topk_w, void* stream);

/* ------------------------------------------------------------------------
 * moe_router_gate - the linear router in front of the gate (Section 2.1):
 *   logits[t][e] = sum_i x[t][i] * W_g[i][e] + bias[e],   then moe_topk_gate,
 * in one kernel: the selection runs on the logits while they are still on the
 * compute unit.
 *
 *   x        [T,d] dt
 *   packed_router     W_g [d,E] re-laid out once by moe_pack_router (opaque,
 *                     >= moe_router_packed_bytes(d,E,dt) bytes)
 *   bias     [E] float, or NULL
 *   logits   [T,E] float  out, or NULL when the caller does not need them
 *   topk_idx, topk_w      as in moe_topk_gate
 *
 * MOE_BF16: bf16 inputs, fp32 accumulation in a fixed order; requires
 * d % 64 == 0.  MOE_F32: fp32 throughout.  Because the logits are rounded
 * differently than an exact product, a token whose k-th and (k+1)-th logits are
 * closer than that rounding may legitimately select the other expert.
 * ---------------------------------------------------------------------- */
size_t moe_router_packed_bytes(int d, int E, moe_dtype_t dt);

int moe_pack_router(const void* w_g /*[d,E] dt*/, int d, int E, moe_dtype_t dt,
                    void* packed, size_t packed_bytes, void* stream);

int moe_router_gate(const void* x, moe_dtype_t dt, const void* packed_router, const float* bias,
                    int T, int d, int E, int k,
                    float* logits, int32_t* topk_idx, float* topk_w, void* stream);

/* ------------------------------------------------------------------------
 * moe_dispatch - placement-aware token dispatch (Section 1 and Section 2.2:
 * tokens whose expert lives on another GPU are sent there by all-to-all;
 * Section 3.1: the expert->GPU map is per layer, arbitrary, and GPUs may own
 * different numbers of experts).
 *
 * Stable counting sort of the N routes by the key (placement[e], e): the
 * sorted order is GPU ascending, expert ascending inside a GPU, token
 * ascending inside an expert.  Produces the all-to-all send layout; nothing
 * is sent.
 *
 *   x             [T,d] dt      activations (may be NULL: index outputs only,
 *                               then send_buf may be NULL too)
 *   topk_idx      [T,k] int32
 *   placement     [E]   int32   placement[e] = GPU that owns expert e
 *   send_buf      [N,d] dt      out: send_buf[p] = x[perm[p] / k], bit copy
 *   perm          [N]   int32   out: sorted position -> route id
 *   inv_perm      [N]   int32   out: route id -> sorted position
 *   expert_counts [E]   int32   out: routes per expert (P_{e,l} of this batch)
 *   expert_start  [E]   int32   out: first sorted position of expert e (where
 *                               it would start if it is empty); not monotone
 *                               in e for non-contiguous maps
 *   gpu_counts    [G]   int32   out: routes per destination GPU (send splits)
 *   gpu_offsets   [G+1] int32   out: exclusive scan of gpu_counts
 *   workspace                   >= moe_dispatch_workspace_bytes(T,E,k) bytes
 *
 * GPUs that own no expert are allowed (empty bucket).  T = 0 is allowed.
 * ---------------------------------------------------------------------- */
size_t moe_dispatch_workspace_bytes(int T, int E, int k);

int moe_dispatch(const void* x, moe_dtype_t dt, const int32_t* topk_idx,
                 int T, int d, int E, int k,
                 const int32_t* placement, int G,
                 void* send_buf, int32_t* perm, int32_t* inv_perm,
                 int32_t* expert_counts, int32_t* expert_start,
                 int32_t* gpu_counts, int32_t* gpu_offsets,
                 void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------
 * moe_dispatch_noalloc - moe_dispatch for callers that cannot allocate device
 * memory or carry a workspace around: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, outputs,
 * kernels and errors as moe_dispatch, minus the workspace: the per-chunk
 * histograms go to a buffer of moe_dispatch_static_scratch_bytes() (256 KiB)
 * that is part of the loaded library on every GPU.  The call allocates and
 * frees nothing.  A problem with moe_dispatch_workspace_bytes(T,E,k) above
 * that size is rejected with MOE_ERR_WORKSPACE (nothing is enqueued); E = 8
 * fits for every T*k, E = 64 up to about one million routes.  All calls on one
 * GPU share the buffer: calls that may overlap there (different streams,
 * different threads) race - serialise them or use moe_dispatch.  Nothing in
 * the buffer has to survive or be cleared between calls.  The first call on a
 * device looks the buffer's address up (a host-side query, no allocation);
 * make that call before a stream capture begins.
 * ---------------------------------------------------------------------- */
size_t moe_dispatch_static_scratch_bytes(void);

int moe_dispatch_noalloc(const void* x, moe_dtype_t dt, const int32_t* topk_idx,
                         int T, int d, int E, int k,
                         const int32_t* placement, int G,
                         void* send_buf, int32_t* perm, int32_t* inv_perm,
                         int32_t* expert_counts, int32_t* expert_start,
                         int32_t* gpu_counts, int32_t* gpu_offsets, void* stream);

/* ------------------------------------------------------------------------
 * moe_pack_weights - one-time re-layout of the expert weights into the order
 * the FFN kernels stream them in (off the hot path; run once per layer).
 *
 *   w1, w3 [E,d,f] dt   up projections: W1 feeds the SiLU, W3 is the linear
 *                       branch
 *   w2     [E,f,d] dt   down projection
 *   packed              out: >= moe_packed_weights_bytes(E,d,f,dt) bytes;
 *                       opaque, only valid for the same (E,d,f,dt)
 * ---------------------------------------------------------------------- */
size_t moe_packed_weights_bytes(int E, int d, int f, moe_dtype_t dt);

int moe_pack_weights(const void* w1, const void* w3, const void* w2,
                     int E, int d, int f, moe_dtype_t dt,
                     void* packed, size_t packed_bytes, void* stream);

/* ------------------------------------------------------------------------
 * moe_expert_ffn_grouped - the expert FFN ("token processing", Section 2.2 /
 * Fig. 2b, the quantity ILP 1 balances) for every expert resident on
 * local_gpu, as a grouped GEMM over the experts' contiguous buckets:
 *
 *   for e with placement[e] == local_gpu (all e when local_gpu == -1),
 *   rows A = send_buf[expert_start[e] .. +expert_counts[e]):
 *       H = silu(A W1_e) * (A W3_e)          silu(u) = u / (1 + exp(-u))
 *       ffn_out[same rows] = H W2_e
 *
 * No gate weight is applied here.  expert_counts / expert_start are read on
 * the device (no host round trip).  MOE_BF16: inputs, H and ffn_out are bf16
 * (round to nearest even), accumulation is fp32; requires d % 64 == 0 and
 * f % 64 == 0.  MOE_F32: everything fp32; requires d % 4 == 0, f % 4 == 0.
 *
 *   send_buf  [N,d] dt
 *   ffn_out   [N,d] dt   out: rows of non-resident experts are left untouched
 *   workspace            >= moe_ffn_workspace_bytes(N,d,f,E,dt) bytes
 * ---------------------------------------------------------------------- */
size_t moe_ffn_workspace_bytes(int N, int d, int f, int E, moe_dtype_t dt);

int moe_expert_ffn_grouped(const void* send_buf, moe_dtype_t dt,
                           int N, int d, int f, int E,
                           const void* packed_weights,
                           const int32_t* expert_counts, const int32_t* expert_start,
                           const int32_t* placement, int local_gpu,
                           void* ffn_out,
                           void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------
 * moe_expert_ffn_segments - the same expert FFN on the receiving side of the
 * first all-to-all (Section 2.2 / Fig. 2b): the receive buffer is the
 * concatenation, source GPU after source GPU, of buckets that each source
 * sorted by expert, so an expert's rows arrive as one segment per source.
 * Segment s is the seg_counts[s] rows of recv_buf that start at seg_start[s]
 * and is multiplied with the weights of expert seg_expert[s]:
 *
 *       H = silu(A W1_e) * (A W3_e),   ffn_out[same rows] = H W2_e
 *
 * Several segments may name the same expert; segments must not overlap (not
 * checked).  A segment that does not lie inside [0,N) or names an expert
 * outside [0,E) is skipped.  seg_* are device arrays of n_seg <=
 * MOE_MAX_EXPERTS entries, read on the device.  Everything else (dtypes,
 * shapes, packed weights, workspace size, rows outside every segment left
 * untouched) as in moe_expert_ffn_grouped.
 * ---------------------------------------------------------------------- */
int moe_expert_ffn_segments(const void* recv_buf, moe_dtype_t dt,
                            int N, int d, int f, int E,
                            const void* packed_weights, int n_seg,
                            const int32_t* seg_expert, const int32_t* seg_counts,
                            const int32_t* seg_start, void* ffn_out,
                            void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------
 * moe_receive_segments - the segment table of the buffer GPU `dest` receives
 * from the first all-to-all (Section 2.2 / Fig. 2b), built on the device from
 * the ranks' gathered expert counts, for moe_expert_ffn_segments.
 *
 * Source rank s sends dest its bucket for dest, sorted by expert, and the
 * receive buffer is the concatenation of those buckets in source order.  With
 * e_0 < e_1 < ... the experts that placement maps to dest, segment
 * s * n_local + i names expert e_i and holds expert_counts_all[s][e_i] rows;
 * seg_start is the exclusive running sum in that order.
 *
 *   expert_counts_all [G,E] int32   row s = expert_counts of source rank s
 *                                   (what an all-gather of moe_dispatch's
 *                                   expert_counts yields); negative = 0
 *   placement         [E]   int32
 *   seg_expert, seg_counts, seg_start [max_seg] int32   out; entries past the
 *                                   last segment are empty segments (0 rows)
 *                                   at the end of the buffer, so max_seg can
 *                                   be passed on as n_seg
 *   src_offset        [G+1] int32   out, or NULL: first row of each source's
 *                                   rows; [G] = rows received in all
 *   n_seg             [1]   int32   out, or NULL: G * n_local, the number of
 *                                   segments there are; when it exceeds
 *                                   max_seg only the first max_seg were
 *                                   written and the table must not be used
 *
 * Requires 1 <= max_seg <= MOE_MAX_EXPERTS (the limit of
 * moe_expert_ffn_segments), dest in [0,G).  One small kernel; nothing visits
 * the host.
 * ---------------------------------------------------------------------- */
int moe_receive_segments(const int32_t* expert_counts_all, const int32_t* placement,
                         int E, int G, int dest, int max_seg,
                         int32_t* seg_expert, int32_t* seg_counts, int32_t* seg_start,
                         int32_t* src_offset, int32_t* n_seg, void* stream);

/* ------------------------------------------------------------------------
 * moe_combine - un-permute and gate-weight the expert outputs (the step after
 * the second all-to-all of Fig. 2b):
 *
 *   y[t] = sum over j = 0..k-1 with placement[topk_idx[t,j]] == local_gpu of
 *          topk_w[t,j] * ffn_out[inv_perm[t*k + j]]
 *
 * j ascending, fp32 accumulation, no atomics (bitwise reproducible).  Routes
 * to experts on other GPUs contribute nothing; tokens without a local route
 * give exact zeros.  local_gpu == -1: every route is local.
 *
 *   ffn_out [N,d] dt,  y [T,d] dt (out)
 * ---------------------------------------------------------------------- */
int moe_combine(const void* ffn_out, moe_dtype_t dt, const int32_t* inv_perm,
                const int32_t* topk_idx, const float* topk_w,
                const int32_t* placement, int local_gpu,
                int T, int d, int E, int k, void* y, void* stream);

/* ------------------------------------------------------------------------
 * moe_transition_counts - routing history table between neighbouring layers
 * (Section 2.4; Section 3.1 "Token Routing Profile"; ILP 2 input R):
 *
 *   R[e1][e2] += #{(t, j1, j2): idx_l[t,j1] == e1 and idx_l1[t,j2] == e2}
 *
 * All k_l * k_l1 expert pairs of a token are counted.  R is accumulated in
 * place so that a profile can be gathered over many batches; the caller zeroes
 * it first.
 *
 *   idx_l [T,k_l] int32 (layer l),  idx_l1 [T,k_l1] int32 (layer l+1)
 *   R     [E_l,E_l1] int64
 * ---------------------------------------------------------------------- */
int moe_transition_counts(const int32_t* idx_l, const int32_t* idx_l1,
                          int T, int k_l, int k_l1, int E_l, int E_l1,
                          int64_t* R, void* stream);

/* moe_transition_counts with the counted pairs spelled out (Section 3.1 says
 * "tokens routed between experts e1 and e2" without fixing what a top-k token
 * contributes).  MOE_PAIRS_ALL is moe_transition_counts; MOE_PAIRS_TOP1 adds one
 * pair per token, (idx_l[t][0], idx_l1[t][0]).  Same arguments and errors. */
int moe_transition_counts_pairs(const int32_t* idx_l, const int32_t* idx_l1,
                                int T, int k_l, int k_l1, int E_l, int E_l1,
                                moe_pairs_t pairs, int64_t* R, void* stream);

/* ------------------------------------------------------------------------
 * Placement evaluators: the inputs and objective terms of the paper's two ILPs
 * (Section 3.2) for a GIVEN expert->GPU map.  The ILP solve is not part of
 * this library.  All arrays are device memory; every call is one small kernel.
 *
 * moe_accumulate_counts: P[e] += expert_counts[e]; gathers P_{e,l} (ILP 1
 *   input) over the batches of a profiling run.  P [E] int64, caller-zeroed.
 *
 * moe_placement_loads: Eq. 2, T_c[c] = sum over e with placement[e] == c of
 *   P[e], for c in [0,G); and, when imbalance != NULL, one layer's term of
 *   Eq. 1 with the mean of Eq. 3: sum_c |T_c - (sum_e P[e]) / G| in fp64.
 *   T_c [G] int64 out, imbalance [1] double out.
 *
 * moe_placement_traffic: Eq. 9, C[c1][c2] = sum of R[e1][e2] over e1 with
 *   placement_l[e1] == c1 and e2 with placement_l1[e2] == c2 (placement_l is
 *   layer l's map, placement_l1 layer l+1's).  When max_cost != NULL it also
 *   gives one layer's term of Eq. 8 with clusters already on their GPUs:
 *   max over GPU pairs of C[g1][g2] / B[g1][g2] (B == NULL: bandwidth 1).
 *   R [E_l,E_l1] int64, C [G,G] int64 out, B [G,G] double, max_cost [1] double.
 * ---------------------------------------------------------------------- */
int moe_accumulate_counts(const int32_t* expert_counts, int E, int64_t* P, void* stream);
int moe_placement_loads(const int64_t* P, const int32_t* placement, int E, int G,
                        int64_t* T_c, double* imbalance, void* stream);
int moe_placement_traffic(const int64_t* R, const int32_t* placement_l, const int32_t* placement_l1,
                          int E_l, int E_l1, int G, int64_t* C, const double* B,
                          double* max_cost, void* stream);

/* ------------------------------------------------------------------------
 * Kernel timing.  Between moe_timing_begin and moe_timing_end every launch of
 * a kernel whose bit (1u << moe_kernel_id_t) is set in `mask` is bracketed by
 * a pair of HIP events on the stream it is launched on.  moe_timing_end
 * waits for the recorded events, then fills (host arrays of MOE_K_COUNT
 * entries) the summed milliseconds and the number of launches per kernel id.
 * At most max_records launches are recorded; later ones run untimed.  One
 * session at a time per process, begun and ended by one thread; launches
 * from other threads while it is open are recorded too, but no library call
 * may be in flight on another thread while moe_timing_end runs.
 * ---------------------------------------------------------------------- */
int moe_timing_begin(unsigned mask, int max_records);
int moe_timing_end(double* sum_ms /*host [MOE_K_COUNT]*/, int* launches /*host [MOE_K_COUNT]*/);

#ifdef __cplusplus
}
#endif
#endif /* MOETUNER_H */
