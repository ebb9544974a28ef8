"""ctypes binding of libmoetuner_hip.so: argument marshalling only.

Every function has the name and argument order of its C entry point in
include/moetuner.h and takes torch tensors that already live on the GPU (torch
is used for device memory and streams, nothing else).  Kernels are enqueued on
torch's current stream.  There is no fallback: if the shared library is missing
the import fails, and a non-zero status raises MoeError with the library's
message.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmoetuner_hip.so")

MOE_F32, MOE_BF16 = 0, 1
MOE_NORM_SOFTMAX_SELECTED, MOE_NORM_SOFTMAX_ALL = 0, 1
MOE_PAIRS_ALL, MOE_PAIRS_TOP1 = 0, 1
MOE_MAX_EXPERTS, MOE_MAX_GPUS, MOE_MAX_TOPK = 256, 256, 16
FFN_STREAMING_MAX_ROWS = 160      # bf16 batches of at most this many routes run the weight-streaming FFN kernels
KERNEL_NAMES = ["gate", "dispatch_count", "dispatch_scan", "dispatch_rank", "dispatch_rows",
                "ffn_plan", "ffn_up", "ffn_down", "combine", "transition", "router"]
MOE_K_COUNT = len(KERNEL_NAMES)

EXPORTS = ["moe_last_error", "moe_version", "moe_topk_gate", "moe_topk_gate_norm", "moe_router_packed_bytes", "moe_pack_router", "moe_router_gate", "moe_dispatch_workspace_bytes", "moe_dispatch",
           "moe_dispatch_static_scratch_bytes", "moe_dispatch_noalloc",
           "moe_packed_weights_bytes", "moe_pack_weights", "moe_ffn_workspace_bytes", "moe_expert_ffn_grouped", "moe_expert_ffn_segments",
           "moe_receive_segments", "moe_combine", "moe_transition_counts", "moe_transition_counts_pairs", "moe_accumulate_counts", "moe_placement_loads",
           "moe_placement_traffic", "moe_timing_begin", "moe_timing_end"]


class MoeError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__(f"libmoetuner_hip status {status}: {msg}")
        self.status = status


if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2502_06643_amd.build` "
                      "(there is no fallback path)")
_lib = ctypes.CDLL(LIB_PATH)

_vp, _i, _sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
_lib.moe_last_error.restype = ctypes.c_char_p
_lib.moe_version.restype = ctypes.c_char_p
_lib.moe_topk_gate.argtypes = [_vp, _i, _i, _i, _vp, _vp, _vp]
_lib.moe_topk_gate_norm.argtypes = [_vp, _i, _i, _i, _i, _vp, _vp, _vp]
_lib.moe_router_packed_bytes.argtypes = [_i, _i, _i]
_lib.moe_router_packed_bytes.restype = _sz
_lib.moe_pack_router.argtypes = [_vp, _i, _i, _i, _vp, _sz, _vp]
_lib.moe_router_gate.argtypes = [_vp, _i, _vp, _vp, _i, _i, _i, _i, _vp, _vp, _vp, _vp]
_lib.moe_dispatch_workspace_bytes.argtypes = [_i, _i, _i]
_lib.moe_dispatch_workspace_bytes.restype = _sz
_lib.moe_dispatch.argtypes = [_vp, _i, _vp, _i, _i, _i, _i, _vp, _i, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.moe_dispatch_static_scratch_bytes.argtypes = []
_lib.moe_dispatch_static_scratch_bytes.restype = _sz
_lib.moe_dispatch_noalloc.argtypes = [_vp, _i, _vp, _i, _i, _i, _i, _vp, _i, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]
_lib.moe_packed_weights_bytes.argtypes = [_i, _i, _i, _i]
_lib.moe_packed_weights_bytes.restype = _sz
_lib.moe_pack_weights.argtypes = [_vp, _vp, _vp, _i, _i, _i, _i, _vp, _sz, _vp]
_lib.moe_ffn_workspace_bytes.argtypes = [_i, _i, _i, _i, _i]
_lib.moe_ffn_workspace_bytes.restype = _sz
_lib.moe_expert_ffn_grouped.argtypes = [_vp, _i, _i, _i, _i, _i, _vp, _vp, _vp, _vp, _i, _vp, _vp, _sz, _vp]
_lib.moe_expert_ffn_segments.argtypes = [_vp, _i, _i, _i, _i, _i, _vp, _i, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.moe_receive_segments.argtypes = [_vp, _vp, _i, _i, _i, _i, _vp, _vp, _vp, _vp, _vp, _vp]
_lib.moe_combine.argtypes = [_vp, _i, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _vp, _vp]
_lib.moe_transition_counts.argtypes = [_vp, _vp, _i, _i, _i, _i, _i, _vp, _vp]
_lib.moe_transition_counts_pairs.argtypes = [_vp, _vp, _i, _i, _i, _i, _i, _i, _vp, _vp]
_lib.moe_accumulate_counts.argtypes = [_vp, _i, _vp, _vp]
_lib.moe_placement_loads.argtypes = [_vp, _vp, _i, _i, _vp, _vp, _vp]
_lib.moe_placement_traffic.argtypes = [_vp, _vp, _vp, _i, _i, _i, _vp, _vp, _vp, _vp]
_lib.moe_timing_begin.argtypes = [ctypes.c_uint, _i]
_lib.moe_timing_end.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int)]


def lib() -> ctypes.CDLL:
    return _lib


def _check(status: int) -> None:
    if status != 0:
        raise MoeError(status, _lib.moe_last_error().decode())


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return MOE_F32
    if t.dtype == torch.bfloat16:
        return MOE_BF16
    raise TypeError(f"activations must be float32 or bfloat16, got {t.dtype}")


def _dev(*tensors):
    for t in tensors:
        if t is not None and not (t.is_cuda and t.is_contiguous()):
            raise ValueError("tensors must be contiguous GPU tensors")


def moe_version() -> str:
    return _lib.moe_version().decode()


def moe_last_error() -> str:
    return _lib.moe_last_error().decode()


def moe_topk_gate(logits, T, E, k, topk_idx, topk_w):
    _dev(logits, topk_idx, topk_w)
    _check(_lib.moe_topk_gate(_ptr(logits), T, E, k, _ptr(topk_idx), _ptr(topk_w), _stream()))


def moe_topk_gate_norm(logits, T, E, k, norm, topk_idx, topk_w):
    _dev(logits, topk_idx, topk_w)
    _check(_lib.moe_topk_gate_norm(_ptr(logits), T, E, k, norm, _ptr(topk_idx), _ptr(topk_w), _stream()))


def moe_router_packed_bytes(d, E, dt) -> int:
    return _lib.moe_router_packed_bytes(d, E, dt)


def moe_pack_router(w_g, d, E, dt, packed):
    _dev(w_g, packed)
    _check(_lib.moe_pack_router(_ptr(w_g), d, E, dt, _ptr(packed), packed.numel() * packed.element_size(), _stream()))


def moe_router_gate(x, dt, packed_router, bias, T, d, E, k, logits, topk_idx, topk_w):
    _dev(x, packed_router, bias, logits, topk_idx, topk_w)
    _check(_lib.moe_router_gate(_ptr(x), dt, _ptr(packed_router), _ptr(bias), T, d, E, k, _ptr(logits), _ptr(topk_idx),
                                _ptr(topk_w), _stream()))


def moe_dispatch_workspace_bytes(T, E, k) -> int:
    return _lib.moe_dispatch_workspace_bytes(T, E, k)


def moe_dispatch(x, dt, topk_idx, T, d, E, k, placement, G, send_buf, perm, inv_perm, expert_counts,
                 expert_start, gpu_counts, gpu_offsets, workspace):
    _dev(x, topk_idx, placement, send_buf, perm, inv_perm, expert_counts, expert_start, gpu_counts, gpu_offsets, workspace)
    _check(_lib.moe_dispatch(_ptr(x), dt, _ptr(topk_idx), T, d, E, k, _ptr(placement), G, _ptr(send_buf), _ptr(perm),
                             _ptr(inv_perm), _ptr(expert_counts), _ptr(expert_start), _ptr(gpu_counts),
                             _ptr(gpu_offsets), _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()))


def moe_dispatch_static_scratch_bytes() -> int:
    return _lib.moe_dispatch_static_scratch_bytes()


def moe_dispatch_noalloc(x, dt, topk_idx, T, d, E, k, placement, G, send_buf, perm, inv_perm, expert_counts,
                         expert_start, gpu_counts, gpu_offsets):
    _dev(x, topk_idx, placement, send_buf, perm, inv_perm, expert_counts, expert_start, gpu_counts, gpu_offsets)
    _check(_lib.moe_dispatch_noalloc(_ptr(x), dt, _ptr(topk_idx), T, d, E, k, _ptr(placement), G, _ptr(send_buf), _ptr(perm),
                                     _ptr(inv_perm), _ptr(expert_counts), _ptr(expert_start), _ptr(gpu_counts),
                                     _ptr(gpu_offsets), _stream()))


def moe_packed_weights_bytes(E, d, f, dt) -> int:
    return _lib.moe_packed_weights_bytes(E, d, f, dt)


def moe_pack_weights(w1, w3, w2, E, d, f, dt, packed):
    _dev(w1, w3, w2, packed)
    _check(_lib.moe_pack_weights(_ptr(w1), _ptr(w3), _ptr(w2), E, d, f, dt, _ptr(packed),
                                 packed.numel() * packed.element_size(), _stream()))


def moe_ffn_workspace_bytes(N, d, f, E, dt) -> int:
    return _lib.moe_ffn_workspace_bytes(N, d, f, E, dt)


def moe_expert_ffn_grouped(send_buf, dt, N, d, f, E, packed_weights, expert_counts, expert_start, placement,
                           local_gpu, ffn_out, workspace):
    _dev(send_buf, packed_weights, expert_counts, expert_start, placement, ffn_out, workspace)
    _check(_lib.moe_expert_ffn_grouped(_ptr(send_buf), dt, N, d, f, E, _ptr(packed_weights), _ptr(expert_counts),
                                       _ptr(expert_start), _ptr(placement), local_gpu, _ptr(ffn_out), _ptr(workspace),
                                       workspace.numel() * workspace.element_size(), _stream()))


def moe_expert_ffn_segments(recv_buf, dt, N, d, f, E, packed_weights, n_seg, seg_expert, seg_counts, seg_start, ffn_out, workspace):
    _dev(recv_buf, packed_weights, seg_expert, seg_counts, seg_start, ffn_out, workspace)
    _check(_lib.moe_expert_ffn_segments(_ptr(recv_buf), dt, N, d, f, E, _ptr(packed_weights), n_seg, _ptr(seg_expert),
                                        _ptr(seg_counts), _ptr(seg_start), _ptr(ffn_out), _ptr(workspace),
                                        workspace.numel() * workspace.element_size(), _stream()))


def moe_receive_segments(expert_counts_all, placement, E, G, dest, max_seg, seg_expert, seg_counts, seg_start, src_offset=None,
                         n_seg=None):
    _dev(expert_counts_all, placement, seg_expert, seg_counts, seg_start, src_offset, n_seg)
    _check(_lib.moe_receive_segments(_ptr(expert_counts_all), _ptr(placement), E, G, dest, max_seg, _ptr(seg_expert),
                                     _ptr(seg_counts), _ptr(seg_start), _ptr(src_offset), _ptr(n_seg), _stream()))


def moe_combine(ffn_out, dt, inv_perm, topk_idx, topk_w, placement, local_gpu, T, d, E, k, y):
    _dev(ffn_out, inv_perm, topk_idx, topk_w, placement, y)
    _check(_lib.moe_combine(_ptr(ffn_out), dt, _ptr(inv_perm), _ptr(topk_idx), _ptr(topk_w), _ptr(placement),
                            local_gpu, T, d, E, k, _ptr(y), _stream()))


def moe_transition_counts(idx_l, idx_l1, T, k_l, k_l1, E_l, E_l1, R):
    _dev(idx_l, idx_l1, R)
    _check(_lib.moe_transition_counts(_ptr(idx_l), _ptr(idx_l1), T, k_l, k_l1, E_l, E_l1, _ptr(R), _stream()))


def moe_transition_counts_pairs(idx_l, idx_l1, T, k_l, k_l1, E_l, E_l1, pairs, R):
    _dev(idx_l, idx_l1, R)
    _check(_lib.moe_transition_counts_pairs(_ptr(idx_l), _ptr(idx_l1), T, k_l, k_l1, E_l, E_l1, pairs, _ptr(R), _stream()))


def moe_accumulate_counts(expert_counts, E, P):
    _dev(expert_counts, P)
    _check(_lib.moe_accumulate_counts(_ptr(expert_counts), E, _ptr(P), _stream()))


def moe_placement_loads(P, placement, E, G, T_c, imbalance):
    _dev(P, placement, T_c, imbalance)
    _check(_lib.moe_placement_loads(_ptr(P), _ptr(placement), E, G, _ptr(T_c), _ptr(imbalance), _stream()))


def moe_placement_traffic(R, placement_l, placement_l1, E_l, E_l1, G, C, B, max_cost):
    _dev(R, placement_l, placement_l1, C, B, max_cost)
    _check(_lib.moe_placement_traffic(_ptr(R), _ptr(placement_l), _ptr(placement_l1), E_l, E_l1, G, _ptr(C), _ptr(B),
                                      _ptr(max_cost), _stream()))


def moe_timing_begin(mask: int, max_records: int) -> None:
    _check(_lib.moe_timing_begin(mask, max_records))


def moe_timing_end():
    """Returns ({kernel name: summed ms}, {kernel name: launches})."""
    ms = (ctypes.c_double * MOE_K_COUNT)()
    n = (ctypes.c_int * MOE_K_COUNT)()
    _check(_lib.moe_timing_end(ms, n))
    return ({KERNEL_NAMES[i]: ms[i] for i in range(MOE_K_COUNT)},
            {KERNEL_NAMES[i]: n[i] for i in range(MOE_K_COUNT)})
