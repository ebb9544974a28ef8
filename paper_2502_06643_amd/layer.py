"""Device buffers for one MoE layer and the call sequence of the hot path.

Plumbing only: torch allocates the device memory, every step is a call into
libmoetuner_hip through `binding`.  Nothing here computes.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B


def to_device(a: np.ndarray, device="cuda") -> torch.Tensor:
    """numpy -> GPU tensor; uint16 arrays are bf16 bit patterns."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(a).to(device)


def to_host(t: torch.Tensor) -> np.ndarray:
    """GPU tensor -> numpy; bf16 tensors come back as uint16 bit patterns."""
    t = t.detach()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


class MoELayer:
    """Buffers and packed weights of one layer on one GPU.

    T tokens, hidden d, FFN width f, E experts, top-k, expert->GPU map
    `placement` over G GPUs, this GPU being `local_gpu` (-1: all resident).
    """

    def __init__(self, T, d, f, E, k, G, local_gpu, dtype, device="cuda"):
        assert dtype in ("f32", "bf16")
        self.T, self.d, self.f, self.E, self.k, self.G, self.local_gpu = T, d, f, E, k, G, local_gpu
        self.N = T * k
        self.dt = B.MOE_BF16 if dtype == "bf16" else B.MOE_F32
        self.tdtype = torch.bfloat16 if dtype == "bf16" else torch.float32
        self.device = device
        i32 = dict(dtype=torch.int32, device=device)
        N = self.N
        self.topk_idx = torch.empty((T, k), **i32)
        self.topk_w = torch.empty((T, k), dtype=torch.float32, device=device)
        self.send_buf = torch.empty((N, d), dtype=self.tdtype, device=device)
        self.perm = torch.empty(N, **i32)
        self.inv_perm = torch.empty(N, **i32)
        self.expert_counts = torch.empty(E, **i32)
        self.expert_start = torch.empty(E, **i32)
        self.gpu_counts = torch.empty(G, **i32)
        self.gpu_offsets = torch.empty(G + 1, **i32)
        self.ffn_out = torch.zeros((N, d), dtype=self.tdtype, device=device)
        self.y = torch.empty((T, d), dtype=self.tdtype, device=device)
        self.dispatch_ws = torch.empty(max(256, B.moe_dispatch_workspace_bytes(T, E, k)), dtype=torch.uint8, device=device)
        self.ffn_ws = torch.empty(B.moe_ffn_workspace_bytes(N, d, f, E, self.dt), dtype=torch.uint8, device=device)
        self.placement = None
        self.packed = None

    def set_placement(self, placement: np.ndarray):
        self.placement = torch.from_numpy(np.ascontiguousarray(placement, dtype=np.int32)).to(self.device)

    def set_weights(self, w1, w3, w2):
        """w1, w3 [E,d,f], w2 [E,f,d] as numpy arrays or GPU tensors; packs them once."""
        ws = [w if isinstance(w, torch.Tensor) else to_device(w, self.device) for w in (w1, w3, w2)]
        nbytes = B.moe_packed_weights_bytes(self.E, self.d, self.f, self.dt)
        self.packed = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        B.moe_pack_weights(ws[0], ws[1], ws[2], self.E, self.d, self.f, self.dt, self.packed)
        torch.cuda.synchronize()

    # -- the five calls ---------------------------------------------------------
    def gate(self, logits):
        B.moe_topk_gate(logits, self.T, self.E, self.k, self.topk_idx, self.topk_w)

    def dispatch(self, x):
        B.moe_dispatch(x, self.dt, self.topk_idx, self.T, self.d, self.E, self.k, self.placement, self.G,
                       self.send_buf, self.perm, self.inv_perm, self.expert_counts, self.expert_start,
                       self.gpu_counts, self.gpu_offsets, self.dispatch_ws)

    def ffn(self):
        B.moe_expert_ffn_grouped(self.send_buf, self.dt, self.N, self.d, self.f, self.E, self.packed,
                                 self.expert_counts, self.expert_start, self.placement, self.local_gpu,
                                 self.ffn_out, self.ffn_ws)

    def combine(self):
        B.moe_combine(self.ffn_out, self.dt, self.inv_perm, self.topk_idx, self.topk_w, self.placement,
                      self.local_gpu, self.T, self.d, self.E, self.k, self.y)

    def forward(self, x, logits):
        """One pass of the hot path: gate -> dispatch -> expert FFN -> combine."""
        self.gate(logits)
        self.dispatch(x)
        self.ffn()
        self.combine()
        return self.y
