"""An expert-parallel group of G GPUs emulated on the one GPU that is there.

The G ranks run one after the other.  Every rank gates and dispatches its own
tokens with the library; the two all-to-alls of the layer are replaced by
device-to-device copies of the buckets (the split sizes travel to the host
first, as they do for a real all-to-all-v); every rank in turn then acts as
receiver and runs `moe_expert_ffn_segments` over the (source rank, expert)
segments it was sent; the results are copied back to the senders' bucket
positions and every rank combines.  Plumbing only: nothing here computes.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B
from .layer import MoELayer, to_device


class ExpertParallelGroup:
    def __init__(self, G, T_rank, d, f, E, k, placement, dtype, w1, w3, w2, device="cuda"):
        self.G, self.T_rank, self.d, self.f, self.E, self.k = G, T_rank, d, f, E, k
        self.placement = np.ascontiguousarray(placement, dtype=np.int32)
        # senders: all experts' outputs come back before the combine, so they combine with local_gpu = -1
        self.ranks = [MoELayer(T_rank, d, f, E, k, G, -1, dtype, device) for _ in range(G)]
        for r in self.ranks:
            r.set_placement(self.placement)
        # one packed copy of all experts serves every virtual receiver (a real rank packs only its own experts)
        self.ranks[0].set_weights(w1, w3, w2)
        self.packed, self.dt, self.tdtype = self.ranks[0].packed, self.ranks[0].dt, self.ranks[0].tdtype
        self.n_max = G * T_rank * k
        self.ws = torch.empty(B.moe_ffn_workspace_bytes(self.n_max, d, f, E, self.dt), dtype=torch.uint8, device=device)
        self.device = device
        self.received = {}        # dest -> dict(recv_buf, seg_expert, seg_counts, seg_start, out), kept for inspection

    def segments_for(self, dest, expert_counts_host):
        """(source, expert on dest) segments of dest's receive buffer, source-major, expert ascending."""
        experts = [e for e in range(self.E) if self.placement[e] == dest]
        seg_expert = np.array(experts * self.G, dtype=np.int32)
        seg_counts = np.array([expert_counts_host[s][e] for s in range(self.G) for e in experts], dtype=np.int32)
        seg_start = np.concatenate([[0], np.cumsum(seg_counts)[:-1]]).astype(np.int32) if len(seg_counts) else seg_counts
        return seg_expert, seg_counts, seg_start

    def forward(self, xs, logits):
        """xs[r] [T_rank,d] and logits[r] [T_rank,E] on the device, per rank.  Returns the ranks' y tensors."""
        for r, x, lg in zip(self.ranks, xs, logits):
            r.gate(lg)
            r.dispatch(x)
        # split sizes of the all-to-alls: to the host, like the sizes handed to an all-to-all-v
        gpu_counts = torch.stack([r.gpu_counts for r in self.ranks]).cpu().numpy()
        gpu_offsets = torch.stack([r.gpu_offsets for r in self.ranks]).cpu().numpy()
        expert_counts = torch.stack([r.expert_counts for r in self.ranks]).cpu().numpy()
        self.received = {}
        for dest in range(self.G):
            pieces = [self.ranks[s].send_buf[gpu_offsets[s][dest]:gpu_offsets[s][dest] + gpu_counts[s][dest]] for s in range(self.G)]
            recv = torch.cat(pieces, dim=0).contiguous()                       # first all-to-all
            seg_expert, seg_counts, seg_start = self.segments_for(dest, expert_counts)
            out = torch.zeros_like(recv)
            n_recv = recv.shape[0]
            if n_recv and len(seg_expert):
                B.moe_expert_ffn_segments(recv, self.dt, n_recv, self.d, self.f, self.E, self.packed, len(seg_expert),
                                          to_device(seg_expert, self.device), to_device(seg_counts, self.device),
                                          to_device(seg_start, self.device), out, self.ws)
            src_off = np.concatenate([[0], np.cumsum(gpu_counts[:, dest])])
            for s in range(self.G):                                             # second all-to-all
                lo, n = gpu_offsets[s][dest], gpu_counts[s][dest]
                self.ranks[s].ffn_out[lo:lo + n] = out[src_off[s]:src_off[s + 1]]
            self.received[dest] = dict(recv_buf=recv, seg_expert=seg_expert, seg_counts=seg_counts, seg_start=seg_start, out=out)
        for r in self.ranks:
            r.combine()
        return [r.y for r in self.ranks]
