"""An expert-parallel group of G GPUs emulated on the one GPU that is there.

The G ranks run one after the other.  Every rank gates and dispatches its own
tokens with the library; the two all-to-alls of the layer are replaced by
device-to-device copies of the buckets (their split sizes travel to the host
first, as they do for a real all-to-all-v, and are used for nothing but the
copies); every rank in turn then acts as receiver: `moe_receive_segments`
builds its (source rank, expert) segment table on the device from the ranks'
stacked expert_counts (an all-gather in a real group) and
`moe_expert_ffn_segments` runs over it; the results are copied back to the
senders' bucket positions and every rank combines.  Plumbing only: nothing
here computes.
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
        self.received = {}        # dest -> dict(recv_buf, segment tables (device tensors), out), kept for inspection

    def forward(self, xs, logits):
        """xs[r] [T_rank,d] and logits[r] [T_rank,E] on the device, per rank.  Returns the ranks' y tensors."""
        for r, x, lg in zip(self.ranks, xs, logits):
            r.gate(lg)
            r.dispatch(x)
        # split sizes of the all-to-alls: to the host, like the sizes handed to an all-to-all-v
        gpu_counts = torch.stack([r.gpu_counts for r in self.ranks]).cpu().numpy()
        gpu_offsets = torch.stack([r.gpu_offsets for r in self.ranks]).cpu().numpy()
        counts_all = torch.stack([r.expert_counts for r in self.ranks]).contiguous()      # [G,E], stays on the device
        self.received = {}
        for dest in range(self.G):
            pieces = [self.ranks[s].send_buf[gpu_offsets[s][dest]:gpu_offsets[s][dest] + gpu_counts[s][dest]] for s in range(self.G)]
            recv = torch.cat(pieces, dim=0).contiguous()                       # first all-to-all
            n_seg = self.G * int((self.placement == dest).sum())              # from the map alone: no bucket size involved
            i32 = dict(dtype=torch.int32, device=self.device)
            seg_expert, seg_counts, seg_start = (torch.empty(max(1, n_seg), **i32) for _ in range(3))
            src_offset, n_seg_dev = torch.empty(self.G + 1, **i32), torch.empty(1, **i32)
            out = torch.zeros_like(recv)
            n_recv = recv.shape[0]
            if n_seg:
                B.moe_receive_segments(counts_all, self.ranks[0].placement, self.E, self.G, dest, n_seg, seg_expert, seg_counts,
                                       seg_start, src_offset, n_seg_dev)
                if n_recv:
                    B.moe_expert_ffn_segments(recv, self.dt, n_recv, self.d, self.f, self.E, self.packed, n_seg, seg_expert,
                                              seg_counts, seg_start, out, self.ws)
            src_off = np.concatenate([[0], np.cumsum(gpu_counts[:, dest])])
            for s in range(self.G):                                             # second all-to-all
                lo, n = gpu_offsets[s][dest], gpu_counts[s][dest]
                self.ranks[s].ffn_out[lo:lo + n] = out[src_off[s]:src_off[s + 1]]
            self.received[dest] = dict(recv_buf=recv, n_seg=n_seg, seg_expert=seg_expert[:n_seg], seg_counts=seg_counts[:n_seg],
                                       seg_start=seg_start[:n_seg], src_offset=src_offset, n_seg_dev=n_seg_dev, out=out)
        for r in self.ranks:
            r.combine()
        return [r.y for r in self.ranks]
