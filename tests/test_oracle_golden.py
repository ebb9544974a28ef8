"""Pins of the oracle to what the paper prints (tests/golden/*.txt, each file
cites its passage): the contiguous baseline placement and the GPU load it
implies for the skewed layer the paper describes.  CPU only."""
import os

import numpy as np

from oracle import moe_oracle as O
from paper_2502_06643_amd import synth

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def read_pairs(name):
    rows = []
    for line in open(os.path.join(GOLDEN, name)):
        line = line.strip()
        if line and not line.startswith("#"):
            rows.append([int(v) for v in line.split()])
    return np.array(rows)


def test_contiguous_placement_is_the_papers():
    table = read_pairs("contiguous_placement_8_experts_4_gpus.txt")
    want = np.empty(8, dtype=np.int32)
    want[table[:, 0]] = table[:, 1]
    assert np.array_equal(synth.placement_contiguous(8, 4), want)


def test_dispatch_under_the_papers_placement_sends_each_expert_pair_to_its_gpu():
    table = read_pairs("contiguous_placement_8_experts_4_gpus.txt")
    pl = np.empty(8, dtype=np.int32)
    pl[table[:, 0]] = table[:, 1]
    idx = synth.random_topk_idx(3, 500, 8, 2)
    d = O.dispatch(None, idx, pl, 4)
    counts = np.bincount(idx.reshape(-1), minlength=8)
    # GPU g receives exactly the routes of experts 2g and 2g+1, as one contiguous range of the send order
    assert np.array_equal(d["gpu_counts"], counts.reshape(4, 2).sum(axis=1))
    e_sorted = idx.reshape(-1)[d["perm"]]
    for g in range(4):
        seg = e_sorted[d["gpu_offsets"][g]:d["gpu_offsets"][g + 1]]
        assert set(seg.tolist()) <= {2 * g, 2 * g + 1}


def test_layer14_skew_puts_64_percent_on_gpu0():
    share = read_pairs("layer14_skew_under_contiguous_placement.txt")
    P = np.zeros(8, dtype=np.int64)
    P[share[:, 0]] = share[:, 1] * 1000          # tokens per expert, 100000 in total
    pl = synth.placement_contiguous(8, 4)
    loads = O.cluster_loads(P, pl, 4)
    assert loads[0] == 64 * 1000 and loads.sum() == 100 * 1000
    # the same through the data path: routes with these expert frequencies, dispatched under the map
    idx = np.repeat(np.arange(8, dtype=np.int32), P // 1000)[:, None]        # 100 tokens, top-1
    d = O.dispatch(None, idx, pl, 4)
    assert d["gpu_counts"][0] == 64 and d["gpu_counts"].sum() == 100
