"""GPU parity at sizes whose buffers pass 4 GiB and 2^31 elements.

The configurations' own buffers stay below 2^31 bytes, so an element or byte
offset kept in 32 bits anywhere in the row copy, the combine or the grouped
GEMM would pass every other test.  Here the send buffer of moe_dispatch is
4.9 GB (2.46e9 bf16 elements) and the intermediate H of the expert FFN 4.6 GB
(2.29e9 elements); the rows checked include the last ones, which lie at the
highest offsets.  Integer outputs and row copies are compared in full, float
outputs on sampled rows that the oracle computes one by one.
"""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from paper_2502_06643_amd import synth
from paper_2502_06643_amd.layer import MoELayer, to_device, to_host
from util import TOL_BF16, as_f64, rel_err

pytestmark = pytest.mark.gpu


def ends_and_random(rng, n, n_ends, n_random):
    """first and last n_ends of range(n) plus n_random others, sorted, distinct"""
    pick = set(range(min(n_ends, n))) | set(range(max(0, n - n_ends), n))
    pick |= set(rng.integers(0, n, size=n_random).tolist())
    return np.array(sorted(pick), dtype=np.int64)


def test_dispatch_rows_and_combine_past_4_GiB(lib):
    T, d, E, k, G = 300_000, 4096, 8, 2, 4
    assert T * k * d > 2 ** 31 and T * k * d * 2 > 2 ** 32
    x = synth.normal(71, 0, (T, d), 1.0, "bf16")
    idx = synth.random_topk_idx(71, T, E, k)
    pl = synth.placement_contiguous(E, G)
    rng = np.random.default_rng(71)
    w = rng.random((T, k)).astype(np.float32)
    ref = O.dispatch(x, idx, pl, G)

    L = MoELayer(T, d, 64, E, k, G, -1, "bf16")
    L.set_placement(pl)
    L.topk_idx.copy_(torch.from_numpy(idx))
    L.topk_w.copy_(torch.from_numpy(w))
    L.send_buf.fill_(3.0)
    L.dispatch(to_device(x))
    torch.cuda.synchronize()
    for n in ("expert_counts", "expert_start", "gpu_counts", "gpu_offsets", "perm", "inv_perm"):
        np.testing.assert_array_equal(getattr(L, n).cpu().numpy(), ref[n], err_msg=n)
    step = 50_000
    for r0 in range(0, T * k, step):                       # bit copies, compared in pieces to bound the temporaries
        got = to_host(L.send_buf[r0:r0 + step])
        assert np.array_equal(got, ref["send_buf"][r0:r0 + step]), f"send_buf rows {r0}..{r0 + step}"

    # combine on the oracle's own buffers: the expert outputs are the oracle's send buffer (an identity expert)
    L.ffn_out.copy_(to_device(ref["send_buf"]))
    L.inv_perm.copy_(torch.from_numpy(ref["inv_perm"]))
    tokens = ends_and_random(rng, T, 32, 400)
    o_sub = ref["send_buf"][ref["inv_perm"].reshape(T, k)[tokens].reshape(-1)]
    inv_sub = np.arange(len(tokens) * k, dtype=np.int32)
    for local in (-1, G - 1):                              # all resident; the last GPU, whose buckets lie at the highest offsets
        L.local_gpu = local
        L.y.fill_(5.0)
        L.combine()
        torch.cuda.synchronize()
        got = as_f64(to_host(L.y[torch.from_numpy(tokens).cuda()]))
        want = O.combine(o_sub, inv_sub, idx[tokens], w[tokens], pl, local)
        assert rel_err(got, want) <= 4e-3, local           # one bf16 rounding of a fp32 sum of k terms
        if local >= 0:
            none_local = ~(pl[idx[tokens]] == local).any(axis=1)
            assert none_local.any() and not got[none_local].any()


def test_expert_ffn_with_an_intermediate_past_2_to_31_elements(lib):
    cfg = synth.config("c2").with_(T=80_000, name="c2@T=80000")
    N = cfg.T * cfg.k
    assert N * cfg.f > 2 ** 31
    x = synth.make_x(cfg)
    idx = synth.random_topk_idx(72, cfg.T, cfg.E, cfg.k)
    pl = synth.make_placement(cfg)
    weights = synth.make_expert_weights(cfg)
    dsp = O.dispatch(x, idx, pl, cfg.G)

    L = MoELayer(cfg.T, cfg.d, cfg.f, cfg.E, cfg.k, cfg.G, -1, "bf16")
    L.set_placement(pl)
    L.set_weights(*weights)
    L.send_buf.copy_(to_device(dsp["send_buf"]))
    L.expert_counts.copy_(torch.from_numpy(dsp["expert_counts"]))
    L.expert_start.copy_(torch.from_numpy(dsp["expert_start"]))
    L.ffn()
    torch.cuda.synchronize()

    rng = np.random.default_rng(72)
    rows = []
    for e in range(cfg.E):                                 # per bucket: its ends (first and last row tiles) and random rows
        c, s = int(dsp["expert_counts"][e]), int(dsp["expert_start"][e])
        rows.append(s + ends_and_random(rng, c, 3, 6))
    rows = np.concatenate(rows)
    assert rows.max() == N - 1
    want = O.expert_ffn_grouped(dsp["send_buf"], *weights, dsp["expert_counts"], dsp["expert_start"], pl, -1, positions=rows)[rows]
    got = as_f64(to_host(L.ffn_out[torch.from_numpy(rows).cuda()]))
    err = rel_err(got, want)
    print(f"\nffn_out on {len(rows)} sampled rows of {N}: rel_err {err:.3e}")
    assert err <= TOL_BF16
