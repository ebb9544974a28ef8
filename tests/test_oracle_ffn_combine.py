"""Pins for oracle.expert_ffn_grouped and oracle.combine (Section 2.2 / Fig. 2:
expert FFN between two all-to-alls, then the weighted sum).

The paper prints no FFN values.  Pins: a scalar-loop fp64 SwiGLU on tiny
shapes, the closed form for d=f=1, structural identities that break under a
swapped branch / transposed weight / dropped term (W1=0 gives 0, linearity in
W3 and W2 but not in W1, row independence), the single-expert case against a
library fp64 matmul + library SiLU, identity-expert and partition-of-unity
invariants for combine, and k=1 = pure un-permute.
"""
import math

import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from paper_2502_06643_amd import synth


def scalar_ffn_row(a, W1, W3, W2):
    d, f = W1.shape
    h = []
    for i in range(f):
        u = 0.0
        v = 0.0
        for c in range(d):
            u += float(a[c]) * float(W1[c, i])
            v += float(a[c]) * float(W3[c, i])
        h.append(u / (1.0 + math.exp(-u)) * v)
    out = []
    for c in range(W2.shape[1]):
        s = 0.0
        for i in range(f):
            s += h[i] * float(W2[i, c])
        out.append(s)
    return out


def small_problem(seed, T=21, d=5, f=7, E=4, k=2, G=2):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((T, d)).astype(np.float32)
    w1 = rng.standard_normal((E, d, f)).astype(np.float32)
    w3 = rng.standard_normal((E, d, f)).astype(np.float32)
    w2 = rng.standard_normal((E, f, d)).astype(np.float32)
    idx = synth.random_topk_idx(seed, T, E, k)
    pl = (np.arange(E) % G).astype(np.int32)
    dsp = O.dispatch(x, idx, pl, G)
    return x, w1, w3, w2, idx, pl, dsp


@pytest.mark.parametrize("local_gpu", [-1, 0, 1])
def test_ffn_matches_scalar_loops(local_gpu):
    x, w1, w3, w2, idx, pl, dsp = small_problem(1)
    o = O.expert_ffn_grouped(dsp["send_buf"], w1, w3, w2, dsp["expert_counts"],
                             dsp["expert_start"], pl, local_gpu)
    e_sorted = idx.reshape(-1)[dsp["perm"]]
    for p in range(len(e_sorted)):
        e = e_sorted[p]
        if local_gpu >= 0 and pl[e] != local_gpu:
            assert not o[p].any()
            continue
        np.testing.assert_allclose(o[p], scalar_ffn_row(dsp["send_buf"][p], w1[e], w3[e], w2[e]),
                                   rtol=1e-12, atol=1e-12)


def test_ffn_scalar_closed_form():
    # d = f = 1:  o = silu(a w1) * (a w3) * w2
    a, w1, w3, w2 = 2.0, 0.75, -1.5, 3.0
    o = O.expert_ffn_grouped(np.array([[a]]), np.array([[[w1]]]), np.array([[[w3]]]),
                             np.array([[[w2]]]), [1], [0], [0], -1)
    u = a * w1
    assert o[0, 0] == pytest.approx(u / (1 + math.exp(-u)) * (a * w3) * w2, rel=1e-15)
    # swapping the branches must give something else (SiLU sits on W1)
    o2 = O.expert_ffn_grouped(np.array([[a]]), np.array([[[w3]]]), np.array([[[w1]]]),
                              np.array([[[w2]]]), [1], [0], [0], -1)
    assert abs(o2[0, 0] - o[0, 0]) > 0.1


def test_ffn_structure():
    x, w1, w3, w2, idx, pl, dsp = small_problem(2)
    w1, w3, w2 = (w.astype(np.float64) for w in (w1, w3, w2))
    args = (dsp["expert_counts"], dsp["expert_start"], pl, -1)
    base = O.expert_ffn_grouped(dsp["send_buf"], w1, w3, w2, *args)
    assert not O.expert_ffn_grouped(dsp["send_buf"], 0 * w1, w3, w2, *args).any()   # silu(0)=0
    np.testing.assert_allclose(O.expert_ffn_grouped(dsp["send_buf"], w1, 2 * w3, w2, *args), 2 * base, rtol=1e-13)
    np.testing.assert_allclose(O.expert_ffn_grouped(dsp["send_buf"], w1, w3, -3 * w2, *args), -3 * base, rtol=1e-13)
    assert not np.allclose(O.expert_ffn_grouped(dsp["send_buf"], 2 * w1, w3, w2, *args), 2 * base, rtol=1e-3)
    # row independence: reversing the rows inside one expert's bucket reverses its outputs
    e = int(np.argmax(dsp["expert_counts"]))
    s, c = dsp["expert_start"][e], dsp["expert_counts"][e]
    sb = dsp["send_buf"].copy()
    sb[s:s + c] = sb[s:s + c][::-1]
    np.testing.assert_allclose(O.expert_ffn_grouped(sb, w1, w3, w2, *args)[s:s + c], base[s:s + c][::-1], rtol=1e-13)


def test_ffn_single_expert_against_library_matmul_and_silu():
    rng = np.random.default_rng(3)
    n, d, f = 17, 12, 20
    a = rng.standard_normal((n, d)); w1 = rng.standard_normal((1, d, f))
    w3 = rng.standard_normal((1, d, f)); w2 = rng.standard_normal((1, f, d))
    o = O.expert_ffn_grouped(a, w1, w3, w2, [n], [0], [0], -1)
    ta = torch.from_numpy(a)
    ref = (torch.nn.functional.silu(ta @ torch.from_numpy(w1[0])) * (ta @ torch.from_numpy(w3[0]))) @ torch.from_numpy(w2[0])
    np.testing.assert_allclose(o, ref.numpy(), rtol=1e-12, atol=1e-12)


def test_ffn_bf16_bits_are_widened_exactly_and_positions_subset():
    rng = np.random.default_rng(4)
    T, d, f, E = 30, 8, 16, 4
    xb = synth.f32_to_bf16_bits(rng.standard_normal((T, d)).astype(np.float32))
    wb = [synth.f32_to_bf16_bits(rng.standard_normal(s).astype(np.float32)) for s in ((E, d, f), (E, d, f), (E, f, d))]
    idx = synth.random_topk_idx(4, T, E, 2)
    pl = np.zeros(E, dtype=np.int32)
    dsp = O.dispatch(xb, idx, pl, 1)
    full = O.expert_ffn_grouped(dsp["send_buf"], *wb, dsp["expert_counts"], dsp["expert_start"], pl, -1)
    asf = [synth.bf16_bits_to_f32(w) for w in wb]
    ref = O.expert_ffn_grouped(synth.bf16_bits_to_f32(dsp["send_buf"]), *asf, dsp["expert_counts"], dsp["expert_start"], pl, -1)
    np.testing.assert_array_equal(full, ref)
    # hand-decoded bf16: 0x3FC0 = 1.5, 0xC000 = -2.0
    np.testing.assert_array_equal(O.widen(np.array([0x3FC0, 0xC000, 0x0000, 0x3F80], dtype=np.uint16)), [1.5, -2.0, 0.0, 1.0])
    pos = np.array([0, 5, 2 * T - 1])
    part = O.expert_ffn_grouped(dsp["send_buf"], *wb, dsp["expert_counts"], dsp["expert_start"], pl, -1, positions=pos)
    np.testing.assert_allclose(part[pos], full[pos], rtol=1e-13)     # BLAS blocking differs with the row count
    mask = np.ones(2 * T, dtype=bool); mask[pos] = False
    assert not part[mask].any()


# ------------------------------- combine ---------------------------------
def test_combine_matches_definition_loop():
    x, w1, w3, w2, idx, pl, dsp = small_problem(5, k=3, E=6, G=3)
    rng = np.random.default_rng(5)
    o = rng.standard_normal((idx.size, 5))
    w = rng.random(idx.shape)
    for local in (-1, 0, 2):
        y = O.combine(o, dsp["inv_perm"], idx, w, pl, local)
        for t in range(idx.shape[0]):
            acc = [0.0] * 5
            for j in range(3):
                if local >= 0 and pl[idx[t, j]] != local:
                    continue
                row = o[list(dsp["perm"]).index(t * 3 + j)]       # position found by search, not inv_perm
                for c in range(5):
                    acc[c] += w[t, j] * row[c]
            np.testing.assert_allclose(y[t], acc, rtol=1e-14, atol=1e-15)


def test_identity_expert_returns_gate_weighted_input():
    """combine(dispatch(x)) with the FFN replaced by a copy: all experts
    resident -> x (weights sum to one); partial -> (sum of local weights) * x."""
    rng = np.random.default_rng(6)
    T, d, E, k, G = 64, 9, 8, 2, 4
    x = rng.standard_normal((T, d))
    lg = rng.standard_normal((T, E)).astype(np.float32)
    idx, w = O.topk_gate(lg, k)
    pl = synth.placement_contiguous(E, G)
    dsp = O.dispatch(x, idx, pl, G)
    y = O.combine(dsp["send_buf"], dsp["inv_perm"], idx, w, pl, -1)
    np.testing.assert_allclose(y, x, rtol=1e-14, atol=1e-15)
    total = np.zeros_like(x)
    for g in range(G):
        yg = O.combine(dsp["send_buf"], dsp["inv_perm"], idx, w, pl, g)
        local_w = (w * (pl[idx] == g)).sum(axis=1)
        np.testing.assert_allclose(yg, local_w[:, None] * x, rtol=1e-14, atol=1e-15)
        assert not yg[local_w == 0].any()                      # exact zeros without a local route
        total += yg
    np.testing.assert_allclose(total, y, rtol=1e-12, atol=1e-14)   # partition of unity


def test_combine_k1_is_pure_unpermute():
    rng = np.random.default_rng(7)
    T, d, E = 50, 4, 8
    x = rng.standard_normal((T, d))
    idx = synth.random_topk_idx(7, T, E, 1)
    pl = np.array([1, 0, 1, 0, 2, 2, 0, 1], dtype=np.int32)
    dsp = O.dispatch(x, idx, pl, 3)
    y = O.combine(dsp["send_buf"], dsp["inv_perm"], idx, np.ones((T, 1)), pl, -1)
    np.testing.assert_array_equal(y, x)


def test_whole_layer_equals_dense_definition():
    """y[t] = sum_j w[t,j] * FFN_{e(t,j)}(x[t]) computed token by token without
    any permutation."""
    x, w1, w3, w2, idx, pl, dsp = small_problem(8, T=15, d=4, f=6, E=4, k=2, G=2)
    lg = np.random.default_rng(8).standard_normal((15, 4)).astype(np.float32)
    r = O.moe_layer(x, lg, 2, w1, w3, w2, pl, 2, -1)
    for t in range(15):
        acc = np.zeros(4)
        for j in range(2):
            e = r["topk_idx"][t, j]
            acc += r["topk_w"][t, j] * np.array(scalar_ffn_row(x[t], w1[e], w3[e], w2[e]))
        np.testing.assert_allclose(r["y"][t], acc, rtol=1e-12, atol=1e-13)


# ---- receive side: the FFN over (source GPU, expert) segments and the exchange that builds them ----

def ranks_problem(seed, G=4, T_rank=13, d=5, f=7, E=8, k=2):
    rng = np.random.default_rng(seed)
    w1 = rng.standard_normal((E, d, f)).astype(np.float32)
    w3 = rng.standard_normal((E, d, f)).astype(np.float32)
    w2 = rng.standard_normal((E, f, d)).astype(np.float32)
    pl = rng.permutation(np.arange(E) % G).astype(np.int32)          # non-contiguous map, 2 experts per GPU
    xs = [rng.standard_normal((T_rank, d)).astype(np.float32) for _ in range(G)]
    idxs = [synth.random_topk_idx(seed * 10 + r, T_rank, E, k) for r in range(G)]
    dsps = [O.dispatch(xs[r], idxs[r], pl, G) for r in range(G)]
    return w1, w3, w2, pl, xs, idxs, dsps


def test_segments_equal_the_grouped_ffn_when_segments_are_the_experts():
    x, w1, w3, w2, idx, pl, dsp = small_problem(3)
    E = len(pl)
    a = O.expert_ffn_grouped(dsp["send_buf"], w1, w3, w2, dsp["expert_counts"], dsp["expert_start"], pl, -1)
    b = O.expert_ffn_segments(dsp["send_buf"], w1, w3, w2, np.arange(E), dsp["expert_counts"], dsp["expert_start"])
    np.testing.assert_array_equal(a, b)
    # an expert split into two segments, listed in another order: every row still gets the same result
    c0 = dsp["expert_counts"].astype(np.int64); s0 = dsp["expert_start"].astype(np.int64)
    half = c0 // 2
    se = np.concatenate([np.arange(E)[::-1], np.arange(E)])
    sc = np.concatenate([(c0 - half)[::-1], half])
    ss = np.concatenate([(s0 + half)[::-1], s0])
    np.testing.assert_allclose(O.expert_ffn_segments(dsp["send_buf"], w1, w3, w2, se, sc, ss), a, rtol=1e-13, atol=1e-13)


def test_segments_match_scalar_loops_and_reject_bad_segments():
    w1, w3, w2, pl, xs, idxs, dsps = ranks_problem(4)
    ex = O.exchange_to(dsps, pl, 2)
    o = O.expert_ffn_segments(ex["recv_buf"], w1, w3, w2, ex["seg_expert"], ex["seg_counts"], ex["seg_start"])
    for s_ in range(len(ex["seg_expert"])):
        e = ex["seg_expert"][s_]
        for p in range(ex["seg_start"][s_], ex["seg_start"][s_] + ex["seg_counts"][s_]):
            np.testing.assert_allclose(o[p], scalar_ffn_row(ex["recv_buf"][p], w1[e], w3[e], w2[e]), rtol=1e-12, atol=1e-12)
    with pytest.raises(ValueError):
        O.expert_ffn_segments(ex["recv_buf"], w1, w3, w2, [0, 1], [3, 3], [0, 2])          # overlap
    with pytest.raises(ValueError):
        O.expert_ffn_segments(ex["recv_buf"], w1, w3, w2, [0], [len(ex["recv_buf"]) + 1], [0])
    with pytest.raises(ValueError):
        O.expert_ffn_segments(ex["recv_buf"], w1, w3, w2, [99], [1], [0])


def test_exchange_routes_every_row_to_the_gpu_of_its_expert():
    w1, w3, w2, pl, xs, idxs, dsps = ranks_problem(5)
    G = 4
    total = 0
    for dest in range(G):
        ex = O.exchange_to(dsps, pl, dest)
        total += len(ex["recv_buf"])
        assert ex["seg_counts"].sum() == len(ex["recv_buf"]) == sum(int(d["gpu_counts"][dest]) for d in dsps)
        assert np.all(pl[ex["seg_expert"]] == dest)
        # brute force: walk the sources' routes in their sorted order and keep those bound for dest
        rows, experts = [], []
        for src in range(G):
            e_sorted = idxs[src].reshape(-1)[dsps[src]["perm"]]
            for p, e in enumerate(e_sorted):
                if pl[e] == dest:
                    rows.append(xs[src][dsps[src]["perm"][p] // idxs[src].shape[1]]); experts.append(e)
        np.testing.assert_array_equal(ex["recv_buf"], np.array(rows).reshape(len(rows), xs[0].shape[1]))
        seg_of_row = np.repeat(ex["seg_expert"], ex["seg_counts"])
        np.testing.assert_array_equal(seg_of_row, np.array(experts, dtype=np.int32))
        assert np.array_equal(ex["seg_start"], np.concatenate([[0], np.cumsum(ex["seg_counts"])[:-1]]))
    assert total == sum(x.shape[0] for x in xs) * idxs[0].shape[1]


def test_expert_parallel_layer_equals_the_single_gpu_layer_per_source():
    """All G receivers compute their segments, the outputs go back to the sources' bucket positions, and
    each source combines with every expert's output present: that is the all-resident layer."""
    w1, w3, w2, pl, xs, idxs, dsps = ranks_problem(6)
    G, k = 4, idxs[0].shape[1]
    back = [np.zeros((x.shape[0] * k, x.shape[1])) for x in xs]
    for dest in range(G):
        ex = O.exchange_to(dsps, pl, dest)
        o = O.expert_ffn_segments(ex["recv_buf"], w1, w3, w2, ex["seg_expert"], ex["seg_counts"], ex["seg_start"])
        for src in range(G):
            lo = int(dsps[src]["gpu_offsets"][dest]); n = int(dsps[src]["gpu_counts"][dest])
            back[src][lo:lo + n] = o[ex["src_offset"][src]:ex["src_offset"][src + 1]]
    rng = np.random.default_rng(0)
    for src in range(G):
        w = rng.random((xs[src].shape[0], k))
        y = O.combine(back[src], dsps[src]["inv_perm"], idxs[src], w, pl, -1)
        single = O.expert_ffn_grouped(dsps[src]["send_buf"], w1, w3, w2, dsps[src]["expert_counts"], dsps[src]["expert_start"], pl, -1)
        np.testing.assert_allclose(back[src], single, rtol=1e-13, atol=1e-13)
        np.testing.assert_allclose(y, O.combine(single, dsps[src]["inv_perm"], idxs[src], w, pl, -1), rtol=1e-13, atol=1e-13)
