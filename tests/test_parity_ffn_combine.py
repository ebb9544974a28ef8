"""GPU parity: moe_expert_ffn_grouped and moe_combine vs the oracle.

fp32 path: max relative error <= 1e-4; bf16 in / fp32 accumulate: <= 2e-2,
with the error measured as max |got - ref| / max(|ref|, rms(ref)) and also as
a Frobenius ratio.  Sizes span several row/column tiles and ragged tails.
"""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from paper_2502_06643_amd import synth
from paper_2502_06643_amd.layer import MoELayer, to_device, to_host
from util import TOL_BF16, TOL_F32, as_f64, fro_err, rel_err

pytestmark = pytest.mark.gpu


def make_problem(seed, T, d, f, E, k, G, dtype, wscale=1.0):
    x = synth.normal(seed, 0, (T, d), 1.0, dtype)
    w1 = synth.normal(seed, 2, (E, d, f), wscale / np.sqrt(d), dtype)
    w3 = synth.normal(seed, 3, (E, d, f), wscale / np.sqrt(d), dtype)
    w2 = synth.normal(seed, 4, (E, f, d), wscale / np.sqrt(f), dtype)
    idx = synth.random_topk_idx(seed, T, E, k)
    pl = (np.arange(E) % G).astype(np.int32)
    return x, w1, w3, w2, idx, pl


def gpu_ffn(lib, x, w1, w3, w2, idx, pl, G, local_gpu, dtype):
    T, d = x.shape
    E, _, f = w1.shape
    k = idx.shape[1]
    L = MoELayer(T, d, f, E, k, G, local_gpu, dtype)
    L.set_placement(pl)
    L.set_weights(w1, w3, w2)
    L.topk_idx.copy_(torch.from_numpy(idx))
    L.dispatch(to_device(x))
    L.ffn_out.fill_(7.0)                      # sentinel: rows of non-resident experts must stay untouched
    L.ffn()
    torch.cuda.synchronize()
    return L


@pytest.mark.parametrize("dtype,T,d,f,E,k,G,local", [
    ("f32", 256, 128, 256, 8, 2, 4, 0),
    ("f32", 300, 36, 100, 5, 2, 2, 1),
    ("f32", 100, 64, 64, 3, 3, 1, -1),
    ("bf16", 700, 128, 192, 4, 2, 2, 0),
    ("bf16", 1500, 256, 320, 4, 2, 1, -1),
    ("bf16", 64, 128, 128, 8, 2, 1, -1),
    ("bf16", 900, 192, 64, 16, 4, 4, 3),
    ("bf16", 130, 64, 1408, 64, 6, 8, 2),
    ("bf16", 1700, 128, 192, 2, 1, 1, -1),      # large mean bucket: the 384-row tile path
    ("bf16", 3000, 256, 2048, 1, 1, 1, -1),     # 384-row tiles with a k-split tail in the down projection
    ("bf16", 3000, 256, 2048, 8, 1, 2, 1),      # 256-row tiles with a k-split tail
    ("bf16", 150, 128, 192, 1, 1, 1, -1),       # decode-sized batch, one bucket of 150 rows: three passes of the streaming kernels
    ("bf16", 70, 64, 1408, 2, 2, 2, 1),         # decode-sized batch, one of two experts resident, k parts in the down projection
    ("bf16", 17, 4096, 512, 8, 2, 1, -1),       # decode-sized batch at the Mixtral hidden size
])
def test_ffn_matches_oracle(lib, dtype, T, d, f, E, k, G, local):
    x, w1, w3, w2, idx, pl = make_problem(T + d, T, d, f, E, k, G, dtype)
    L = gpu_ffn(lib, x, w1, w3, w2, idx, pl, G, local, dtype)
    dsp = O.dispatch(x, idx, pl, G)
    ref = O.expert_ffn_grouped(dsp["send_buf"], w1, w3, w2, dsp["expert_counts"], dsp["expert_start"], pl, local)
    got = as_f64(to_host(L.ffn_out))
    e_sorted = idx.reshape(-1)[dsp["perm"]]
    is_local = np.ones(len(e_sorted), dtype=bool) if local < 0 else (pl[e_sorted] == local)
    tol = TOL_BF16 if dtype == "bf16" else TOL_F32
    assert is_local.any()
    assert rel_err(got[is_local], ref[is_local]) <= tol
    assert fro_err(got[is_local], ref[is_local]) <= tol
    assert np.all(got[~is_local] == 7.0)


@pytest.mark.parametrize("seed", [1, 2])
def test_ffn_random_shapes_and_routings(lib, seed):
    """25 seeded random bf16 problems per seed: sizes from a handful of rows to several thousand, 1-64 experts,
    uniform to heavily skewed routing, every expert resident or a random subset.  Together they reach every
    path of the grouped GEMM (decode kernels, both tile heights, small tiles, split tails)."""
    rng = np.random.default_rng(seed)
    for case in range(25):
        E = int(rng.choice([1, 2, 3, 4, 8, 16, 64]))
        k = int(rng.integers(1, min(E, 6) + 1))
        G = int(rng.choice([g for g in (1, 2, 4, 8) if g <= E]))
        local = -1 if G == 1 or rng.random() < 0.4 else int(rng.integers(0, G))
        d, f = 64 * int(rng.integers(1, 17)), 64 * int(rng.integers(1, 33))
        T = max(1, int(rng.choice([30, 90, 200, 500, 1100, 2300, 4000, 6000])) // k)
        x, w1, w3, w2, _, _ = make_problem(1000 * seed + case, T, d, f, E, k, G, "bf16")
        p = 1.0 / np.arange(1, E + 1) ** float(rng.choice([0.0, 1.0, 2.0]))
        idx = np.stack([rng.choice(E, size=k, replace=False, p=p / p.sum()) for _ in range(T)]).astype(np.int32)
        pl = rng.permutation(np.arange(E) % G).astype(np.int32)
        print(f"case {case}: T={T} d={d} f={f} E={E} k={k} G={G} local={local}", flush=True)
        L = gpu_ffn(lib, x, w1, w3, w2, idx, pl, G, local, "bf16")
        dsp = O.dispatch(x, idx, pl, G)
        ref = O.expert_ffn_grouped(dsp["send_buf"], w1, w3, w2, dsp["expert_counts"], dsp["expert_start"], pl, local)
        got = as_f64(to_host(L.ffn_out))
        e_sorted = idx.reshape(-1)[dsp["perm"]]
        is_local = np.ones(len(e_sorted), dtype=bool) if local < 0 else (pl[e_sorted] == local)
        if is_local.any():
            assert rel_err(got[is_local], ref[is_local]) <= TOL_BF16, case
            assert fro_err(got[is_local], ref[is_local]) <= TOL_BF16, case
        assert np.all(got[~is_local] == 7.0), case


def test_ffn_skewed_buckets_including_empty_and_single_row_experts(lib):
    T, d, f, E, k = 600, 128, 256, 8, 1
    x, w1, w3, w2, _, pl = make_problem(5, T, d, f, E, k, 1, "bf16")
    idx = np.zeros((T, 1), dtype=np.int32)
    idx[:400, 0] = 3          # one big bucket (several row tiles + a ragged tail)
    idx[400:599, 0] = 6
    idx[599, 0] = 1           # a single-row bucket; experts 0,2,4,5,7 stay empty
    L = gpu_ffn(lib, x, w1, w3, w2, idx, pl, 1, -1, "bf16")
    dsp = O.dispatch(x, idx, pl, 1)
    ref = O.expert_ffn_grouped(dsp["send_buf"], w1, w3, w2, dsp["expert_counts"], dsp["expert_start"], pl, -1)
    assert rel_err(as_f64(to_host(L.ffn_out)), ref) <= TOL_BF16


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_ffn_when_this_gpu_owns_no_expert_or_no_route(lib, dtype):
    """local_gpu owns no expert (the ILP forbids it, the library tolerates it), and a GPU whose experts got no route:
    nothing may be written and nothing may fault."""
    x, w1, w3, w2, idx, pl = make_problem(11, 200, 128, 128, 4, 1, 2, dtype)
    pl[:] = 0                                                # GPU 1 owns nothing
    L = gpu_ffn(lib, x, w1, w3, w2, idx, pl, 2, 1, dtype)
    assert torch.all(L.ffn_out.float() == 7.0)
    pl = np.array([0, 0, 0, 1], dtype=np.int32)
    idx = np.minimum(idx, 2)                                 # expert 3 (GPU 1's only one) receives nothing
    L = gpu_ffn(lib, x, w1, w3, w2, idx, pl, 2, 1, dtype)
    assert torch.all(L.ffn_out.float() == 7.0)


def test_ffn_with_the_maximum_number_of_experts(lib):
    T, d, f, E, k = 900, 64, 64, 256, 16
    x, w1, w3, w2, idx, pl = make_problem(12, T, d, f, E, k, 16, "bf16")
    L = gpu_ffn(lib, x, w1, w3, w2, idx, pl, 16, 5, "bf16")
    dsp = O.dispatch(x, idx, pl, 16)
    ref = O.expert_ffn_grouped(dsp["send_buf"], w1, w3, w2, dsp["expert_counts"], dsp["expert_start"], pl, 5)
    e_sorted = idx.reshape(-1)[dsp["perm"]]
    loc = pl[e_sorted] == 5
    got = as_f64(to_host(L.ffn_out))
    assert loc.any() and rel_err(got[loc], ref[loc]) <= TOL_BF16
    assert np.all(got[~loc] == 7.0)


# row sizes: 0.5 KB (one thread per 16-byte unit), 4 KB (four tokens per workgroup; 777 tokens leave the last
# workgroup one token), 8 KB and 16 KB (one workgroup per token, two and four units per thread)
@pytest.mark.parametrize("d_bytes", [512, 4096, 8192, 16384])
@pytest.mark.parametrize("dtype,local", [("f32", -1), ("f32", 1), ("bf16", -1), ("bf16", 2)])
def test_combine_matches_oracle(lib, dtype, local, d_bytes):
    T, E, k, G = 777, 8, 3, 4
    d = d_bytes // (2 if dtype == "bf16" else 4)
    rng = np.random.default_rng(3)
    idx = synth.random_topk_idx(3, T, E, k)
    pl = synth.placement_from_sizes((1, 1, 2, 4), seed=3)
    w = rng.random((T, k)).astype(np.float32)
    o = synth.normal(3, 9, (T * k, d), 1.0, dtype)
    dsp = O.dispatch(None, idx, pl, G)
    y = torch.full((T, d), 3.0, dtype=torch.bfloat16 if dtype == "bf16" else torch.float32, device="cuda")
    dt = lib.MOE_BF16 if dtype == "bf16" else lib.MOE_F32
    lib.moe_combine(to_device(o), dt, torch.from_numpy(dsp["inv_perm"]).cuda(), torch.from_numpy(idx).cuda(),
                    torch.from_numpy(w).cuda(), torch.from_numpy(pl).cuda(), local, T, d, E, k, y)
    torch.cuda.synchronize()
    ref = O.combine(o, dsp["inv_perm"], idx, w, pl, local)
    got = as_f64(to_host(y))
    # bf16 output rounding alone is 2^-9 relative; fp32 accumulation of k terms ~1e-7
    assert rel_err(got, ref) <= (4e-3 if dtype == "bf16" else 1e-6)
    if local >= 0:
        none_local = ~(pl[idx] == local).any(axis=1)
        assert none_local.any() and not got[none_local].any()          # exact zeros


def test_identity_expert_round_trip(lib):
    """combine(dispatch(x)) with the FFN left out returns the gate-weighted
    input: x itself when every expert is resident (fp32: to rounding)."""
    cfg = synth.config("c1b")
    x = synth.make_x(cfg)
    lg = synth.make_logits(cfg, x)
    pl = synth.make_placement(cfg)
    L = MoELayer(cfg.T, cfg.d, cfg.f, cfg.E, cfg.k, cfg.G, -1, "f32")
    L.set_placement(pl)
    L.gate(torch.from_numpy(lg).cuda())
    L.dispatch(torch.from_numpy(x).cuda())
    L.ffn_out.copy_(L.send_buf)
    L.combine()
    torch.cuda.synchronize()
    np.testing.assert_allclose(L.y.cpu().numpy(), x, rtol=1e-6, atol=1e-6)
    total = np.zeros_like(x, dtype=np.float64)
    for g in range(cfg.G):
        L.local_gpu = g
        L.combine()
        torch.cuda.synchronize()
        total += L.y.cpu().numpy()
    np.testing.assert_allclose(total, x, rtol=1e-6, atol=1e-6)            # partition of unity over the GPUs
