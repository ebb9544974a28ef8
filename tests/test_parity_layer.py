"""GPU parity of the whole hot path (gate -> dispatch -> expert FFN -> combine,
plus transition counts) on the benchmark configurations, in the launch
configuration the benchmark times.

Every configuration is compared in full: all integer outputs bit for bit, every
resident row of the expert outputs and every token of y element by element
against the fp64 oracle (its BLAS-backed FFN finishes the Mixtral-shaped
prefill batch in seconds), at the stated tolerances, end to end included.  The
measured errors are printed (run with -s to see them).
"""
import json
import os

import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from paper_2502_06643_amd import binding as B
from paper_2502_06643_amd import synth
from paper_2502_06643_amd.layer import MoELayer, to_device, to_host
from util import TOL_BF16, TOL_F32, as_f64, fro_err, rel_err

pytestmark = pytest.mark.gpu

INT_OUTPUTS = ("perm", "inv_perm", "expert_counts", "expert_start", "gpu_counts", "gpu_offsets")


def run_gpu_layer(cfg, x, lg, weights, pl, local_gpu):
    L = MoELayer(cfg.T, cfg.d, cfg.f, cfg.E, cfg.k, cfg.G, local_gpu, cfg.dtype)
    L.set_placement(pl)
    L.set_weights(*weights)
    L.forward(to_device(x), torch.from_numpy(lg).cuda())
    torch.cuda.synchronize()
    return L


def check_ints(L, ref):
    np.testing.assert_array_equal(L.topk_idx.cpu().numpy(), ref["topk_idx"])
    for n in INT_OUTPUTS:
        np.testing.assert_array_equal(getattr(L, n).cpu().numpy(), ref[n], err_msg=n)
    np.testing.assert_array_equal(to_host(L.send_buf), ref["send_buf"])
    gw = L.topk_w.cpu().numpy().astype(np.float64)
    assert np.max(np.abs(gw - ref["topk_w"]) / np.maximum(ref["topk_w"], 1e-30)) <= 1e-4


@pytest.mark.parametrize("name", ["c1", "c1b"])
@pytest.mark.parametrize("map_kind,local_gpu", [("contiguous", 0), ("contiguous", 3), ("interleaved", 1),
                                                ("uneven_1124", 3), ("uneven_1124", 0), ("contiguous", -1)])
def test_tiny_fp32_layer_full_oracle(lib, name, map_kind, local_gpu):
    cfg = synth.config(name)
    x = synth.make_x(cfg)
    lg = synth.make_logits(cfg, x)
    weights = synth.make_expert_weights(cfg)
    pl = {"contiguous": synth.placement_contiguous(8, 4),
          "interleaved": np.array([3, 0, 2, 1, 0, 3, 1, 2], dtype=np.int32),
          "uneven_1124": synth.placement_from_sizes((1, 1, 2, 4), seed=7)}[map_kind]
    ref = O.moe_layer(x, lg, cfg.k, *weights, pl, cfg.G, local_gpu)
    L = run_gpu_layer(cfg, x, lg, weights, pl, local_gpu)
    check_ints(L, ref)
    e_sorted = ref["topk_idx"].reshape(-1)[ref["perm"]]
    is_local = np.ones(cfg.T * cfg.k, dtype=bool) if local_gpu < 0 else (pl[e_sorted] == local_gpu)
    if is_local.any():
        assert rel_err(L.ffn_out.cpu().numpy()[is_local], ref["ffn_out"][is_local]) <= TOL_F32
    assert rel_err(L.y.cpu().numpy(), ref["y"]) <= TOL_F32
    assert fro_err(L.y.cpu().numpy(), ref["y"]) <= TOL_F32


def tensor_rel_err(got, ref):
    """max |got - ref| / max(|ref|, rms(ref)) with the root-mean-square of the WHOLE tensor as the floor: the
    metric for batches whose rows are all of one scale (every configuration but the chained one)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(ref * ref))) or 1.0
    return float(np.max(np.abs(got - ref) / np.maximum(np.abs(ref), rms)))


def resident_rows(ref, pl, local_gpu, N):
    """Sorted positions of the routes whose expert lives on local_gpu."""
    if local_gpu < 0:
        return np.arange(N, dtype=np.int64)
    rows = [np.arange(int(ref["expert_start"][e]), int(ref["expert_start"][e]) + int(ref["expert_counts"][e]))
            for e in range(len(pl)) if pl[e] == local_gpu]
    return np.sort(np.concatenate(rows)).astype(np.int64) if rows else np.zeros(0, dtype=np.int64)


MEASURED = []        # (label, metric, value) of every float comparison below


@pytest.fixture(scope="module", autouse=True)
def report_measured_errors():
    """After the module's tests: the table of measured errors, printed, and written as JSON to the file
    named by MOE_PARITY_REPORT when that variable is set."""
    yield
    if not MEASURED:
        return
    print("\nmeasured float errors (label | metric | value):")
    for label, metric, value in MEASURED:
        print(f"  {label} | {metric} | {value:.3e}")
    path = os.environ.get("MOE_PARITY_REPORT")
    if path:
        with open(path, "w") as fh:
            json.dump([dict(label=a, metric=b, value=c) for a, b, c in MEASURED], fh, indent=1)


def check_full_layer(cfg, L, x, lg, weights, pl, local_gpu, label, same_scale_rows=True, same_scale_tokens=None):
    """Integer outputs in full; EVERY resident row of ffn_out and EVERY token of y against the fp64 oracle
    (the fp64 FFN of all 8192 routes of the Mixtral-shaped prefill batch takes a few seconds of BLAS time).
    same_scale_rows: the rows of ffn_out are all of one scale, so the tensor-wide floor is asserted too.
    same_scale_tokens (default: same_scale_rows and the gate weights of a token's resident experts sum to
    one or nearly so, i.e. at most top-2 routing): the same for y.  With 8 of 64 experts resident and top-6
    routing a token's y is scaled by whatever part of its gate mass is local (anything from 0 to 1, most
    tokens exact zeros), a small element of a large row is then measured against a floor far below that
    row's own scale, and the tensor-wide figure is printed but not asserted.
    Returns the oracle's integer outputs and its y.  No oracle input comes from the GPU."""
    if same_scale_tokens is None:
        same_scale_tokens = same_scale_rows and cfg.k <= 2
    idx, w = O.topk_gate(lg, cfg.k)
    ref = O.dispatch(x, idx, pl, cfg.G)
    ref.update(topk_idx=idx, topk_w=w)
    check_ints(L, ref)
    N = cfg.T * cfg.k
    tol = TOL_BF16 if cfg.dtype == "bf16" else TOL_F32
    rows = resident_rows(ref, pl, local_gpu, N)
    o_ref = O.expert_ffn_grouped(ref["send_buf"], *weights, ref["expert_counts"], ref["expert_start"], pl, local_gpu)
    o_bits = to_host(L.ffn_out)
    o_gpu = as_f64(o_bits)

    def record(metric, value, bound):
        MEASURED.append((label, metric, value))
        print(f"{label}: {metric} = {value:.3e} (bound {bound:.0e})", flush=True)
        assert value <= bound, (label, metric, value)

    if rows.size:
        record("ffn_out rel_err(row rms)", rel_err(o_gpu[rows], o_ref[rows]), tol)
        if same_scale_rows:
            record("ffn_out rel_err(tensor rms)", tensor_rel_err(o_gpu[rows], o_ref[rows]), tol)
        record("ffn_out fro_err", fro_err(o_gpu[rows], o_ref[rows]), tol)
    y_gpu = as_f64(to_host(L.y))
    # combine as a stage, on inputs that come from the oracle alone: its expert outputs rounded to the activation
    # dtype and its gate weights in fp32, uploaded and combined by the library, against the oracle's combine of the same
    o_in = synth.f32_to_bf16_bits(o_ref.astype(np.float32)) if cfg.dtype == "bf16" else o_ref.astype(np.float32)
    w_in = w.astype(np.float32)
    y_stage_dev = torch.empty_like(L.y)
    B.moe_combine(to_device(o_in), L.dt, torch.from_numpy(ref["inv_perm"]).cuda(), torch.from_numpy(idx).cuda(),
                  torch.from_numpy(w_in).cuda(), L.placement, local_gpu, cfg.T, cfg.d, cfg.E, cfg.k, y_stage_dev)
    torch.cuda.synchronize()
    y_stage = O.combine(o_in, ref["inv_perm"], idx, w_in, pl, local_gpu)
    record("y (combine stage) rel_err(row rms)", rel_err(as_f64(to_host(y_stage_dev)), y_stage), tol)
    del y_stage_dev
    # end to end against the all-fp64 layer, at the same tolerance
    y_ref = O.combine(o_ref, ref["inv_perm"], idx, w, pl, local_gpu)
    record("y (end to end) rel_err(row rms)", rel_err(y_gpu, y_ref), tol)
    if same_scale_rows:
        record("y (end to end) rel_err(tensor rms)", tensor_rel_err(y_gpu, y_ref), tol if same_scale_tokens else float("inf"))
    record("y (end to end) fro_err", fro_err(y_gpu, y_ref), tol)
    ref["y"] = y_ref
    return ref


@pytest.mark.parametrize("name", ["c2", "c2b", "c3", "c4"])
def test_bf16_configs_full_size_every_row(lib, name):
    cfg = synth.config(name)
    x = synth.make_x(cfg)
    lg = synth.make_logits(cfg, x)
    weights = synth.make_expert_weights(cfg)
    pl = synth.make_placement(cfg)
    L = run_gpu_layer(cfg, x, lg, weights, pl, cfg.local_gpu)
    ref = check_full_layer(cfg, L, x, lg, weights, pl, cfg.local_gpu, name)
    share = ref["expert_counts"].max() / ref["expert_counts"].sum()
    print(f"{name}: largest expert holds {share:.3f} of the routes; gpu_counts {ref['gpu_counts'].tolist()}")


def test_c5_chained_layers_and_transition_counts(lib):
    """Four Mixtral-shaped layers.  Router logits of every layer come from the
    seeded layer-0 activations (plus the successor bonus keyed on the previous
    layer's top-1 expert), so both sides see identical logits.  Activations
    flow down the ORACLE's chain: the input of layer l+1, for the GPU and the
    oracle alike, is the oracle's y of layer l rounded to bf16 (no residual, no
    norm: the configuration names none), so no oracle input ever comes from the
    GPU; every layer's floats are checked on every row and every token.  Rows
    of the later layers differ by orders of magnitude, so only the row-scaled
    metric is asserted there.  The GPU's own y of layer l is compared with the
    same oracle y (the end-to-end check), which bounds what a free-running GPU
    chain would feed the next layer."""
    cfg = synth.config("c5")
    x0 = synth.make_x(cfg)
    pl = synth.make_placement(cfg)
    L = MoELayer(cfg.T, cfg.d, cfg.f, cfg.E, cfg.k, cfg.G, cfg.local_gpu, cfg.dtype)
    L.set_placement(pl)
    x_host = x0
    prev_idx_dev, prev_idx_ref, prev_top1 = None, None, None
    affinity = []
    for layer in range(cfg.layers):
        lg = synth.make_logits(cfg, x0, layer, prev_top1)
        weights = synth.make_expert_weights(cfg, layer)
        L.set_weights(*weights)
        L.forward(to_device(x_host), torch.from_numpy(lg).cuda())
        torch.cuda.synchronize()
        ref = check_full_layer(cfg, L, x_host, lg, weights, pl, cfg.local_gpu, f"c5 layer {layer}", same_scale_rows=layer == 0)
        if layer > 0:
            R = torch.zeros((cfg.E, cfg.E), dtype=torch.int64, device="cuda")
            lib.moe_transition_counts(prev_idx_dev, L.topk_idx, cfg.T, cfg.k, cfg.k, cfg.E, cfg.E, R)
            torch.cuda.synchronize()
            np.testing.assert_array_equal(R.cpu().numpy(), O.transition_counts(prev_idx_ref, ref["topk_idx"], cfg.E, cfg.E))
            succ = synth.successors(cfg.seed(layer - 1), cfg.E)
            affinity.append(float(np.mean([ref["topk_idx"][t, 0] in succ[prev_top1[t]] for t in range(0, cfg.T, 16)])))
        prev_idx_dev, prev_idx_ref, prev_top1 = L.topk_idx.clone(), ref["topk_idx"], ref["topk_idx"][:, 0]
        x_host = synth.f32_to_bf16_bits(ref["y"].astype(np.float32))        # the oracle's y, rounded: the next layer's input
        del weights, ref
    print("c5: fraction of tokens whose next-layer top-1 is a successor expert:", affinity)


@pytest.mark.parametrize("tp", [2, 4])
def test_tensor_parallel_expert_shards_full_size_every_row(lib, tp):
    """Section 4 runs 4EP-2TP and 4EP-4TP: every expert's FFN is cut along f over tp ranks.  One rank's
    share is the same path at f / tp (its slices of W1, W3 and W2); the all-reduce of the partial outputs
    is not part of this build.  Mixtral shape, EP=4 map, every row against the oracle like the other configs."""
    cfg = synth.config("c2b")
    cfg = cfg.with_(f=cfg.f // tp, name=f"c2b_tp{tp}")
    x = synth.make_x(cfg)
    lg = synth.make_logits(cfg, x)
    weights = synth.make_expert_weights(cfg)
    pl = synth.make_placement(cfg)
    L = run_gpu_layer(cfg, x, lg, weights, pl, cfg.local_gpu)
    check_full_layer(cfg, L, x, lg, weights, pl, cfg.local_gpu, cfg.name)


def test_tensor_parallel_shards_add_up_to_the_whole_expert(lib):
    """SwiGLU is element-wise along f, so the down projections of the f-shards add up to the unsharded
    FFN: checked on the fp32 path (1e-4), where the only difference is the order of the fp32 sums."""
    T, d, f, E, k, tp = 300, 64, 256, 4, 2, 4
    x = synth.normal(5, 0, (T, d), 1.0, "f32")
    w1 = synth.normal(5, 2, (E, d, f), 1 / np.sqrt(d), "f32")
    w3 = synth.normal(5, 3, (E, d, f), 1 / np.sqrt(d), "f32")
    w2 = synth.normal(5, 4, (E, f, d), 1 / np.sqrt(f), "f32")
    idx = synth.random_topk_idx(5, T, E, k)
    pl = np.zeros(E, dtype=np.int32)

    def ffn(w1s, w3s, w2s):
        L = MoELayer(T, d, w1s.shape[2], E, k, 1, -1, "f32")
        L.set_placement(pl)
        L.set_weights(np.ascontiguousarray(w1s), np.ascontiguousarray(w3s), np.ascontiguousarray(w2s))
        L.topk_idx.copy_(torch.from_numpy(idx))
        L.dispatch(to_device(x))
        L.ffn()
        torch.cuda.synchronize()
        return L.ffn_out.cpu().numpy().astype(np.float64)

    whole = ffn(w1, w3, w2)
    fs = f // tp
    parts = sum(ffn(w1[:, :, r * fs:(r + 1) * fs], w3[:, :, r * fs:(r + 1) * fs], w2[:, r * fs:(r + 1) * fs, :]) for r in range(tp))
    assert rel_err(parts, whole) <= TOL_F32
    dsp = O.dispatch(x, idx, pl, 1)
    ref = O.expert_ffn_grouped(dsp["send_buf"], w1, w3, w2, dsp["expert_counts"], dsp["expert_start"], pl, -1)
    assert rel_err(parts, ref) <= TOL_F32
