#!/usr/bin/env python3
"""Benchmark of the MoE-layer hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2] [--no-cpu-baseline]

One step = one pass of the whole hot path over one synthetic batch that is
already resident in HBM: moe_topk_gate -> moe_dispatch -> moe_expert_ffn_grouped
-> moe_combine, plus moe_transition_counts between the previous step's routing
and this one's.  The default workload is the Mixtral-8x7B-shaped prefill layer
(T=4096, d=4096, f=14336, E=8, top-2, bf16, all experts resident).  Prints ONE
JSON line; `value` is tokens/s of the whole layer.

The `roofline` object is for the dominant kernel, the up-projection grouped
GEMM with the SwiGLU epilogue: algorithmic flops (4*d*f per route that exists)
divided by that kernel's mean duration, measured with HIP events recorded
around the kernel inside the library on the stream it runs on, during the same
timed steps.  `kernels` is a per-kernel breakdown from a second, separately
timed pass (event pairs around every kernel perturb the stream slightly, so it
is kept out of `value`); the two GEMMs also report the rate at which they stream
the touched experts' weights (the bound that matters when buckets are small).
`scaled` holds the bandwidth-bound kernels (gate, transition histogram, fused
router+gate, dispatch row copy, combine) at sizes that can be held against the
HBM roofline, each once warm (one buffer set, cache resident when it fits) and
once cold (rotating buffer sets larger than the 256 MB Infinity Cache); it is
kept out of `value` as well.  `cpu_baseline` times the fp64 oracle on the host
on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E

# Bytes that cross the L2 boundary per launch of the dominant kernel (up projection), from two
# rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE) scaled by a plain 1 GiB copy of known size.  The figure is
# not measured here (counters need the profiler): it is read from the tracked summary of that measurement,
# which names the commit and the commands it came from, and is null for workloads without such a summary.
TRAFFIC_SUMMARY = os.path.join(ROOT, "profiles", "ffn_up_l2_traffic.txt")


def measured_traffic(workload):
    """{'bytes': fetch + write bytes per launch, 'commit': ...} from profiles/ffn_up_l2_traffic.txt, or None."""
    try:
        rows = [l.split() for l in open(TRAFFIC_SUMMARY) if l.strip() and not l.startswith("#")]
    except OSError:
        return None
    for r in rows:                      # workload commit fetch_bytes write_bytes
        if len(r) >= 4 and r[0] == workload:
            return {"bytes": float(r[2]) + float(r[3]), "commit": r[1]}
    return None


def scaled_block(torch, B):
    """The bandwidth-bound kernels at sizes where a launch moves enough bytes to be measured against HBM
    (at the configurations' own sizes they are launch-latency bound): algorithmic bytes / mean kernel time
    (HIP event pairs inside the library) / 8 TB/s.  'warm' repeats the call on ONE set of buffers (sets below
    256 MB then live in the Infinity Cache), 'cold' rotates over enough sets (at least 4, more than 256 MB in
    all) that every call finds its inputs in DRAM."""
    dev = "cuda"
    i32 = dict(dtype=torch.int32, device=dev)

    def timed(kernel, calls, n_sets, reps=12):
        out = {}
        for mode, sets in (("warm", 1), ("cold", n_sets)):
            for i in range(2 * sets):
                calls[i % sets]()
            torch.cuda.synchronize()
            B.moe_timing_begin(1 << B.KERNEL_NAMES.index(kernel), reps + 4)
            for i in range(reps):
                calls[i % sets]()
            torch.cuda.synchronize()
            ms, n = B.moe_timing_end()
            out[mode] = ms[kernel] / max(1, n[kernel])
        return out

    def entry(alg_bytes, t, n_sets, set_bytes, **shape):
        e = dict(shape, algorithmic_bytes=alg_bytes, buffer_sets_cold=n_sets, bytes_per_set=set_bytes)
        for mode in ("warm", "cold"):
            gbs = alg_bytes / (t[mode] * 1e-3) / 1e9
            e[mode] = {"ms": round(t[mode], 5), "GBps": round(gbs, 1), "frac": round(gbs / PEAK_HBM_GBS, 4)}
        return e

    def n_sets_for(set_bytes):
        return max(4, -(-(320 << 20) // set_bytes))

    res = {"peak_GBps": PEAK_HBM_GBS, "gate": [], "transition": [], "router_gate": [], "dispatch_rows": [], "combine": []}
    E, k = 8, 2
    for T in (1 << 20, 1 << 22):
        set_bytes = T * E * 4
        R = n_sets_for(set_bytes)
        lg = [torch.randn(T, E, device=dev) for _ in range(R)]
        idx = [torch.empty(T, k, **i32) for _ in range(R)]
        w = [torch.empty(T, k, device=dev) for _ in range(R)]
        calls = [(lambda i=i: B.moe_topk_gate(lg[i], T, E, k, idx[i], w[i])) for i in range(R)]
        res["gate"].append(entry(T * (4 * E + 8 * k), timed("gate", calls, R), R, set_bytes, T=T, E=E, k=k))
        # the histogram between two routings of the same batch: the indices just produced and a second set
        for i in range(R):
            calls[i]()
        idx2 = [torch.roll(a, 1, 0).contiguous() for a in idx]
        Rm = torch.zeros(E, E, dtype=torch.int64, device=dev)
        hcalls = [(lambda i=i: B.moe_transition_counts(idx[i], idx2[i], T, k, k, E, E, Rm)) for i in range(R)]
        res["transition"].append(entry(T * 8 * k, timed("transition", hcalls, R), R, 2 * T * k * 4, T=T, E=E, k=k))
        del lg, idx, idx2, w, calls, hcalls
    d = 4096
    for T in (16384, 65536):
        set_bytes = T * d * 2
        R = n_sets_for(set_bytes)
        x = [torch.randn(T, d, device=dev, dtype=torch.bfloat16) for _ in range(R)]
        wg = (torch.randn(d, E, device=dev) / d ** 0.5).bfloat16()
        packed = torch.empty(B.moe_router_packed_bytes(d, E, B.MOE_BF16), dtype=torch.uint8, device=dev)
        B.moe_pack_router(wg, d, E, B.MOE_BF16, packed)
        idx = [torch.empty(T, k, **i32) for _ in range(R)]
        w = [torch.empty(T, k, device=dev) for _ in range(R)]
        calls = [(lambda i=i: B.moe_router_gate(x[i], B.MOE_BF16, packed, None, T, d, E, k, None, idx[i], w[i])) for i in range(R)]
        res["router_gate"].append(entry(T * d * 2 + T * k * 8, timed("router", calls, R), R, set_bytes, T=T, d=d, E=E, k=k))
        if T != 65536:
            del x, idx, w, calls
            continue
        # dispatch rows and combine at T = 65536: x [T,d] -> send_buf [T k, d] -> y [T,d]
        N = T * k
        for i in range(R):
            calls[i]()
        pl = torch.zeros(E, **i32)
        sb = [torch.empty(N, d, device=dev, dtype=torch.bfloat16) for _ in range(R)]
        perm, inv = [torch.empty(N, **i32) for _ in range(R)], [torch.empty(N, **i32) for _ in range(R)]
        cnt, start = torch.empty(E, **i32), torch.empty(E, **i32)
        gc, go = torch.empty(1, **i32), torch.empty(2, **i32)
        ws = torch.empty(max(256, B.moe_dispatch_workspace_bytes(T, E, k)), dtype=torch.uint8, device=dev)
        dcalls = [(lambda i=i: B.moe_dispatch(x[i], B.MOE_BF16, idx[i], T, d, E, k, pl, 1, sb[i], perm[i], inv[i], cnt, start, gc, go, ws))
                  for i in range(R)]
        t = timed("dispatch_rows", dcalls, R)
        res["dispatch_rows"].append(entry(T * d * 2 + N * d * 2 + 4 * N, t, R, set_bytes * (1 + k), T=T, d=d, k=k))
        y = [torch.empty(T, d, device=dev, dtype=torch.bfloat16) for _ in range(R)]
        ccalls = [(lambda i=i: B.moe_combine(sb[i], B.MOE_BF16, inv[i], idx[i], w[i], pl, -1, T, d, E, k, y[i])) for i in range(R)]
        t = timed("combine", ccalls, R)
        res["combine"].append(entry(N * d * 2 + T * d * 2 + 12 * N, t, R, set_bytes * (1 + k), T=T, d=d, k=k))
        del x, idx, w, sb, y, perm, inv, calls, dcalls, ccalls
    torch.cuda.empty_cache()
    return res


def cpu_baseline(cfg, x, lg, weights, pl, budget_rows=8192):
    """The oracle as it stands, on the host: gate and dispatch over the whole
    batch, the fp64 expert FFN on a seeded sample of bucket rows, combine on the
    tokens that own those rows; the layer time is the integer stages plus the
    FFN/combine time scaled from the sampled routes to all routes."""
    import numpy as np
    from oracle import moe_oracle as O
    from paper_2502_06643_amd import synth

    t0 = time.perf_counter()
    idx, w = O.topk_gate(lg, cfg.k)
    dsp = O.dispatch(x, idx, pl, cfg.G)
    t_int = time.perf_counter() - t0

    rng = np.random.default_rng(0)
    e_sorted = idx.reshape(-1)[dsp["perm"]]
    local = np.ones(cfg.T * cfg.k, dtype=bool) if cfg.local_gpu < 0 else (pl[e_sorted] == cfg.local_gpu)
    cand = np.nonzero(local)[0]
    pos = np.sort(rng.choice(cand, size=min(budget_rows, cand.size), replace=False))
    t0 = time.perf_counter()
    o = O.expert_ffn_grouped(dsp["send_buf"], *weights, dsp["expert_counts"], dsp["expert_start"], pl, cfg.local_gpu, positions=pos)
    t_ffn = time.perf_counter() - t0
    tokens = np.unique(dsp["perm"][pos] // cfg.k)
    t0 = time.perf_counter()
    sub_idx, sub_w = idx[tokens], w[tokens]
    sub_inv = dsp["inv_perm"].reshape(cfg.T, cfg.k)[tokens].reshape(-1)
    O.combine(o, sub_inv, sub_idx, sub_w, pl, cfg.local_gpu)
    t_comb = time.perf_counter() - t0
    n_local = int(cand.size)
    scale = n_local / max(1, pos.size)
    t_layer = t_int + t_ffn * scale + t_comb * (cfg.T / max(1, tokens.size))
    return {
        "value": cfg.T / t_layer, "unit": "tokens/s", "cores": synth.n_threads(), "kind": "oracle",
        "sample": (f"gate+dispatch on all {cfg.T} tokens ({t_int:.2f} s); fp64 FFN on {pos.size} of {n_local} resident routes "
                   f"({t_ffn:.2f} s, includes widening the experts' weights to fp64) and combine on their {tokens.size} tokens, "
                   f"scaled to the whole batch"),
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="c2")
    ap.add_argument("--tokens", type=int, default=0,
                    help="override the workload's token count T (scaled shapes for the bandwidth-bound kernels)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-breakdown", action="store_true")
    ap.add_argument("--no-scaled", action="store_true",
                    help="skip the 'scaled' block (gate, histogram, router, dispatch rows and combine at sizes that can be held "
                         "against the HBM roofline, warm and cold)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device-to-device copy three times, so that a rocprofv3 --pmc run of this "
                         "command holds a kernel of known traffic to scale FETCH_SIZE / WRITE_SIZE with")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (no collectives, no sharding); run it with --gpus 1")

    import numpy as np
    import torch
    from paper_2502_06643_amd import binding as B
    from paper_2502_06643_amd import synth
    from paper_2502_06643_amd.layer import MoELayer, to_device

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    torch.cuda.set_device(0)

    cfg = synth.config(args.workload)
    if args.tokens > 0:
        cfg = cfg.with_(T=args.tokens, name=f"{cfg.name}@T={args.tokens}")
    x = synth.make_x(cfg)
    lg = synth.make_logits(cfg, x)
    weights = synth.make_expert_weights(cfg)
    pl = synth.make_placement(cfg)

    L = MoELayer(cfg.T, cfg.d, cfg.f, cfg.E, cfg.k, cfg.G, cfg.local_gpu, cfg.dtype)
    L.set_placement(pl)
    L.set_weights(*weights)
    x_dev, lg_dev = to_device(x), torch.from_numpy(lg).cuda()
    prev_idx = torch.zeros_like(L.topk_idx)
    R = torch.zeros((cfg.E, cfg.E), dtype=torch.int64, device="cuda")

    def step():
        L.forward(x_dev, lg_dev)
        B.moe_transition_counts(prev_idx, L.topk_idx, cfg.T, cfg.k, cfg.k, cfg.E, cfg.E, R)
        prev_idx.copy_(L.topk_idx, non_blocking=True)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    up_bit = 1 << B.KERNEL_NAMES.index("ffn_up")
    B.moe_timing_begin(up_bit, args.steps + 4)
    torch.cuda.synchronize()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]   # step boundaries, for min / max
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(args.steps):
        step()
        marks[i + 1].record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    per_step = [marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps)]
    ms_sum, launches = B.moe_timing_end()
    ms_per_step = elapsed / args.steps * 1e3

    counts = L.expert_counts.cpu().numpy()
    n_local = int(counts.sum() if cfg.local_gpu < 0 else counts[pl == cfg.local_gpu].sum())
    elt = 2 if cfg.dtype == "bf16" else 4
    up_ms = ms_sum["ffn_up"] / max(1, launches["ffn_up"])
    up_flops = 4.0 * cfg.d * cfg.f * n_local
    achieved = up_flops / (up_ms * 1e-3) / 1e12
    peak = PEAK_BF16_TFLOPS if cfg.dtype == "bf16" else 157.3
    roofline = {"bound": "mfma", "kernel": "ffn_up (A.[W1|W3] + SwiGLU)", "achieved": round(achieved, 2), "peak": peak,
                "unit": "TFLOP/s", "frac": round(achieved / peak, 4), "traffic": None,
                "ms": round(up_ms, 4), "flops_per_launch": up_flops}
    if cfg.dtype == "bf16" and cfg.T * cfg.k <= B.FFN_STREAMING_MAX_ROWS:
        # decode-sized batch: the up projection streams every touched expert's W1 and W3 once and is bound by HBM
        touched = int((counts > 0).sum() if cfg.local_gpu < 0 else (counts[pl == cfg.local_gpu] > 0).sum())
        up_bytes = touched * 2.0 * cfg.d * cfg.f * elt + n_local * (cfg.d + cfg.f) * elt
        gbs = up_bytes / (up_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": "ffn_up (weight streaming, decode-sized batch)", "achieved": round(gbs, 1),
                    "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(gbs / PEAK_HBM_GBS, 4), "traffic": None,
                    "ms": round(up_ms, 4), "bytes_per_launch": up_bytes}

    traffic = measured_traffic(cfg.name)
    if traffic is not None:
        roofline["traffic"] = traffic["bytes"]
        roofline["traffic_source"] = f"profiles/ffn_up_l2_traffic.txt (rocprofv3 --pmc FETCH_SIZE + WRITE_SIZE, measured on commit {traffic['commit']})"

    out = {
        "metric": "MoE-layer tokens/s on 1 MI355X (Mixtral-8x7B shape)", "value": round(cfg.T / (ms_per_step * 1e-3), 1),
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "ms_per_step_min": round(min(per_step), 4), "ms_per_step_max": round(max(per_step), 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: T={cfg.T} d={cfg.d} f={cfg.f} E={cfg.E} top-{cfg.k}, {cfg.dtype}, "
                               f"G={cfg.G} local_gpu={cfg.local_gpu}, Zipf({cfg.zipf_s}) router bias",
                   "routes_on_this_gpu": n_local, "largest_expert_share": round(float(counts.max()) / max(1, counts.sum()), 4)},
        "roofline": roofline,
    }

    if args.copy_calibration:
        src = torch.zeros(1 << 28, dtype=torch.int32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if not args.no_breakdown:
        n_rep = max(5, min(args.steps, 20))
        B.moe_timing_begin((1 << B.MOE_K_COUNT) - 1, n_rep * 16)
        for _ in range(n_rep):
            step()
        torch.cuda.synchronize()
        ms_all, n_all = B.moe_timing_end()
        N, T, d, f, E, k = cfg.T * cfg.k, cfg.T, cfg.d, cfg.f, cfg.E, cfg.k
        alg_bytes = {
            "gate": T * (4 * E + 8 * k),
            "dispatch_rows": T * d * elt + N * d * elt + 4 * N,
            "combine": n_local * d * elt + T * d * elt + 12 * N,
            "transition": 8 * N,
        }
        alg_flops = {"ffn_up": 4.0 * d * f * n_local, "ffn_down": 2.0 * d * f * n_local}
        # the grouped GEMMs also stream every touched resident expert's weights once: the second bound, which is the
        # binding one when buckets are small (decode-sized batches, the many-expert layer)
        resident = counts if cfg.local_gpu < 0 else counts[pl == cfg.local_gpu]
        touched_experts = int((resident > 0).sum())
        weight_bytes = {"ffn_up": touched_experts * 2.0 * d * f * elt, "ffn_down": touched_experts * 1.0 * d * f * elt}
        kern = {}
        for name in B.KERNEL_NAMES:
            if not n_all[name]:
                continue
            ms = ms_all[name] / n_all[name]
            ent = {"ms": round(ms, 5)}
            if name in alg_bytes:
                gbs = alg_bytes[name] / (ms * 1e-3) / 1e9
                ent.update(bound="hbm", achieved_GBps=round(gbs, 1), frac=round(gbs / PEAK_HBM_GBS, 4))
            if name in alg_flops:
                tf = alg_flops[name] / (ms * 1e-3) / 1e12
                wgbs = weight_bytes[name] / (ms * 1e-3) / 1e9
                ent.update(bound="mfma", achieved_TFLOPs=round(tf, 1), frac=round(tf / peak, 4),
                           weight_stream_GBps=round(wgbs, 1), weight_stream_frac=round(wgbs / PEAK_HBM_GBS, 4))
            kern[name] = ent
        out["kernels"] = kern

    if not args.no_scaled:
        del L, x_dev, lg_dev
        torch.cuda.empty_cache()
        out["scaled"] = scaled_block(torch, B)

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, x, lg, weights, pl)
        out["cpu_baseline"]["value"] = round(out["cpu_baseline"]["value"], 2)

    print(json.dumps(out))


if __name__ == "__main__":
    main()
