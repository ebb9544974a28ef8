"""CPU oracle for the expert-parallel MoE layer hot path (TEST INFRASTRUCTURE ONLY).

This module is the slow, plain, fp64 statement of what the HIP library computes.
It exists so that tests, the smoke check and the benchmark's CPU-baseline leg
have something independent to compare against.  The product path never imports
it, and it imports nothing from the product path: no kernels, tables, helpers
or pre/post-processing are shared.  Only numpy is used; every function works on
host arrays and returns new host arrays.

What the paper fixes and what it leaves open
--------------------------------------------
The paper (MoETuner, Sections 1-3) states the problem: E experts per layer, a
sparse top-k router (Mixtral: top-2, Section 2.1), an expert->GPU map that puts
each expert of a layer on one of G GPUs (contiguous by default, Section 1 and
Section 4.2 "Baseline"; arbitrary and uneven per layer after the ILP, Section
3.1 "Custom Expert Parallelism"), tokens dispatched to the GPU that owns their
expert before the expert FFN and brought back afterwards (Section 2.2, Fig. 2b),
and two profiled statistics: P_{e,l}, the number of tokens routed to expert e in
layer l (ILP 1 inputs), and R_{e1,e2,l}, the number of tokens routed between
expert e1 of layer l and expert e2 of layer l+1 (ILP 2 inputs, Section 2.4).
It prints no router formula, FFN formula, buffer layout or numeric example, so
the arithmetic below follows the readings listed in the design notes of this
repository: softmax over the k selected logits, ties to the lower expert index,
SwiGLU with W1 on the SiLU branch, gate weight applied at combine, bucket order
(GPU, expert, token) ascending.

Parity pins (tests/test_oracle_*.py, all CPU): every function here is pinned to
something other than itself - brute-force definitional loops on tiny inputs,
closed forms (two-way softmax = logistic, scalar SwiGLU), library routines used
as textbook special cases (argmax, full softmax, contingency table, fp64 matmul)
and the conservation identities of Eq. 2-3 and Eq. 9.  No function is unpinned.

bf16 inputs are passed as uint16 bit patterns and widened exactly; fp32 inputs
are widened exactly; all arithmetic is fp64.
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "widen",
    "router_logits",
    "router_gate",
    "topk_gate",
    "dispatch",
    "expert_ffn_grouped",
    "combine",
    "transition_counts",
    "cluster_loads",
    "load_imbalance",
    "cluster_traffic",
    "max_pair_cost",
    "moe_layer",
]


# --------------------------------------------------------------------------
# input widening
# --------------------------------------------------------------------------
def widen(a) -> np.ndarray:
    """Exact widening of an input tensor to fp64.

    uint16 arrays are bf16 bit patterns (sign, 8 exponent bits, 7 mantissa bits
    = the upper half of an IEEE fp32); float32/float64 arrays are taken as they
    are.  Nothing is rounded: every bf16 and fp32 value is an fp64 value.
    """
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    if a.dtype in (np.float32, np.float64):
        return a.astype(np.float64)
    raise TypeError(f"unsupported input dtype {a.dtype}; pass float32, float64 or uint16 (bf16 bits)")


def _check_index_array(name, a, lo, hi):
    a = np.asarray(a)
    if not np.issubdtype(a.dtype, np.integer):
        raise TypeError(f"{name} must be an integer array")
    if a.size and (a.min() < lo or a.max() >= hi):
        raise ValueError(f"{name} has entries outside [{lo}, {hi})")
    return a.astype(np.int64)


# --------------------------------------------------------------------------
# router projection (the step in front of the gate)
# --------------------------------------------------------------------------
def router_logits(x, w_g, bias=None):
    """Router logits of a linear router (Section 2.1 describes the router that
    scores the experts for each token; the linear form is this repository's
    reading, as in Mixtral):
    logits[t, e] = sum_i x[t, i] * W_g[i, e] + bias[e], in fp64.
    x [T,d], w_g [d,E] (fp32, fp64 or bf16 bits), bias [E] or None."""
    xa, wa = widen(x), widen(w_g)
    if xa.ndim != 2 or wa.ndim != 2 or xa.shape[1] != wa.shape[0]:
        raise ValueError("x must be [T,d] and w_g [d,E]")
    lg = xa @ wa
    if bias is not None:
        b = np.asarray(bias, dtype=np.float64)
        if b.shape != (wa.shape[1],):
            raise ValueError("bias must be [E]")
        lg = lg + b[None, :]
    return lg


def router_gate(x, w_g, bias, k: int):
    """router_logits followed by topk_gate, all in fp64.
    Returns (logits float64 [T,E], topk_idx int32 [T,k], topk_w float64 [T,k])."""
    lg = router_logits(x, w_g, bias)
    idx, w = topk_gate(lg, k)
    return lg, idx, w


# --------------------------------------------------------------------------
# a1  top-k gate
# --------------------------------------------------------------------------
def topk_gate(logits, k: int, norm: str = "selected"):
    """Top-k router (Section 2.1: each token goes to its k most relevant
    experts; Mixtral uses k=2).

    For every token the experts are ranked by the total order "larger logit
    first; equal logits -> smaller expert index first" and the first k are
    kept, slot 0 being the top-1 expert.  Gate weights are the softmax over the
    k kept logits (identical to a softmax over all experts renormalised over
    the kept ones).  -0.0 and +0.0 compare equal.  Non-finite logits are
    rejected.

    norm = "all" is the other common gating rule (the paper does not say which
    one its models use beyond "top-2 router"): the weights are the softmax over
    all E logits read at the kept experts, without renormalisation, so they sum
    to the probability mass of the kept experts (< 1 unless k = E).  The
    selection is the same.

    Returns (topk_idx int32 [T,k], topk_w float64 [T,k]).
    """
    lg = np.asarray(logits)
    if lg.ndim != 2:
        raise ValueError("logits must be [T,E]")
    T, E = lg.shape
    if not (1 <= k <= E):
        raise ValueError("need 1 <= k <= E")
    lg = widen(lg)
    if not np.all(np.isfinite(lg)):
        raise ValueError("non-finite router logit")
    # stable ascending sort of the negated logits = descending logits with the
    # lower index winning ties
    order = np.argsort(-lg, axis=1, kind="stable")
    idx = order[:, :k]
    sel = np.take_along_axis(lg, idx, axis=1)
    p = np.exp(sel - sel[:, :1])
    if norm == "selected":
        w = p / p.sum(axis=1, keepdims=True)
    elif norm == "all":
        w = p / np.exp(lg - sel[:, :1]).sum(axis=1, keepdims=True)
    else:
        raise ValueError("norm must be 'selected' or 'all'")
    return idx.astype(np.int32), w


# --------------------------------------------------------------------------
# a2  placement-aware dispatch
# --------------------------------------------------------------------------
def dispatch(x, topk_idx, placement, G: int):
    """Permute the T*k routes into per-destination-GPU, per-expert buckets
    (Section 1 / Section 2.2: tokens go to the GPU that holds their expert;
    Section 3.1: the expert->GPU map is arbitrary per layer and GPUs may hold
    different numbers of experts).

    Route r = t*k + j is the j-th choice of token t.  Routes are stably sorted
    by the key (placement[expert], expert); within one expert they therefore
    stay in ascending token order.  Nothing is sent anywhere: the result is the
    send buffer layout.

    x may be None (index outputs only).  Returns a dict with
      perm          int32 [N]   sorted position -> route id
      inv_perm      int32 [N]   route id -> sorted position
      expert_counts int32 [E]   routes per expert (= P_{e,l} for this batch)
      expert_start  int32 [E]   first sorted position of expert e's bucket (the
                                position it would start at when it is empty)
      gpu_counts    int32 [G]   routes per destination GPU (all-to-all splits)
      gpu_offsets   int32 [G+1] exclusive scan of gpu_counts
      send_buf      [N,d]       x[perm // k] bit for bit, in x's dtype
    """
    idx = np.asarray(topk_idx)
    if idx.ndim != 2:
        raise ValueError("topk_idx must be [T,k]")
    T, k = idx.shape
    pl = np.asarray(placement)
    E = pl.shape[0]
    if G < 1:
        raise ValueError("G must be >= 1")
    pl = _check_index_array("placement", pl, 0, G)
    e_of_route = _check_index_array("topk_idx", idx, 0, E).reshape(T * k)
    N = T * k

    key = pl[e_of_route] * E + e_of_route
    perm = np.argsort(key, kind="stable")
    inv_perm = np.empty(N, dtype=np.int64)
    inv_perm[perm] = np.arange(N)

    expert_counts = np.zeros(E, dtype=np.int64)
    for e in e_of_route:
        expert_counts[e] += 1

    # experts in bucket order: GPUs ascending, experts ascending inside a GPU
    expert_start = np.zeros(E, dtype=np.int64)
    gpu_counts = np.zeros(G, dtype=np.int64)
    pos = 0
    for g in range(G):
        for e in range(E):
            if pl[e] == g:
                expert_start[e] = pos
                pos += expert_counts[e]
                gpu_counts[g] += expert_counts[e]
    gpu_offsets = np.zeros(G + 1, dtype=np.int64)
    for g in range(G):
        gpu_offsets[g + 1] = gpu_offsets[g] + gpu_counts[g]

    out = {
        "perm": perm.astype(np.int32),
        "inv_perm": inv_perm.astype(np.int32),
        "expert_counts": expert_counts.astype(np.int32),
        "expert_start": expert_start.astype(np.int32),
        "gpu_counts": gpu_counts.astype(np.int32),
        "gpu_offsets": gpu_offsets.astype(np.int32),
        "send_buf": None,
    }
    if x is not None:
        xa = np.asarray(x)
        if xa.ndim != 2 or xa.shape[0] != T:
            raise ValueError("x must be [T,d]")
        out["send_buf"] = xa[perm // k].copy()
    return out


# --------------------------------------------------------------------------
# a3  expert FFN over the local buckets
# --------------------------------------------------------------------------
def expert_ffn_grouped(send_buf, w1, w3, w2, expert_counts, expert_start,
                       placement, local_gpu: int, positions=None):
    """SwiGLU expert FFN ("token processing", Section 2.2 / Fig. 2) for every
    expert that lives on local_gpu, over that expert's contiguous bucket rows.

    For a row a of expert e:  u = a W1_e,  v = a W3_e,
    h_i = u_i / (1 + exp(-u_i)) * v_i,  o = h W2_e.   W1,W3 are [E,d,f], W2 is
    [E,f,d].  The gate weight is NOT applied here.  local_gpu = -1 means every
    expert is resident.  No intermediate is rounded.

    positions: optional 1-D array of sorted positions; when given, only those
    rows are computed (others stay zero) - used at sizes where the whole fp64
    FFN is out of reach.  Returns float64 [N,d]; rows outside the local buckets
    are zero and carry no meaning.
    """
    sb = np.asarray(send_buf)
    N, d = sb.shape
    w1 = np.asarray(w1); w3 = np.asarray(w3); w2 = np.asarray(w2)
    E = w1.shape[0]
    f = w1.shape[2]
    if w1.shape != (E, d, f) or w3.shape != (E, d, f) or w2.shape != (E, f, d):
        raise ValueError("weights must be W1,W3 [E,d,f] and W2 [E,f,d]")
    counts = np.asarray(expert_counts).astype(np.int64)
    starts = np.asarray(expert_start).astype(np.int64)
    pl = np.asarray(placement).astype(np.int64)
    want = None
    if positions is not None:
        want = np.zeros(N, dtype=bool)
        want[np.asarray(positions, dtype=np.int64)] = True
    out = np.zeros((N, d), dtype=np.float64)
    for e in range(E):
        if local_gpu >= 0 and pl[e] != local_gpu:
            continue
        rows = np.arange(starts[e], starts[e] + counts[e])
        if want is not None:
            rows = rows[want[rows]]
        if rows.size == 0:
            continue
        a = widen(sb[rows])
        u = a @ widen(w1[e])
        v = a @ widen(w3[e])
        with np.errstate(over="ignore"):
            h = u / (1.0 + np.exp(-u)) * v
        out[rows] = h @ widen(w2[e])
    return out


def expert_ffn_segments(recv_buf, w1, w3, w2, seg_expert, seg_counts, seg_start, positions=None):
    """The same SwiGLU FFN over row segments: segment s is the seg_counts[s]
    rows of recv_buf that start at seg_start[s] and belong to expert
    seg_expert[s].  This is what a GPU computes after the first all-to-all of
    Section 2.2 / Fig. 2b: the buffer it receives is the concatenation, source
    GPU after source GPU, of the buckets the sources sorted by expert, so an
    expert's rows arrive as one segment per source.  Several segments may name
    the same expert; segments must not overlap.  Returns float64 [N,d]; rows
    outside every segment are zero.  positions as in expert_ffn_grouped.
    """
    rb = np.asarray(recv_buf)
    N, d = rb.shape
    w1 = np.asarray(w1); w3 = np.asarray(w3); w2 = np.asarray(w2)
    E, _, f = w1.shape
    if w1.shape != (E, d, f) or w3.shape != (E, d, f) or w2.shape != (E, f, d):
        raise ValueError("weights must be W1,W3 [E,d,f] and W2 [E,f,d]")
    se = _check_index_array("seg_expert", np.asarray(seg_expert), 0, E)
    sc = np.asarray(seg_counts).astype(np.int64)
    ss = np.asarray(seg_start).astype(np.int64)
    if not (se.ndim == 1 and se.shape == sc.shape == ss.shape):
        raise ValueError("seg_expert, seg_counts, seg_start must be 1-D and of one length")
    if np.any(sc < 0) or np.any(ss < 0) or np.any(ss + sc > N):
        raise ValueError("segment outside the buffer")
    covered = np.zeros(N, dtype=np.int64)
    for s_ in range(len(se)):
        covered[ss[s_]:ss[s_] + sc[s_]] += 1
    if np.any(covered > 1):
        raise ValueError("segments overlap")
    want = None
    if positions is not None:
        want = np.zeros(N, dtype=bool)
        want[np.asarray(positions, dtype=np.int64)] = True
    out = np.zeros((N, d), dtype=np.float64)
    for s_ in range(len(se)):
        rows = np.arange(ss[s_], ss[s_] + sc[s_])
        if want is not None:
            rows = rows[want[rows]]
        if rows.size == 0:
            continue
        e = se[s_]
        a = widen(rb[rows])
        u = a @ widen(w1[e])
        v = a @ widen(w3[e])
        with np.errstate(over="ignore"):
            h = u / (1.0 + np.exp(-u)) * v
        out[rows] = h @ widen(w2[e])
    return out


def exchange_to(dispatched, placement, dest: int):
    """What GPU `dest` holds after the first all-to-all (Section 2.2): the
    dest-buckets of every source GPU's send buffer, source after source.

    dispatched: one dispatch() result per source GPU, in source order, all with
    the same expert -> GPU map.  Returns a dict: recv_buf [N_recv,d]; seg_expert,
    seg_counts, seg_start, seg_source (one segment per (source, expert on
    dest) in source-major, expert-ascending order, empty segments included);
    src_offset [G+1] = where each source's rows start in recv_buf.
    """
    pl = np.asarray(placement).astype(np.int64)
    experts = [e for e in range(len(pl)) if pl[e] == dest]
    bufs, seg_e, seg_c, seg_s, seg_src, src_off = [], [], [], [], [], [0]
    pos = 0
    for src, dsp in enumerate(dispatched):
        lo = int(dsp["gpu_offsets"][dest]); n = int(dsp["gpu_counts"][dest])
        bufs.append(np.asarray(dsp["send_buf"])[lo:lo + n])
        for e in experts:                              # the source sorted its dest-bucket by expert
            c = int(dsp["expert_counts"][e])
            seg_e.append(e); seg_c.append(c); seg_s.append(pos); seg_src.append(src)
            pos += c
        if pos - src_off[-1] != n:
            raise ValueError("a source's bucket for dest does not add up to its experts' counts")
        src_off.append(pos)
    recv = np.concatenate(bufs, axis=0) if bufs else np.zeros((0, 0))
    return dict(recv_buf=recv, seg_expert=np.array(seg_e, dtype=np.int32), seg_counts=np.array(seg_c, dtype=np.int32),
                seg_start=np.array(seg_s, dtype=np.int32), seg_source=np.array(seg_src, dtype=np.int32),
                src_offset=np.array(src_off, dtype=np.int64))


# --------------------------------------------------------------------------
# a4  gate-weighted combine
# --------------------------------------------------------------------------
def combine(ffn_out, inv_perm, topk_idx, topk_w, placement, local_gpu: int):
    """Un-permute and gate-weight the expert outputs (the step after the second
    all-to-all of Fig. 2b):

        y[t] = sum over j = 0..k-1 with placement[topk_idx[t,j]] == local_gpu
               of  topk_w[t,j] * ffn_out[inv_perm[t*k + j]]

    j ascending.  Routes whose expert is elsewhere contribute nothing (their
    results would come back over the return all-to-all, which is never run);
    tokens without a local route give zeros.  local_gpu = -1: no mask.
    Returns float64 [T,d].
    """
    o = widen(ffn_out)
    idx = np.asarray(topk_idx).astype(np.int64)
    T, k = idx.shape
    w = widen(topk_w)
    ip = np.asarray(inv_perm).astype(np.int64)
    pl = np.asarray(placement).astype(np.int64)
    y = np.zeros((T, o.shape[1]), dtype=np.float64)
    for t in range(T):
        for j in range(k):
            if local_gpu >= 0 and pl[idx[t, j]] != local_gpu:
                continue
            y[t] += w[t, j] * o[ip[t * k + j]]
    return y


# --------------------------------------------------------------------------
# a5  layer-l -> layer-(l+1) transition counts
# --------------------------------------------------------------------------
def transition_counts(idx_l, idx_l1, E_l: int, E_l1: int, R=None, top1_only: bool = False):
    """Routing history table between neighbouring layers (Section 2.4,
    Section 3.1 "Token Routing Profile", ILP 2 input R_{e1,e2,l}):

        R[e1][e2] += #{(t, j1, j2) : idx_l[t,j1] == e1 and idx_l1[t,j2] == e2}

    e1 is an expert of layer l, e2 an expert of layer l+1; with top-k routing
    every one of the k_l * k_{l+1} expert pairs of a token is counted.  R is
    int64 and is accumulated in place when given (profiling runs over many
    batches).  top1_only counts one pair per token instead, its top-1 expert
    in either layer (slot 0): the table of a top-1 reading of "tokens routed
    between experts e1 and e2".
    """
    a = np.asarray(idx_l)
    b = np.asarray(idx_l1)
    if a.ndim != 2 or b.ndim != 2 or a.shape[0] != b.shape[0]:
        raise ValueError("idx_l [T,k_l] and idx_l1 [T,k_l1] must share T")
    if top1_only:
        a, b = a[:, :1], b[:, :1]
    a = _check_index_array("idx_l", a, 0, E_l)
    b = _check_index_array("idx_l1", b, 0, E_l1)
    if R is None:
        R = np.zeros((E_l, E_l1), dtype=np.int64)
    elif R.shape != (E_l, E_l1) or R.dtype != np.int64:
        raise ValueError("R must be int64 [E_l,E_l1]")
    T = a.shape[0]
    for t in range(T):
        for e1 in a[t]:
            for e2 in b[t]:
                R[e1, e2] += 1
    return R


# --------------------------------------------------------------------------
# placement evaluators (inputs/objectives of the ILPs; the solve is not here)
# --------------------------------------------------------------------------
def cluster_loads(P_l, placement, G: int):
    """Eq. 2 for one layer: T_{c,l} = sum_e P_{e,l} * x_{c,e,l}, with the
    cluster of expert e given as placement[e] (x_{c,e,l} = [placement[e]==c]).
    The summation over t printed in Eq. 2 is not in Eq. 6 and is ignored."""
    P_l = np.asarray(P_l).astype(np.int64)
    pl = _check_index_array("placement", placement, 0, G)
    T_c = np.zeros(G, dtype=np.int64)
    for e in range(P_l.shape[0]):
        T_c[pl[e]] += P_l[e]
    return T_c


def load_imbalance(P_l, placement, G: int) -> float:
    """One layer's term of Eq. 1: sum_c |T_{c,l} - mean_l| with the mean of
    Eq. 3, mean_l = (1/G) sum_e P_{e,l}."""
    T_c = cluster_loads(P_l, placement, G).astype(np.float64)
    mean = float(np.asarray(P_l, dtype=np.float64).sum()) / G
    return float(np.abs(T_c - mean).sum())


def cluster_traffic(R_l, placement_l, placement_l1, G: int):
    """Eq. 9: C_{c1,c2,l} = sum_{e1,e2} R_{e1,e2,l} x_{c1,e1,l} x_{c2,e2,l+1}
    (the second factor belongs to layer l+1, as the definition of C says)."""
    R_l = np.asarray(R_l).astype(np.int64)
    pa = _check_index_array("placement_l", placement_l, 0, G)
    pb = _check_index_array("placement_l1", placement_l1, 0, G)
    C = np.zeros((G, G), dtype=np.int64)
    for e1 in range(R_l.shape[0]):
        for e2 in range(R_l.shape[1]):
            C[pa[e1], pb[e2]] += R_l[e1, e2]
    return C


def max_pair_cost(C_l, B) -> float:
    """One layer's term of Eq. 8 with clusters already mapped to GPUs
    (y = identity): max over GPU pairs (g1,g2) of C_{g1,g2,l} / B_{g1,g2}."""
    C = np.asarray(C_l, dtype=np.float64)
    B = np.asarray(B, dtype=np.float64)
    return float((C / B).max())


# --------------------------------------------------------------------------
# the whole layer, for convenience in tests
# --------------------------------------------------------------------------
def moe_layer(x, logits, k, w1, w3, w2, placement, G, local_gpu, positions=None):
    """gate -> dispatch -> expert FFN -> combine, all in fp64.  Returns a dict
    with every intermediate."""
    idx, w = topk_gate(logits, k)
    dsp = dispatch(x, idx, placement, G)
    o = expert_ffn_grouped(dsp["send_buf"], w1, w3, w2, dsp["expert_counts"],
                           dsp["expert_start"], placement, local_gpu, positions)
    y = combine(o, dsp["inv_perm"], idx, w, placement, local_gpu)
    res = dict(dsp)
    res.update(topk_idx=idx, topk_w=w, ffn_out=o, y=y)
    return res
