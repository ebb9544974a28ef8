"""Seeded synthetic inputs for the MoE-layer hot path.

This module only *makes inputs*: activations, router logits, expert weights,
expert->GPU maps.  It contains none of the layer's arithmetic (no top-k, no
sort, no FFN, no combine, no counting) and is the one module the HIP tests, the
CPU oracle tests and the benchmark all share, so that both sides of a parity
check consume identical bits.

The paper measured Mixtral-8x7B on public language-modelling corpora
(Section 4.1); neither the weights nor the corpora are used here.  What is kept
is their structure: 8 experts, top-2, four expert-parallel ranks with two
experts each by default (Section 1, Section 4.2), a strong per-layer load skew
(Section 2.3: single GPUs seeing 64-69 % of the tokens) and a strong
layer-to-layer routing affinity (Section 2.4).  A Zipf log-bias on the router
reproduces the skew; a logit bonus on seeded "successor" experts reproduces the
affinity.

Conventions
-----------
* N(0, sigma): sigma is the standard deviation.
* Random streams: numpy Philox, key = (seed, tensor_id, chunk); large tensors
  are filled chunk by chunk on a thread pool, so the values do not depend on
  the number of threads.
* bf16 tensors are uint16 bit patterns (round-to-nearest-even of the fp32
  draw); fp32 tensors are float32.
* Router logits are computed once, on the host, in fp64 and rounded to fp32:
  logits = fp32(x . W_g + bias [+ bonus]).  Both sides of a parity check receive
  that same fp32 array.
"""
from __future__ import annotations

import math
import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field

import numpy as np

# tensor ids inside one (config, layer) seed space
TID_X, TID_WG, TID_W1, TID_W3, TID_W2, TID_PLACEMENT, TID_SUCC, TID_RANKPERM = range(8)

_CHUNK = 1 << 22  # elements per Philox stream


def n_threads() -> int:
    try:
        avail = len(os.sched_getaffinity(0))
    except AttributeError:  # pragma: no cover
        avail = os.cpu_count() or 1
    env = os.environ.get("OMP_NUM_THREADS")
    if env and env.isdigit():
        avail = min(avail, int(env))
    return max(1, min(avail, 16))


# --------------------------------------------------------------------------
# bf16 bit helpers (input quantisation only)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even); returns uint16 bit patterns.
    Inputs here are finite, so no NaN handling is needed."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------
# seeded normal tensors
# --------------------------------------------------------------------------
def _fill_chunk(args):
    seed, tid, c, n, sigma, as_bf16 = args
    rng = np.random.Generator(np.random.Philox(key=[(seed << 8) + tid, c]))
    v = rng.standard_normal(n, dtype=np.float32)
    if sigma != 1.0:
        v *= np.float32(sigma)
    return f32_to_bf16_bits(v) if as_bf16 else v


def normal(seed: int, tid: int, shape, sigma: float, dtype: str) -> np.ndarray:
    """N(0, sigma) tensor of the given shape; dtype 'f32' -> float32 array,
    'bf16' -> uint16 bit patterns."""
    assert dtype in ("f32", "bf16")
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16 if dtype == "bf16" else np.float32)
    jobs = [(seed, tid, c, min(_CHUNK, n - c * _CHUNK), float(sigma), dtype == "bf16")
            for c in range((n + _CHUNK - 1) // _CHUNK)]
    if len(jobs) <= 1:
        for j in jobs:
            out[: j[3]] = _fill_chunk(j)
    else:
        with ThreadPoolExecutor(n_threads()) as ex:
            for j, v in zip(jobs, ex.map(_fill_chunk, jobs)):
                out[j[2] * _CHUNK: j[2] * _CHUNK + j[3]] = v
    return out.reshape(shape)


def to_f64(a: np.ndarray) -> np.ndarray:
    if a.dtype == np.uint16:
        return bf16_bits_to_f32(a).astype(np.float64)
    return a.astype(np.float64)


# --------------------------------------------------------------------------
# router bias, logits, successor bonus
# --------------------------------------------------------------------------
def zipf_log_bias(E: int, s: float, rank_of_expert=None) -> np.ndarray:
    """b_e = -s ln(rank_e) - ln(sum_i i^-s): the log of Zipf(s) weights.
    rank_of_expert[e] in 1..E; default rank_e = e + 1 (hot experts have low
    ids, so the contiguous map puts the hot pair on GPU 0)."""
    rank = np.arange(1, E + 1, dtype=np.float64) if rank_of_expert is None \
        else np.asarray(rank_of_expert, dtype=np.float64)
    z = sum(i ** (-s) for i in range(1, E + 1))
    return -s * np.log(rank) - math.log(z)


def synthetic_logits(x, w_g, bias, bonus=None) -> np.ndarray:
    """The recipe of the synthetic logits handed, bit for bit, to both the GPU
    path and the oracle: fp32( fp64(x) @ fp64(w_g) + bias (+ bonus) ), x [T,d],
    w_g [d,E].  An input generator, not the library's router: that is
    moe_router_gate, and its checker is the oracle's router_logits; neither is
    tested against this function."""
    z = to_f64(x) @ to_f64(w_g) + np.asarray(bias, dtype=np.float64)[None, :]
    if bonus is not None:
        z = z + bonus
    return z.astype(np.float32)


def successor_bonus(prev_top1: np.ndarray, succ: np.ndarray, E: int, amount: float) -> np.ndarray:
    """[T,E] array holding `amount` at the successor experts succ[prev_top1[t]]
    of each token and 0 elsewhere.  prev_top1 is supplied by the caller (it is
    an output of the layer before, not something this module computes)."""
    T = prev_top1.shape[0]
    b = np.zeros((T, E), dtype=np.float64)
    rows = np.repeat(np.arange(T), succ.shape[1])
    b[rows, succ[prev_top1].reshape(-1)] = amount
    return b


def successors(seed: int, E: int, n_succ: int = 2) -> np.ndarray:
    """succ[e] = n_succ distinct seeded experts of the next layer."""
    rng = np.random.Generator(np.random.Philox(key=[(seed << 8) + TID_SUCC, 0]))
    return np.stack([rng.permutation(E)[:n_succ] for _ in range(E)]).astype(np.int32)


def rank_permutation(seed: int, E: int) -> np.ndarray:
    rng = np.random.Generator(np.random.Philox(key=[(seed << 8) + TID_RANKPERM, 0]))
    return (rng.permutation(E) + 1).astype(np.int64)


# --------------------------------------------------------------------------
# expert -> GPU maps
# --------------------------------------------------------------------------
def placement_contiguous(E: int, G: int) -> np.ndarray:
    """The default map of Section 1 / Section 4.2: GPU g owns experts
    [g*E/G, (g+1)*E/G)."""
    assert E % G == 0
    return (np.arange(E) // (E // G)).astype(np.int32)


def placement_balanced_random(E: int, G: int, seed: int) -> np.ndarray:
    """Shuffle the experts, cut into G equal groups."""
    assert E % G == 0
    rng = np.random.Generator(np.random.Philox(key=[(seed << 8) + TID_PLACEMENT, 0]))
    order = rng.permutation(E)
    pl = np.empty(E, dtype=np.int32)
    pl[order] = np.arange(E) // (E // G)
    return pl


def placement_from_sizes(sizes, seed: int | None = None) -> np.ndarray:
    """Uneven map: GPU g owns sizes[g] experts (Section 3.1 / Section 4.1: the
    number of experts per GPU may differ by layer), e.g. (1,1,2,4).  With a
    seed the experts are shuffled first, otherwise assigned in order."""
    E = int(sum(sizes))
    pl = np.repeat(np.arange(len(sizes)), sizes).astype(np.int32)
    if seed is not None:
        rng = np.random.Generator(np.random.Philox(key=[(seed << 8) + TID_PLACEMENT, 1]))
        pl = pl[rng.permutation(E)]
    return pl


# --------------------------------------------------------------------------
# configurations
# --------------------------------------------------------------------------
@dataclass
class MoEConfig:
    name: str
    cfg_id: int
    dtype: str          # 'f32' or 'bf16'
    T: int
    d: int
    f: int
    E: int
    k: int
    G: int
    local_gpu: int      # -1 = all experts resident
    wg_sigma: float
    zipf_s: float
    layers: int = 1
    placement_kind: str = "contiguous"   # contiguous | balanced_random
    bonus: float = 0.0
    permute_ranks: bool = False
    extra: dict = field(default_factory=dict)

    def seed(self, layer: int = 0) -> int:
        return 1000 * self.cfg_id + 100 * layer

    def with_(self, **kw) -> "MoEConfig":
        d = dict(self.__dict__)
        d.update(kw)
        return MoEConfig(**d)


def config(name: str) -> MoEConfig:
    """Named presets; shapes and distributions as listed for the five
    benchmark configurations of this repository."""
    n = name.lower()
    if n == "c1":      # tiny fp32 layer, oracle runs in full
        return MoEConfig("c1", 1, "f32", 256, 128, 256, 8, 2, 4, 0, 0.02, 1.2)
    if n == "c1b":     # same, router noise 1/sqrt(d) so every bucket is populated
        return MoEConfig("c1b", 6, "f32", 256, 128, 256, 8, 2, 4, 0, 1 / math.sqrt(128), 1.2)
    if n == "c2":      # Mixtral-8x7B-shaped prefill, all experts resident
        return MoEConfig("c2", 2, "bf16", 4096, 4096, 14336, 8, 2, 1, -1, 1 / math.sqrt(4096), 1.0)
    if n == "c2b":     # same batch, EP=4 contiguous, this GPU owns experts 0,1
        return MoEConfig("c2b", 2, "bf16", 4096, 4096, 14336, 8, 2, 4, 0, 1 / math.sqrt(4096), 1.0)
    if n == "c3":      # decode
        return MoEConfig("c3", 3, "bf16", 64, 4096, 14336, 8, 2, 1, -1, 1 / math.sqrt(4096), 1.0)
    if n == "c4":      # fine-grained many-expert layer
        return MoEConfig("c4", 4, "bf16", 8192, 2048, 1408, 64, 6, 8, 0, 1 / math.sqrt(2048), 1.2,
                         placement_kind="balanced_random")
    if n == "c5":      # four chained Mixtral-shaped layers with routing affinity
        return MoEConfig("c5", 5, "bf16", 16384, 4096, 14336, 8, 2, 1, -1, 1 / math.sqrt(4096), 1.0,
                         layers=4, bonus=3.0, permute_ranks=True)
    raise KeyError(name)


def make_placement(cfg: MoEConfig, layer: int = 0) -> np.ndarray:
    if cfg.placement_kind == "balanced_random":
        return placement_balanced_random(cfg.E, cfg.G, cfg.seed(layer))
    return placement_contiguous(cfg.E, cfg.G)


def make_x(cfg: MoEConfig) -> np.ndarray:
    return normal(cfg.seed(0), TID_X, (cfg.T, cfg.d), 1.0, cfg.dtype)


def make_router(cfg: MoEConfig, layer: int = 0):
    """(W_g [d,E], bias [E]) of one layer."""
    w_g = normal(cfg.seed(layer), TID_WG, (cfg.d, cfg.E), cfg.wg_sigma, cfg.dtype)
    ranks = rank_permutation(cfg.seed(layer), cfg.E) if cfg.permute_ranks else None
    return w_g, zipf_log_bias(cfg.E, cfg.zipf_s, ranks)


def make_expert_weights(cfg: MoEConfig, layer: int = 0, experts=None):
    """W1, W3 [E,d,f] ~ N(0, 1/sqrt(d)); W2 [E,f,d] ~ N(0, 1/sqrt(f))."""
    s = cfg.seed(layer)
    w1 = normal(s, TID_W1, (cfg.E, cfg.d, cfg.f), 1 / math.sqrt(cfg.d), cfg.dtype)
    w3 = normal(s, TID_W3, (cfg.E, cfg.d, cfg.f), 1 / math.sqrt(cfg.d), cfg.dtype)
    w2 = normal(s, TID_W2, (cfg.E, cfg.f, cfg.d), 1 / math.sqrt(cfg.f), cfg.dtype)
    return w1, w3, w2


def make_logits(cfg: MoEConfig, x: np.ndarray, layer: int = 0, prev_top1=None) -> np.ndarray:
    """Router logits of one layer from the layer-0 activations x.  For layers
    after the first of a chained configuration, prev_top1 (the previous layer's
    top-1 expert per token, supplied by the caller) selects the successor
    experts that receive the affinity bonus."""
    w_g, bias = make_router(cfg, layer)
    bonus = None
    if layer > 0 and cfg.bonus != 0.0:
        assert prev_top1 is not None
        succ = successors(cfg.seed(layer - 1), cfg.E)
        bonus = successor_bonus(np.asarray(prev_top1), succ, cfg.E, cfg.bonus)
    return synthetic_logits(x, w_g, bias, bonus)


def random_topk_idx(seed: int, T: int, E: int, k: int) -> np.ndarray:
    """[T,k] int32 with k distinct uniformly drawn experts per token (the first
    k entries of a random permutation of the experts), for tests of dispatch,
    combine and transition counts in isolation from the gate."""
    rng = np.random.Generator(np.random.Philox(key=[(seed << 8) + 31, 0]))
    base = np.tile(np.arange(E, dtype=np.int32), (T, 1))
    return np.ascontiguousarray(rng.permuted(base, axis=1)[:, :k])
