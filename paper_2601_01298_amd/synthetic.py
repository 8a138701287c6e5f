"""Seeded synthetic workloads for the Topological Synapse hot path.

The paper (Sec. 5.2) measures on the live KV cache of a chat model; no dataset
or benchmark suite is involved, and no weights are available here.  These
generators stand in for that cache: per KV head a cloud of L keys (and L values)
in R^d with cluster structure, drift, outliers or heavy tails, as listed per
configuration below, plus N agent queries.

This module serves both the CPU oracle's tests and the GPU path.  It holds NO
arithmetic of the method itself (no kernel, no score, no softmax): only random
draws, the rounding of the draws to the storage dtype, and the bandwidth recipe
sigma^2 = tr(Cov)/16, which is an INPUT to the method.

Determinism: every (seed, config, head, tensor) has its own Philox stream, so a
single head can be regenerated alone.  Values are drawn in float32/float64 on
the host and rounded ONCE (round-to-nearest-even) to the configuration's dtype;
arrays are returned as float32 holding exactly representable values, so the
oracle (widening to float64) and the GPU (narrowing to bf16) see the same bits.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass

import numpy as np

BASE_SEED = 20260101
TENSOR_K, TENSOR_V, TENSOR_Q, TENSOR_AUX = 0, 1, 2, 3


@dataclass(frozen=True)
class Workload:
    cfg: int        # 1..5, order of the configuration list
    name: str
    H: int          # KV heads handed to the library (layers x heads, flattened)
    Hq: int         # query heads
    d: int
    L: int
    k: int          # round(0.02 * L)
    N: int          # agents
    dtype: str      # "f32" | "bf16"
    layers: int = 1
    alpha: float = 0.5


WORKLOADS = {
    1: Workload(1, "tiny", H=1, Hq=1, d=64, L=512, k=10, N=4, dtype="f32"),
    2: Workload(2, "single_layer", H=16, Hq=16, d=64, L=4096, k=82, N=100, dtype="bf16"),
    3: Workload(3, "headline", H=24 * 16, Hq=24 * 16, d=64, L=32768, k=655, N=100, dtype="bf16", layers=24),
    4: Workload(4, "agent_scale_out", H=32, Hq=32, d=128, L=8192, k=164, N=1000, dtype="bf16"),
    5: Workload(5, "long_context_gqa", H=8, Hq=32, d=128, L=131072, k=2621, N=256, dtype="bf16"),
}


def _rng(seed: int, cfg: int, head: int, tensor: int) -> np.random.Generator:
    key = [np.uint64(seed), np.uint64((cfg << 40) | (head << 8) | tensor)]
    return np.random.Generator(np.random.Philox(key=key))


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """float32 -> nearest bf16 value (ties to even), returned as float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) & np.uint32(0xFFFF0000)).view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """Upper 16 bits of float32 values that already lie on the bf16 grid."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return (x.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def _store(x: np.ndarray, dtype: str) -> np.ndarray:
    x32 = np.ascontiguousarray(x, dtype=np.float32)
    return round_to_bf16(x32) if dtype == "bf16" else x32


def _mixture(rng, L, d, ncomp, comp_sigma=0.5, centre_sigma=2.0):
    centres = centre_sigma * rng.standard_normal((ncomp, d))
    assign = rng.integers(0, ncomp, size=L)
    x = centres[assign]
    x += comp_sigma * rng.standard_normal((L, d), dtype=np.float32)
    return x


def cloud(w: Workload, head: int, tensor: int, seed: int = BASE_SEED) -> np.ndarray:
    """[L,d] float32 keys (tensor=TENSOR_K) or values (TENSOR_V) of one head."""
    rng = _rng(seed, w.cfg, head, tensor)
    L, d = w.L, w.d
    if w.cfg == 1:
        x = _mixture(rng, L, d, 8)
    elif w.cfg == 2:
        x = _mixture(rng, L, d, 32)
        x *= rng.uniform(0.5, 2.0, size=d)
    elif w.cfg == 3:
        x = _mixture(rng, L, d, 64)
        steps = rng.standard_normal((L, d), dtype=np.float32)
        x += 0.02 * np.cumsum(steps, axis=0, dtype=np.float64)
    elif w.cfg == 4:
        x = _mixture(rng, L, d, 128)
        outlier = rng.random(L) < 0.01
        x[outlier] = rng.uniform(-8.0, 8.0, size=(int(outlier.sum()), d))
    elif w.cfg == 5:
        lam = 1.0 / np.arange(1, d + 1, dtype=np.float64)
        lam *= d / lam.sum()
        U, _ = np.linalg.qr(rng.standard_normal((d, d)))
        tau = rng.standard_t(3.0, size=(L, d))
        x = (tau * np.sqrt(lam)) @ U.T
    else:
        raise ValueError(f"unknown configuration {w.cfg}")
    return _store(x, w.dtype)


def queries(w: Workload, seed: int = BASE_SEED) -> np.ndarray:
    """[N,Hq,d] float32 agent queries ~ N(0, I), rounded to the workload dtype."""
    rng = _rng(seed, w.cfg, 0, TENSOR_Q)
    return _store(rng.standard_normal((w.N, w.Hq, w.d), dtype=np.float32), w.dtype)


def bandwidth(K: np.ndarray) -> np.float32:
    """Per-head bandwidth recipe: sigma^2 = tr(Cov)/16 with the biased
    covariance of the head's keys, in float64; returned as the float32 that is
    handed to both the oracle and the GPU."""
    K64 = np.asarray(K, dtype=np.float64)
    var = K64.var(axis=0)          # biased
    return np.float32(np.sqrt(var.sum() / 16.0))


def small_variant(w: Workload, **kw) -> Workload:
    """Same recipe at another size (tests use reduced L / H / N)."""
    from dataclasses import replace
    return replace(w, **kw)


def clouds(w: Workload, tensor: int, heads=None, seeds=None, threads: int = 8, out=None, bits: bool = False):
    """Stack several heads: [len(heads), L, d] float32, or uint16 bf16 bit
    patterns when bits=True.  `seeds` maps head -> seed (default BASE_SEED)."""
    heads = list(range(w.H)) if heads is None else list(heads)
    seeds = seeds or {}
    if out is None:
        out = np.empty((len(heads), w.L, w.d), dtype=np.uint16 if bits else np.float32)

    def one(slot_head):
        slot, h = slot_head
        x = cloud(w, h, tensor, seeds.get(h, BASE_SEED))
        out[slot] = bf16_bits(x) if bits else x

    with ThreadPoolExecutor(max_workers=max(1, threads)) as ex:
        list(ex.map(one, enumerate(heads)))
    return out


# ---- inputs of the steps next to the hot path (attention mass, gate, injection) ---------------
def main_query(w: Workload, seed: int = BASE_SEED) -> np.ndarray:
    """[Hq,d] float32: the main agent's current query token, one row per query head ~ N(0, I)."""
    rng = _rng(seed, w.cfg, 1, TENSOR_Q)
    return _store(rng.standard_normal((w.Hq, w.d), dtype=np.float32), w.dtype)


def hidden_states(N: int, dm: int, dtype: str, seed: int = BASE_SEED):
    """(h_main [dm], T [N,dm]) float32: final-layer hidden states of the main agent and of N side
    thoughts.  Thought n is a mix a_n * h + noise with a_n spread over [-0.5, 3], so the cosine
    scores cover both sides of any threshold; thought 0 is all zeros (a degenerate case)."""
    rng = _rng(seed, 0, 2, TENSOR_AUX)
    h = rng.standard_normal(dm)
    a = rng.uniform(-0.5, 3.0, size=(N, 1))
    T = a * h + rng.standard_normal((N, dm))
    T[0] = 0.0
    return _store(h, dtype), _store(T, dtype)


def thought_rows(w: Workload, m: int, seed: int = BASE_SEED):
    """(Knew, Vnew [H,m,d], pos [m] int32): un-rotated key/value rows of an injected thought and
    the virtual positions given to them (spread from small indices to far beyond the context)."""
    rng = _rng(seed, w.cfg, 3, TENSOR_AUX)
    Kn = _store(2.0 * rng.standard_normal((w.H, m, w.d), dtype=np.float32), w.dtype)
    Vn = _store(2.0 * rng.standard_normal((w.H, m, w.d), dtype=np.float32), w.dtype)
    pos = np.sort(rng.integers(0, 4 * max(w.L, 1024), size=m)).astype(np.int32)
    pos[0] = 0
    if m > 1:
        pos[-1] = 2_000_000_000
    return Kn, Vn, pos
