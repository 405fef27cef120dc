"""Seeded synthetic inputs: model shapes, weight blobs, length mixes, token ids.

This module serves both the HIP path's callers and the CPU oracle's tests, so
it holds no arithmetic of the method itself: it only names the five workloads,
describes where each tensor lives in the canonical float32 weight blob, and
draws random numbers.

Stand-in note: the paper measures on GLUE samples replayed through a
production request trace (Section 4.1); neither is available offline, so the
workloads below imitate their shape only -- sentence lengths from ten to a few
hundred tokens, ids uniform over the vocabulary, weights N(0, 0.02).

Draw order for a workload with seed s: ``rng = numpy.random.default_rng(s)``;
lengths, then token ids, then the whole weight blob in blob order with one
``standard_normal`` call, after which LayerNorm scales are set to 1 and shifts
to 0 (unless ``ln_random``).
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Iterator, List, Tuple

import numpy as np


@dataclass(frozen=True)
class StudentShape:
    K: int          # students in the group, in training order
    layers: int
    hidden: int
    heads: int
    ffn: int
    vocab: int
    max_pos: int
    classes: int
    ln_eps: float = 1e-12
    dtype: str = "bf16"  # "fp32" or "bf16": arithmetic type of the HIP path


@dataclass(frozen=True)
class Workload:
    name: str
    shape: StudentShape
    batch: int
    lengths: Tuple  # ("uniform", lo, hi) | ("fixed", n) | ("lognormal", median, sigma, lo, hi)
    k_actives: Tuple[int, ...]
    seed: int = 0


_BASE = dict(layers=2, hidden=768, heads=12, ffn=3072, vocab=30522, max_pos=512)

WORKLOADS: Dict[int, Workload] = {
    1: Workload("c1_tiny_fp32", StudentShape(K=2, layers=2, hidden=128, heads=2, ffn=512, vocab=1000, max_pos=64,
                                             classes=2, dtype="fp32"), 4, ("uniform", 8, 32), (2, 1)),
    2: Workload("c2_base_b32", StudentShape(K=4, classes=2, **_BASE), 32, ("uniform", 16, 128), (1, 2, 4)),
    3: Workload("c3_latency_b1", StudentShape(K=8, classes=3, **_BASE), 1, ("fixed", 64), (8, 4, 2, 1)),
    4: Workload("c4_burst_b256", StudentShape(K=8, classes=2, **_BASE), 256, ("lognormal", 48.0, 0.6, 8, 256),
                (8, 4, 2)),
    5: Workload("c5_large_b64", StudentShape(K=6, layers=2, hidden=1024, heads=16, ffn=4096, vocab=30522, max_pos=512,
                                             classes=2), 64, ("uniform", 64, 512), (6,)),
}


# ---- blob geometry ----------------------------------------------------------

def _student_entries(s: StudentShape) -> List[Tuple[str, Tuple[int, ...]]]:
    H, F, C = s.hidden, s.ffn, s.classes
    e: List[Tuple[str, Tuple[int, ...]]] = [("tok_emb", (s.vocab, H)), ("pos_emb", (s.max_pos, H)),
                                            ("emb_ln_g", (H,)), ("emb_ln_b", (H,))]
    for l in range(s.layers):
        p = f"l{l}."
        e += [(p + "Wq", (H, H)), (p + "bq", (H,)), (p + "Wk", (H, H)), (p + "bk", (H,)), (p + "Wv", (H, H)),
              (p + "bv", (H,)), (p + "Wo", (H, H)), (p + "bo", (H,)), (p + "ln1_g", (H,)), (p + "ln1_b", (H,)),
              (p + "W1", (H, F)), (p + "b1", (F,)), (p + "W2", (F, H)), (p + "b2", (H,)), (p + "ln2_g", (H,)),
              (p + "ln2_b", (H,))]
    e += [("Wp", (H, H)), ("bp", (H,)), ("Wc", (H, C)), ("bc", (C,))]
    return e


def student_floats(s: StudentShape) -> int:
    return sum(int(np.prod(shape)) for _, shape in _student_entries(s))


def blob_floats(s: StudentShape) -> int:
    return s.K * student_floats(s)


def student_views(blob: np.ndarray, s: StudentShape, m: int) -> Dict[str, np.ndarray]:
    """Named, writable views of student m's tensors inside the blob ([in][out] matrices)."""
    assert blob.dtype == np.float32 and blob.size == blob_floats(s)
    off = m * student_floats(s)
    out = {}
    for name, shape in _student_entries(s):
        n = int(np.prod(shape))
        out[name] = blob[off:off + n].reshape(shape)
        off += n
    return out


def iter_views(blob: np.ndarray, s: StudentShape) -> Iterator[Tuple[int, Dict[str, np.ndarray]]]:
    for m in range(s.K):
        yield m, student_views(blob, s, m)


# ---- random draws -----------------------------------------------------------

def make_lengths(rng: np.random.Generator, batch: int, recipe: Tuple) -> np.ndarray:
    kind = recipe[0]
    if kind == "fixed":
        return np.full(batch, int(recipe[1]), dtype=np.int32)
    if kind == "uniform":
        return rng.integers(int(recipe[1]), int(recipe[2]) + 1, size=batch).astype(np.int32)
    if kind == "lognormal":
        _, median, sigma, lo, hi = recipe
        raw = np.exp(rng.normal(np.log(median), sigma, size=batch))
        return np.clip(np.rint(raw), lo, hi).astype(np.int32)
    raise ValueError(kind)


def make_arrivals(rng: np.random.Generator, n: int, quiet_per_s: float, burst_per_s: float, quiet_s: float,
                  burst_s: float) -> np.ndarray:
    """Arrival times (integer microseconds, non-decreasing) of n requests: a Poisson process whose rate alternates
    between quiet stretches and bursts (stand-in for the production request trace the paper replays, which is not
    available offline: steady traffic with bursts an order of magnitude denser)."""
    out = np.empty(n, dtype=np.float64)
    t, i, phase_end, burst = 0.0, 0, quiet_s, False
    while i < n:
        rate = burst_per_s if burst else quiet_per_s
        m = min(n - i, max(16, int(rate * (phase_end - t) * 1.2) + 16))
        ts = t + np.cumsum(rng.exponential(1.0 / rate, size=m))
        inside = int(np.searchsorted(ts, phase_end, side="right"))
        out[i:i + inside] = ts[:inside]
        i += inside
        if inside < m or (inside and ts[inside - 1] >= phase_end):
            t, burst = phase_end, not burst
            phase_end = t + (burst_s if burst else quiet_s)
        elif inside:
            t = ts[inside - 1]
    return np.floor(out * 1e6).astype(np.int64)


def make_ids(rng: np.random.Generator, total: int, vocab: int) -> np.ndarray:
    return rng.integers(0, vocab, size=total).astype(np.int32)


def make_weights(rng: np.random.Generator, s: StudentShape, std: float = 0.02, ln_random: bool = False,
                 qk_std: float | None = None) -> np.ndarray:
    """The canonical blob: everything N(0, std) including biases; LayerNorm scale 1, shift 0.

    ``ln_random`` draws scales 1 + 0.1 N(0,1) and shifts 0.1 N(0,1) instead, and
    ``qk_std`` redraws Wq and Wk at that spread; both exist for tests only, so
    that a wrong scale, mask or shift cannot hide behind near-uniform attention.
    """
    blob = rng.standard_normal(blob_floats(s), dtype=np.float32)
    blob *= np.float32(std)
    for _, v in iter_views(blob, s):
        for name, arr in v.items():
            if name.endswith("_g"):
                arr[...] = 1.0 + (0.1 * rng.standard_normal(arr.shape, dtype=np.float32) if ln_random else 0.0)
            elif name.endswith("ln_b") or name.endswith("ln1_b") or name.endswith("ln2_b"):
                arr[...] = 0.1 * rng.standard_normal(arr.shape, dtype=np.float32) if ln_random else 0.0
            elif qk_std is not None and name.endswith(("Wq", "Wk")):
                arr[...] = qk_std * rng.standard_normal(arr.shape, dtype=np.float32)
    return blob


@dataclass
class Batch:
    lengths: np.ndarray   # int32 [B]
    ids: np.ndarray       # int32 [T], packed: sequence b occupies [sum(lengths[:b]), sum(lengths[:b+1]))


def make_workload(w: Workload, with_weights: bool = True, **weight_kw):
    """(Batch, blob) for a named workload, drawn in the documented order."""
    rng = np.random.default_rng(w.seed)
    lengths = make_lengths(rng, w.batch, w.lengths)
    ids = make_ids(rng, int(lengths.sum()), w.shape.vocab)
    blob = make_weights(rng, w.shape, **weight_kw) if with_weights else None
    return Batch(lengths, ids), blob


def small_variant(w: Workload, **shape_overrides) -> Workload:
    """Same recipe with some shape fields replaced (e.g. a smaller vocabulary for quick tests)."""
    return replace(w, shape=replace(w.shape, **shape_overrides))
