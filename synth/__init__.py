"""Seeded synthetic inputs for the certified sub-vocabulary LM-head path.

This module only manufactures inputs (weights, biases, planted cluster labels and
hidden states); it contains none of the method's arithmetic.  The CPU oracle and
the GPU path are both fed the arrays produced here.

The recipes stand in for the Llama-3 / Qwen2.5 / Gemma2 output layers and text
workloads the paper evaluates on (vocabulary sizes from its Table "Vocabulary
Sizes of Some Modern LLMs"); no real weights or datasets are used.

All arrays are deterministic functions of (seed, recipe): every chunk of rows has
its own numpy Generator seeded from (seed, stream id, chunk index), so the result
does not depend on how many threads generate it.
"""
from __future__ import annotations

import math
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace

import numpy as np

SEED = 42  # the seed the paper fixes for all of its runs (Section V, reproducibility setup)

_ROW_CHUNK = 2048

# stream ids: one per generated array
_S_CENTERS, _S_NOISE, _S_BIAS, _S_TOKPERM, _S_ZIPF, _S_HPICK, _S_HNOISE, _S_HISO, _S_HMIX = range(9)


@dataclass(frozen=True)
class Recipe:
    name: str
    V: int
    d: int
    C: int
    B: int
    steps: int
    k: int
    eps: float
    sizes: str = "equal"      # "equal" | "zipf"
    h_mode: str = "single"    # "single": one centre per h; "mix": 1..3 centres, Dirichlet(0.5) weights
    iso_frac: float = 0.0     # probability that an h is an isotropic direction
    center_scale: float = 4.0
    row_noise: float = 0.05
    bias_std: float = 0.1
    h_norm: float = 8.0
    zipf_s: float = 1.1
    zipf_min: int = 8

    @property
    def K_max_rows(self) -> int:
        return self.V // 4

    def scaled(self, **kw) -> "Recipe":
        return replace(self, **kw)


CONFIGS = {
    "c1": Recipe("c1", V=32000, d=1024, C=256, B=1, steps=64, k=10, eps=1e-3),
    "c2": Recipe("c2", V=128256, d=4096, C=1024, B=1, steps=512, k=50, eps=1e-3),
    "c3": Recipe("c3", V=151552, d=5120, C=2048, B=8, steps=256, k=50, eps=1e-4, sizes="zipf", h_mode="mix"),
    "c4": Recipe("c4", V=256000, d=4608, C=4096, B=32, steps=128, k=64, eps=1e-3),
    "c5": Recipe("c5", V=128256, d=8192, C=1024, B=64, steps=128, k=50, eps=1e-4, iso_frac=0.25),
}


def _rng(seed: int, stream: int, chunk: int = 0) -> np.random.Generator:
    return np.random.default_rng(np.random.SeedSequence([seed, stream, chunk]))


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even) and return the 16-bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns to float32 (exact)."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def cluster_sizes(r: Recipe, seed: int = SEED) -> np.ndarray:
    """Rows per planted cluster, int64[C], summing to V."""
    if r.sizes == "equal":
        base, rem = divmod(r.V, r.C)
        n = np.full(r.C, base, dtype=np.int64)
        n[:rem] += 1
        return n
    if r.sizes == "zipf":
        rank = np.arange(1, r.C + 1, dtype=np.float64)
        w = rank ** (-r.zipf_s)
        n = np.maximum(r.zipf_min, np.floor(r.V * w / w.sum())).astype(np.int64)
        diff = r.V - int(n.sum())
        if diff >= 0:
            n[0] += diff
        else:
            # floors plus the minimum overshoot V: take the excess from the largest clusters
            i = 0
            while diff < 0:
                take = min(-diff, int(n[i]) - r.zipf_min)
                n[i] -= take
                diff += take
                i += 1
        assert n.sum() == r.V and n.min() >= 1
        # ranks are handed to cluster ids by a seeded shuffle
        return n[_rng(seed, _S_ZIPF).permutation(r.C)]
    raise ValueError(r.sizes)


def make_head(r: Recipe, seed: int = SEED, threads: int = 8) -> dict:
    """Planted clustered LM head.

    Returns W_bits uint16[V,d] (bf16 patterns, ORIGINAL token order), b float32[V],
    labels int32[V] (planted cluster of each token), centers float32[C,d].
    """
    V, d, C = r.V, r.d, r.C
    centers = (_rng(seed, _S_CENTERS).standard_normal((C, d), dtype=np.float32)
               * np.float32(r.center_scale / math.sqrt(d)))
    n = cluster_sizes(r, seed)
    row_label = np.repeat(np.arange(C, dtype=np.int32), n)          # planted order: cluster-contiguous
    token_of_row = _rng(seed, _S_TOKPERM).permutation(V)            # planted row -> original token id
    labels = np.empty(V, dtype=np.int32)
    labels[token_of_row] = row_label
    b = _rng(seed, _S_BIAS).standard_normal(V, dtype=np.float32) * np.float32(r.bias_std)

    W_bits = np.empty((V, d), dtype=np.uint16)
    sigma = np.float32(r.row_noise / math.sqrt(d))

    def fill(ci: int) -> None:
        lo = ci * _ROW_CHUNK
        hi = min(V, lo + _ROW_CHUNK)
        x = _rng(seed, _S_NOISE, ci).standard_normal((hi - lo, d), dtype=np.float32)
        x *= sigma
        x += centers[row_label[lo:hi]]
        W_bits[token_of_row[lo:hi]] = f32_to_bf16_bits(x)

    nchunks = (V + _ROW_CHUNK - 1) // _ROW_CHUNK
    if threads > 1:
        with ThreadPoolExecutor(threads) as ex:
            list(ex.map(fill, range(nchunks)))
    else:
        for ci in range(nchunks):
            fill(ci)
    return {"W_bits": W_bits, "b": b, "labels": labels, "centers": centers, "sizes": n}


def make_hidden(r: Recipe, centers: np.ndarray, steps: int | None = None, seed: int = SEED) -> np.ndarray:
    """Hidden states, uint16[steps, B, d] bf16 patterns, each with norm h_norm before rounding."""
    steps = r.steps if steps is None else steps
    B, d, C = r.B, r.d, r.C
    n = steps * B
    chat = centers.astype(np.float64)
    chat /= np.linalg.norm(chat, axis=1, keepdims=True)
    g = _rng(seed, _S_HNOISE).standard_normal((n, d))
    g /= np.linalg.norm(g, axis=1, keepdims=True)
    pick = _rng(seed, _S_HPICK)
    if r.h_mode == "single":
        a = chat[pick.integers(0, C, size=n)]
    elif r.h_mode == "mix":
        mix = _rng(seed, _S_HMIX)
        a = np.empty((n, d))
        for i in range(n):
            m = min(int(pick.integers(1, 4)), C)          # at most as many distinct centres as there are
            ids = pick.choice(C, size=m, replace=False)
            w = mix.dirichlet(np.full(m, 0.5))
            v = (w[:, None] * chat[ids]).sum(0)
            a[i] = v / np.linalg.norm(v)
    else:
        raise ValueError(r.h_mode)
    v = 0.9 * a + 0.1 * g
    if r.iso_frac > 0:
        iso = _rng(seed, _S_HISO).random(n) < r.iso_frac
        v[iso] = g[iso]
    v *= r.h_norm / np.linalg.norm(v, axis=1, keepdims=True)
    return f32_to_bf16_bits(v.astype(np.float32)).reshape(steps, B, d)


def small_recipe(name: str = "tiny", **kw) -> Recipe:
    """A reduced recipe for fast tests; same generator, smaller shapes."""
    base = dict(V=2000, d=256, C=16, B=2, steps=4, k=5, eps=1e-3)
    base.update(kw)
    return Recipe(name, **base)
