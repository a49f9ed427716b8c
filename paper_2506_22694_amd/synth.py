"""Seeded synthetic inputs for the trimmed-LM-head path.

This module only *draws inputs* (token-id streams, head matrices, hidden rows)
and converts between storage formats.  It holds none of the method's
arithmetic (no counting, selection, projection or softmax), so both the HIP
path's tests and the CPU oracle's tests may use it.

The workloads stand in for the paper's: Llama-3 LM heads (shapes from the head
sizes of Tables 1 and 3) and calibration corpora whose token frequencies are
heavy-tailed (Fig. 1 and the introduction's description of it).  A bounded
Zipf law over ranks 1..V models that tail; a random rank->id permutation
scatters the hot ids over the vocabulary as a real tokenizer does.
"""
from __future__ import annotations

import dataclasses

import numpy as np


# --------------------------------------------------------------------------
# storage-format helpers (bf16 <-> fp32 bit patterns); no method arithmetic
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even), returned as uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to the fp32 values they denote (exact)."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------
# generators
# --------------------------------------------------------------------------
def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


def zipf_cdf(V: int, s: float) -> np.ndarray:
    """CDF of the bounded Zipf pmf p_r ~ r^-s over ranks r = 1..V (fp64)."""
    p = np.arange(1, V + 1, dtype=np.float64) ** (-s)
    c = np.cumsum(p)
    c /= c[-1]
    c[-1] = 1.0
    return c


def rank_permutation(V: int, seed: int, permute: bool) -> np.ndarray:
    """rank (0-based) -> token id.  Identity when permute is False."""
    if not permute:
        return np.arange(V, dtype=np.int64)
    return _rng(seed).permutation(V).astype(np.int64)


def zipf_ids(N: int, V: int, s: float, seed: int, permute: bool,
             dtype=np.int32, chunk: int = 1 << 24) -> np.ndarray:
    """N token ids: rank ~ bounded Zipf(s) by inverse CDF, then rank -> id.

    seed+1 drives the draws, seed+2 the permutation (seed+0 / seed+3 are the
    head and the hidden rows).
    """
    cdf = zipf_cdf(V, s)
    perm = rank_permutation(V, seed + 2, permute)
    g = _rng(seed + 1)
    out = np.empty(N, dtype=dtype)
    for lo in range(0, N, chunk):
        hi = min(N, lo + chunk)
        u = g.random(hi - lo)
        r = np.searchsorted(cdf, u, side="left")
        np.minimum(r, V - 1, out=r)
        out[lo:hi] = perm[r].astype(dtype, copy=False)
    return out


def head_weights(V: int, d: int, seed: int, dtype: str, std: float = 0.02,
                 chunk_rows: int = 16384) -> np.ndarray:
    """LM head W[V,d] ~ N(0, std^2).  dtype 'f32' -> float32; 'bf16' -> uint16 bit patterns."""
    g = _rng(seed)
    if dtype == "f32":
        out = np.empty((V, d), dtype=np.float32)
    elif dtype == "bf16":
        out = np.empty((V, d), dtype=np.uint16)
    else:
        raise ValueError(dtype)
    for lo in range(0, V, chunk_rows):
        hi = min(V, lo + chunk_rows)
        x = g.standard_normal((hi - lo, d), dtype=np.float32) * np.float32(std)
        out[lo:hi] = x if dtype == "f32" else f32_to_bf16_bits(x)
    return out


def hidden_rows(n: int, d: int, seed: int, dtype: str) -> np.ndarray:
    """Drafter final hidden states h[n,d] ~ N(0,1) in the head's dtype."""
    x = _rng(seed + 3).standard_normal((n, d), dtype=np.float32)
    if dtype == "f32":
        return x
    if dtype == "bf16":
        return f32_to_bf16_bits(x)
    raise ValueError(dtype)


# --------------------------------------------------------------------------
# the five workloads
# --------------------------------------------------------------------------
@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    V: int
    d: int
    dtype: str          # 'f32' | 'bf16'
    n_ids: int
    zipf_s: float
    permute: bool
    k: tuple            # trimmed sizes
    n: tuple            # hidden rows per step
    m: tuple            # top-m
    seed: int


WORKLOADS = {
    "tiny": Workload("tiny", 4096, 256, "f32", 200_000, 1.1, False, (1024,), (4,), (1, 4), 1000),
    "llama1b": Workload("llama1b", 128256, 2048, "bf16", 10_000_000, 1.1, True,
                        (32768, 128256), (1,), (1,), 2000),
    "llama3b": Workload("llama3b", 128256, 3072, "bf16", 10_000_000, 1.1, True,
                        (8192, 16384, 32768, 65536, 128256), (1, 2, 4, 8), (1, 8), 3000),
    "llama8b": Workload("llama8b", 128256, 4096, "bf16", 10_000_000, 1.1, True,
                        (32768,), (64,), (8,), 4000),
    "stress": Workload("stress", 128256, 8192, "bf16", 100_000_000, 1.05, True,
                       (32768,), (256,), (16,), 5000),
}


def trimmed_head_direct(k: int, d: int, seed: int, dtype: str):
    """A [k,d] head plus an ascending id map drawn directly (no full head needed).

    Used where only the draft step is exercised at full size: the rows are
    i.i.d. N(0, 0.02^2) exactly as rows gathered from a full head would be,
    and the map is a sorted random k-subset of the Llama-3 vocabulary.
    """
    W = head_weights(k, d, seed, dtype)
    V = 128256 if k <= 128256 else k
    ids = np.sort(_rng(seed + 2).choice(V, size=k, replace=False)).astype(np.int32)
    return W, ids
