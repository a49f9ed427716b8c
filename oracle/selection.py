"""CPU oracle for the alternative vocabulary-selection criteria and the frequency-rank order.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Sec. 3.2 closes with: besides a fixed k, the trimmed vocabulary may be chosen by Top-P over the
token counts or by a minimum-frequency threshold.  Written out from that sentence:

  rank order   ids sorted by (count descending, id ascending) -- the order in which Top-K(c, k)
               takes them, so every prefix of it is the selection for a smaller k.
  Top-P        the smallest k >= 1 whose k most frequent ids carry at least P of all counted
               tokens:  S_k >= P * S_V  with S_k the sum of the k largest counts.  P * S_V is
               evaluated in fp64 (one multiplication) and S_k, an integer, is compared with its
               ceiling; this fixes what "at least" means when P * S_V is not an integer.
  min count    every id seen at least f_min times:  k = #{ t : c[t] >= f_min }  (may be 0).
  coverage     S_k / S_V, the share of the calibration tokens the trimmed vocabulary covers.
"""
from __future__ import annotations

import math

import numpy as np


def rank_order(counts: np.ndarray) -> np.ndarray:
    """All ids by (count desc, id asc), int32 [V]: a plain full sort of the (count, id) pairs."""
    pairs = [(-int(c), t) for t, c in enumerate(np.asarray(counts, dtype=np.int64).tolist())]
    pairs.sort()                                   # tuples compare by -count, then id
    return np.array([t for _, t in pairs], dtype=np.int32)


def choose_k_top_p(counts: np.ndarray, P: float):
    """Returns (k, covered, total) with k the smallest prefix of the rank order whose mass >= P * total."""
    c = sorted((int(x) for x in np.asarray(counts, dtype=np.int64).tolist()), reverse=True)
    total = sum(c)
    target = int(math.ceil(float(P) * float(total)))     # one fp64 product, then its ceiling
    s = 0
    for k, x in enumerate(c, start=1):
        s += x
        if s >= target:
            return k, s, total
    raise AssertionError("P must be <= 1")


def choose_k_min_count(counts: np.ndarray, f_min: int):
    """Returns (k, covered, total) with k = number of ids counted at least f_min times."""
    c = [int(x) for x in np.asarray(counts, dtype=np.int64).tolist()]
    kept = [x for x in c if x >= int(f_min)]
    return len(kept), sum(kept), sum(c)
