"""CPU oracle for the draft-tree selection steps downstream of the draft head.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

The experimental settings (Sec. 4.1, "Draft Tree") grow an EAGLE-2 style tree: depth 3, top-K = 8
children per level, at most 32 draft tokens (60 in the depth ablation of Sec. 4.2).  What is
computed is a plain definition, written out here with a full sort:

  expansion  every frontier node i proposes its m best tokens with log-probs lp[i, j]; candidate
             (i, j) scores  cum[i] + lp[i, j]  (cumulative log-probability of the path); the K
             best candidates form the next frontier.
  rerank     of all N nodes drafted so far, the T with the best cumulative score are kept and
             handed on in node-index order (parents precede their children in that order).

The score is ONE fp32 addition (the step's log-probs and the running scores are fp32 and the
decision "which candidates survive" is an integer outcome, so both sides take it in fp32).
Ties (equal fp32 scores, -0.0 == +0.0) go to the lower flat candidate index i * m + j,
respectively the lower node index: a reading, the paper does not say.
"""
from __future__ import annotations

import numpy as np


def tree_expand(parent_cum: np.ndarray, step_logp: np.ndarray, step_ids: np.ndarray, K: int):
    """Returns (parent int32 [K], token int32 [K], cum float32 [K]), best candidate first."""
    parent_cum = np.asarray(parent_cum, dtype=np.float32)
    step_logp = np.asarray(step_logp, dtype=np.float32)
    n, m = step_logp.shape
    assert parent_cum.shape == (n,) and step_ids.shape == (n, m) and 1 <= K <= n * m
    score = np.empty((n, m), dtype=np.float32)
    for i in range(n):
        for j in range(m):
            score[i, j] = np.float32(parent_cum[i]) + np.float32(step_logp[i, j])   # one fp32 addition
    flat = score.reshape(-1)
    order = sorted(range(n * m), key=lambda c: (-float(flat[c]), c))[:K]
    parent = np.array([c // m for c in order], dtype=np.int32)
    token = np.array([step_ids[c // m, c % m] for c in order], dtype=np.int32)
    cum = np.array([flat[c] for c in order], dtype=np.float32)
    return parent, token, cum


def tree_rerank(cum: np.ndarray, T: int) -> np.ndarray:
    """Indices (int32 [T], ascending) of the T best cumulative scores; ties -> lower index."""
    cum = np.asarray(cum, dtype=np.float32)
    N = cum.shape[0]
    assert cum.ndim == 1 and 1 <= T <= N
    order = sorted(range(N), key=lambda c: (-float(cum[c]), c))[:T]
    return np.array(sorted(order), dtype=np.int32)
