"""Oracle for the logits front end: temperature, nucleus (top-p) filter, softmax.
TEST INFRASTRUCTURE ONLY.

The paper's experiments sample at temperature 0.2 with nucleus top-p 0.95 (captions of the
result tables in Section 4); the acceptance rule of Section 2.2 consumes the probabilities the
two models assign AFTER that warp, so the warp is what produces the rows p and q.

Definition, per row of V logits, in fp64:
  1. z = logits / T,  P = softmax(z)  (max-subtracted).
  2. Order the tokens by decreasing P, equal probabilities by increasing token id.
  3. Keep the shortest prefix of that order whose probabilities sum to at least top_p (the token
     that crosses top_p is kept; top_p >= 1 keeps everything; at least one token is kept).
  4. Output P on the kept tokens divided by their sum, 0 elsewhere.
Plain numpy; a Python loop over rows.
"""
from __future__ import annotations

import numpy as np


def nucleus_size(sorted_probs: np.ndarray, top_p: float) -> int:
    """Length of the shortest prefix of a decreasing probability vector that sums to >= top_p."""
    if top_p >= 1.0:
        return len(sorted_probs)
    csum = np.cumsum(sorted_probs)
    reached = np.nonzero(csum >= top_p)[0]
    return int(reached[0]) + 1 if len(reached) else len(sorted_probs)


def warp_row(logits: np.ndarray, temperature: float, top_p: float):
    """One row -> (probabilities after the warp, boolean kept mask, softmax before the filter)."""
    z = np.asarray(logits, np.float64) / float(temperature)
    z = z - z.max()
    e = np.exp(z)
    P = e / e.sum()
    ids = np.arange(len(P))
    order = np.lexsort((ids, -P))  # primary key -P (decreasing P), ties by token id
    n = nucleus_size(P[order], float(top_p))
    kept = np.zeros(len(P), bool)
    kept[order[:n]] = True
    out = np.where(kept, P, 0.0)
    return out / out.sum(), kept, P


def warp_probs(logits: np.ndarray, temperature: float, top_p: float) -> np.ndarray:
    """[..., V] logits -> [..., V] fp64 probabilities after temperature and nucleus filtering."""
    logits = np.asarray(logits)
    flat = logits.reshape(-1, logits.shape[-1])
    out = np.empty(flat.shape, np.float64)
    for r in range(flat.shape[0]):
        out[r] = warp_row(flat[r], temperature, top_p)[0]
    return out.reshape(logits.shape)
