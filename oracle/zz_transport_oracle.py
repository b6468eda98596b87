"""fp64 oracle for the paper's transport optimisation (Section 2.2, Eq. 5).

TEST INFRASTRUCTURE ONLY (see oracle/zz_oracle.py); shares no code with the library.

Follows the paper's steps in its own order and notation:
  1. DuoAttention's classification (Section 2.1): heads are sorted by their converged
     importance alpha; with sparsity s the L*H*s heads of smallest alpha are streaming
     heads, the rest retrieval heads.
  2. A candidate is a set of p = s*L layers that become all-streaming; the other q = L-p
     layers become all-retrieval.  That fixes the operation o_{i,j} of every head:
     o0 keep its kind (cost 0), o1 retrieval -> streaming (cost +alpha_{i,j}),
     o2 streaming -> retrieval (cost -omega*alpha_{i,j}).
  3. L_zigzag is the sum of those costs; every candidate is examined one by one and the
     minimum is kept (the paper enumerates; so does this file).

Readings: the printed "-omega*alpha" carries the head's subscripts; the printed count of
candidates is C(L, p); ties between equal alphas at the classification threshold are broken
by (layer, head) order; ties between candidates by the lexicographically smallest layer set.
"""
from __future__ import annotations

from itertools import combinations

import numpy as np


def classify_heads(alpha, sparsity):
    """bool[L,H]: True where DuoAttention makes the head a streaming head."""
    alpha = np.asarray(alpha, dtype=np.float64)
    L, H = alpha.shape
    assert abs(sparsity * L - round(sparsity * L)) < 1e-4, "p / L = s needs a whole number of layers"
    n_stream = int(round(sparsity * L)) * H
    order = sorted(range(L * H), key=lambda t: (alpha.flat[t], t))   # ascending alpha, stable
    is_streaming = np.zeros(L * H, dtype=bool)
    is_streaming[order[:n_stream]] = True
    return is_streaming.reshape(L, H)


def zigzag_loss(alpha, head_is_streaming, streaming_layers, omega):
    """L_zigzag of Eq. 5 for one candidate set of all-streaming layers."""
    alpha = np.asarray(alpha, dtype=np.float64)
    L, H = alpha.shape
    chosen = set(streaming_layers)
    total = 0.0
    for i in range(L):
        for j in range(H):
            was_streaming = bool(head_is_streaming[i, j])
            becomes_streaming = i in chosen
            if was_streaming == becomes_streaming:
                cost = 0.0                                  # o0
            elif becomes_streaming:
                cost = alpha[i, j]                          # o1: retrieval -> streaming
            else:
                cost = -omega * alpha[i, j]                 # o2: streaming -> retrieval
            total += cost
    return total


def solve_by_enumeration(alpha, sparsity, omega):
    """Examines all C(L, p) candidates.  Returns (sorted tuple of streaming layers, loss)."""
    alpha = np.asarray(alpha, dtype=np.float64)
    L, H = alpha.shape
    p = int(round(sparsity * L))
    kinds = classify_heads(alpha, sparsity)
    best, best_loss = None, None
    for cand in combinations(range(L), p):
        loss = zigzag_loss(alpha, kinds, cand, omega)
        if best_loss is None or loss < best_loss - 1e-15:
            best, best_loss = cand, loss
    return best, best_loss
