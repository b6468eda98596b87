"""fp64 CPU oracle for rotary position encoding applied to K at append time.

TEST INFRASTRUCTURE ONLY; shares no code with the HIP path; only tests may import it.

The paper (arXiv 2508.12407) does not mention position encoding; its model (Section 3.1: a
Llama-3-8B long-context model) uses rotary embeddings, and encoding K where it is appended
is a step right next to the hot path (the paper's point, Section 1, is per-layer overhead
around attention).  What is computed is the rotary
embedding of Su et al. in the pairing that model family uses: element i of a head vector is
rotated together with element i + D/2 by the angle of (position, i):

    y[i]       = x[i] * cos[p, i] - x[i + D/2] * sin[p, i]
    y[i + D/2] = x[i + D/2] * cos[p, i] + x[i] * sin[p, i]          0 <= i < D/2

with p the token's absolute position in its sequence (a reading: streaming caches keep the
positions the tokens had; no re-indexing inside the window).  cos and sin are tables
[rows, D/2] handed in by the caller, so the oracle is the rotation alone, in fp64, written out.

Pinned by tests/test_rope_oracle_pins.py: angle 0 is the identity, a quarter turn swaps the
halves with a sign, norms of pairs are preserved, two rotations compose to the rotation by
the sum of the angles, with tables of the form angle = p * f_i a score depends on the
difference of positions only, and the partner of element i is i + D/2 (one-hot probe).
"""
from __future__ import annotations

import numpy as np


def rotate(x, cos_rows, sin_rows):
    """x [..., D] rotated pairwise (i, i + D/2) by angles given as cos_rows, sin_rows [..., D/2]
    (broadcast against x's leading axes)."""
    x = np.asarray(x, dtype=np.float64)
    c = np.asarray(cos_rows, dtype=np.float64)
    s = np.asarray(sin_rows, dtype=np.float64)
    half = x.shape[-1] // 2
    assert x.shape[-1] == 2 * half and c.shape[-1] == half and s.shape[-1] == half
    lo, hi = x[..., :half], x[..., half:]
    out = np.empty_like(x)
    out[..., :half] = lo * c - hi * s
    out[..., half:] = hi * c + lo * s
    return out


def rotate_keys(K, positions, cos, sin):
    """K [B, n, Hkv, D] for tokens at `positions` ([n], or [B, n] when the sequences of the
    batch stand at different positions) -> rotated K, fp64.  cos, sin: [rows, D/2]."""
    K = np.asarray(K, dtype=np.float64)
    B, n, H, D = K.shape
    pos = np.asarray(positions, dtype=np.int64)
    if pos.ndim == 1:
        pos = np.broadcast_to(pos[None, :], (B, n))
    assert pos.shape == (B, n) and pos.min() >= 0 and pos.max() < np.asarray(cos).shape[0]
    c = np.asarray(cos, dtype=np.float64)[pos][:, :, None, :]      # [B, n, 1, D/2]
    s = np.asarray(sin, dtype=np.float64)[pos][:, :, None, :]
    return rotate(K, c, s)
