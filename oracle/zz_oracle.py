"""fp64 CPU oracle for ZigzagAttention's inference hot path.

TEST INFRASTRUCTURE ONLY.  This file is the plain definition of what the GPU
library must compute; it is slow on purpose (O(n^2), no tiling, no online
softmax, no ring buffer inside the attention routine) and shares no code with
the HIP path.  Only tests, the smoke check and the benchmark's `cpu_baseline`
leg may import it; the product never does.

What it follows in the paper (arXiv 2508.12407):
  * Section 1 / Section 2.1: a *retrieval* head runs ordinary full (causal)
    attention over every cached token; a *streaming* head keeps only the
    attention-sink tokens and a recent window and drops the rest of its KV.
  * Section 2.2: ZigzagAttention makes a whole layer one kind or the other
    (p of L layers streaming, p/L = sparsity), so one attention per layer.
  * Section 2.1 (end): the DuoAttention layout mixes both kinds of head in one
    layer (the comparison baseline).
  * Section 3.3: sink size and window length are the two streaming parameters.

Readings where the paper is silent (kept in step with the design notes):
  * the window is the W most recent positions *including* the query's own,
    so a streaming head sees at most S + W tokens;
  * positions < S live in S fixed slots; only positions >= S use the W-slot ring;
  * softmax scale defaults to 1/sqrt(D); no positional re-encoding here;
  * under GQA, "head" kind is a property of the KV head; query head h reads
    KV head h // G with G = Hq / Hkv.

Every function is pinned by tests/test_oracle_pins.py (closed forms, brute
force masks, set identities); nothing here is "parity unpinned".
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor

import numpy as np

# --------------------------------------------------------------------------
# Which past positions j a query at position i may attend to.
# Both accept a scalar i and a scalar or integer array j.
# --------------------------------------------------------------------------


def allowed_retrieval(i, j):
    """Full causal attention (retrieval head, Section 2.1): every j <= i."""
    return np.asarray(j) <= i


def allowed_streaming(i, j, sink, window):
    """Streaming attention (Sections 1, 3.3): causal, and j is either one of the
    first `sink` positions or among the `window` most recent ones (i included)."""
    j = np.asarray(j)
    return (j <= i) & ((j < sink) | (i - j < window))


def attended_positions(i, streaming, sink, window):
    """Sorted array of the positions query i attends to."""
    j = np.arange(i + 1)
    keep = allowed_streaming(i, j, sink, window) if streaming else allowed_retrieval(i, j)
    return j[keep]


# --------------------------------------------------------------------------
# Attention by its definition.
# --------------------------------------------------------------------------


def softmax_weights(scores):
    """p_j = exp(s_j - max s) / sum_j exp(s_j - max s) for a 1-D fp64 vector."""
    s = np.asarray(scores, dtype=np.float64)
    e = np.exp(s - s.max())
    return e / e.sum()


def attention_row(q_vec, K_rows, V_rows, scale):
    """One query against the rows it may see: sum_j softmax_j(scale q.k_j) v_j.
    q_vec [D], K_rows/V_rows [n, D], all promoted to fp64."""
    q = np.asarray(q_vec, dtype=np.float64)
    K = np.asarray(K_rows, dtype=np.float64)
    V = np.asarray(V_rows, dtype=np.float64)
    p = softmax_weights(scale * (K @ q))
    return p @ V


def default_scale(head_dim):
    return 1.0 / np.sqrt(float(head_dim))


def attention(Q, K, V, streaming_per_kv_head, sink, window, scale=None, rows=None):
    """Attention outputs for query positions `rows` (default: all T).

    Q [B,T,Hq,D]; K,V [B,T,Hkv,D] hold *every* token ever seen (never evicted).
    streaming_per_kv_head: bool[Hkv]; a zigzag layer passes all-equal entries
    (Section 2.2), the mixed-head baseline passes a genuine mix (Section 2.1).
    Returns fp64 [B, len(rows), Hq, D].
    """
    Q = np.asarray(Q)
    K = np.asarray(K)
    V = np.asarray(V)
    B, T, Hq, D = Q.shape
    Hkv = K.shape[2]
    assert Hq % Hkv == 0 and K.shape == V.shape and K.shape[0] == B and K.shape[3] == D
    G = Hq // Hkv
    kinds = np.broadcast_to(np.asarray(streaming_per_kv_head, dtype=bool), (Hkv,))
    if scale is None:
        scale = default_scale(D)
    if rows is None:
        rows = range(T)
    rows = list(rows)
    out = np.zeros((B, len(rows), Hq, D), dtype=np.float64)
    for b in range(B):
        for h in range(Hq):
            g = h // G
            Kg = K[b, :, g, :].astype(np.float64)
            Vg = V[b, :, g, :].astype(np.float64)
            for r, i in enumerate(rows):
                J = attended_positions(i, bool(kinds[g]), sink, window)
                out[b, r, h, :] = attention_row(Q[b, i, h, :], Kg[J], Vg[J], scale)
    return out


def attention_layer(Q, K, V, layer_is_streaming, sink, window, scale=None, rows=None):
    """A zigzag layer: every KV head of the layer has the same kind."""
    Hkv = np.asarray(K).shape[2]
    return attention(Q, K, V, np.full(Hkv, bool(layer_is_streaming)), sink, window, scale, rows)


def decode_row(q, K, V, i, streaming_per_kv_head, sink, window, scale=None):
    """Decode at step i == row i of `attention` (not a separate algorithm).
    q [B,Hq,D] is the query of position i; K,V [B,T,Hkv,D] with T > i."""
    q = np.asarray(q)
    B, Hq, D = q.shape
    T = np.asarray(K).shape[1]
    Qfull = np.zeros((B, T, Hq, D), dtype=np.float64)
    Qfull[:, i] = q
    return attention(Qfull, K, V, streaming_per_kv_head, sink, window, scale, rows=[i])[:, 0]


# --------------------------------------------------------------------------
# Cache model (integers only): which position a cache slot holds.
# --------------------------------------------------------------------------


def cache_capacity(streaming, sink, window, max_ctx):
    """Tokens a (layer, KV head) keeps: everything, or sink + window."""
    return sink + window if streaming else max_ctx


def slot_position(slot, n, streaming, sink, window):
    """Position held by `slot` after n tokens (positions 0..n-1) were appended,
    or -1 if the slot was never written.

    Retrieval: slot s holds position s.  Streaming: slots [0,S) hold the sink
    positions; slot S + r holds the newest position p <= n-1 with p >= S and
    (p - S) mod W == r.
    """
    if slot < 0:
        return -1
    if not streaming:
        return slot if slot < n else -1
    if slot < sink:
        return slot if slot < n else -1
    r = slot - sink
    if r >= window or sink + r > n - 1:
        return -1
    newest = n - 1 - sink                       # offset of the newest ring token
    return sink + r + window * ((newest - r) // window)


def n_occupied(n, streaming, sink, window):
    return min(n, sink + window) if streaming else n


def expected_cache(X, n, streaming, sink, window, capacity):
    """Logical cache image after n appends: [B, Hkv, capacity, D] taken from the
    never-evicted X [B,T,Hkv,D], plus bool valid[capacity].  Invalid slots are 0."""
    X = np.asarray(X)
    B, T, Hkv, D = X.shape
    img = np.zeros((B, Hkv, capacity, D), dtype=X.dtype)
    valid = np.zeros(capacity, dtype=bool)
    for s in range(capacity):
        p = slot_position(s, n, streaming, sink, window)
        if p >= 0:
            img[:, :, s, :] = X[:, p, :, :]
            valid[s] = True
    return img, valid


# --------------------------------------------------------------------------
# Bounded bulk evaluation (benchmark's cpu_baseline leg and sampled parity).
# --------------------------------------------------------------------------


def decode_unit(q_group, K_unit, V_unit, scale):
    """All G query heads of one (batch, KV head) unit at the newest position.
    q_group [G,D]; K_unit,V_unit [n,D] are exactly the rows the unit attends to."""
    Kd = np.asarray(K_unit, dtype=np.float64)
    Vd = np.asarray(V_unit, dtype=np.float64)
    return np.stack([attention_row(qh, Kd, Vd, scale) for qh in np.asarray(q_group)])


def decode_units(units, scale, threads=1):
    """units: list of (q_group, K_unit, V_unit).  Independent units are spread
    over `threads` host threads; nothing else is parallelised."""
    if threads <= 1:
        return [decode_unit(q, k, v, scale) for (q, k, v) in units]
    with ThreadPoolExecutor(max_workers=threads) as ex:
        return list(ex.map(lambda u: decode_unit(u[0], u[1], u[2], scale), units))
