"""Pins for the fp64 oracle: each test ties it to something other than itself
(a closed form, a brute-force loop written differently, a library routine, a
set identity), chosen so a dropped term, wrong sign/index or transposed operand
in oracle/zz_oracle.py fails at least one of them."""
import itertools
import os

import numpy as np
import pytest
import scipy.special

import zz_inputs
from oracle import zz_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "closed_forms.txt")


def brute_force_mask(T, streaming, S, W):
    """Third, independent statement of the two masks as an explicit T x T matrix."""
    M = np.zeros((T, T), dtype=bool)
    for i in range(T):
        for j in range(T):
            if j > i:
                continue
            if not streaming:
                M[i, j] = True
            elif j < S:
                M[i, j] = True
            elif j > i - W:
                M[i, j] = True
    return M


def dense_masked_attention(Q, K, V, M, scale):
    """Library route: dense score matrix, -inf outside the mask, scipy softmax."""
    B, T, Hq, D = Q.shape
    Hkv = K.shape[2]
    G = Hq // Hkv
    out = np.zeros((B, T, Hq, D))
    for b in range(B):
        for h in range(Hq):
            g = h // G
            Sc = scale * (Q[b, :, h, :].astype(np.float64) @ K[b, :, g, :].astype(np.float64).T)
            Sc = np.where(M, Sc, -np.inf)
            P = scipy.special.softmax(Sc, axis=1)
            out[b, :, h, :] = P @ V[b, :, g, :].astype(np.float64)
    return out


# ---- P1: softmax weights -------------------------------------------------

def test_p1_softmax_rows_sum_to_one_and_nonnegative():
    rng = np.random.default_rng(0)
    for n in (1, 2, 17, 1000):
        s = rng.standard_normal(n) * 30.0
        p = O.softmax_weights(s)
        assert abs(p.sum() - 1.0) < 1e-12
        assert (p >= 0).all()
        # ratios follow exp of logit differences (definition, not re-use)
        k = int(np.argmax(s))
        assert np.allclose(p / p[k], np.exp(s - s[k]), rtol=1e-12, atol=0)


def test_p1_softmax_huge_logits_do_not_overflow():
    p = O.softmax_weights(np.array([1e4, 1e4 - 1.0, -1e4]))
    assert np.isfinite(p).all()
    assert np.allclose(p, [1 / (1 + np.exp(-1.0)), np.exp(-1.0) / (1 + np.exp(-1.0)), 0.0], atol=1e-15)


# ---- P2: S + W >= T  =>  streaming == full; differs first at T = S + W + 1 ----

@pytest.mark.parametrize("S,W", [(4, 8), (0, 5), (3, 1), (16, 64)])
def test_p2_streaming_equals_full_when_window_covers_context(S, W):
    T = S + W + 1
    q, k, v = zz_inputs.make_qkv(3, 1, T, 4, 2, 16, bf16=False)
    full = O.attention_layer(q, k, v, False, S, W)
    strm = O.attention_layer(q, k, v, True, S, W)
    # rows 0 .. S+W-1 see exactly [0, i] either way
    assert np.array_equal(full[:, : S + W], strm[:, : S + W])
    # the last row loses exactly one token (position S) and must differ
    assert np.abs(full[:, S + W] - strm[:, S + W]).max() > 1e-6
    assert len(O.attended_positions(S + W, True, S, W)) == S + W
    assert S not in set(O.attended_positions(S + W, True, S, W))


# ---- P3 / P11: explicit brute-force mask + scipy softmax ---------------------

@pytest.mark.parametrize("streaming", [False, True])
@pytest.mark.parametrize("S,W,T", [(4, 8, 40), (0, 3, 17), (5, 1, 12), (16, 64, 150)])
def test_p3_matches_dense_attention_under_bruteforce_mask(streaming, S, W, T):
    q, k, v = zz_inputs.make_qkv(11 + T, 2, T, 4, 2, 8, bf16=False)
    got = O.attention_layer(q, k, v, streaming, S, W, scale=0.31)
    M = brute_force_mask(T, streaming, S, W)
    want = dense_masked_attention(q, k, v, M, 0.31)
    assert np.allclose(got, want, rtol=1e-11, atol=1e-12)


def test_p3_predicates_match_bruteforce_mask_elementwise():
    for S, W, T in [(4, 8, 40), (0, 3, 17), (2, 1, 9)]:
        M = brute_force_mask(T, True, S, W)
        R = brute_force_mask(T, False, S, W)
        for i in range(T):
            j = np.arange(T)
            assert np.array_equal(O.allowed_streaming(i, j, S, W), M[i])
            assert np.array_equal(O.allowed_retrieval(i, j), R[i])


# ---- P4: decode step t == prefill row t; chunking is not an algorithm ----------

def test_p4_decode_equals_prefill_row_and_chunks_concatenate():
    S, W, T = 4, 8, 45
    q, k, v = zz_inputs.make_qkv(5, 1, T, 4, 2, 16, bf16=False)
    for streaming in (False, True):
        whole = O.attention_layer(q, k, v, streaming, S, W)
        for t in (0, 3, 4, 11, 12, 13, 44):
            # decode sees only tokens 0..t: truncating K,V after t must not matter
            dec = O.decode_row(q[:, t], k[:, : t + 1], v[:, : t + 1], t, np.full(2, streaming), S, W)
            assert np.allclose(dec, whole[:, t], rtol=1e-13, atol=1e-14)
        for chunk in (7, 8, 9, 45, 100):
            parts = [O.attention_layer(q, k, v, streaming, S, W, rows=range(a, min(a + chunk, T)))
                     for a in range(0, T, chunk)]
            assert np.array_equal(np.concatenate(parts, axis=1), whole)


# ---- P5: uniform keys => mean of V over the attended set (closed forms) ---------

def _golden_rows():
    rows = []
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        rows.append(tuple(int(x) for x in line.split()))
    return rows


@pytest.mark.parametrize("S,W,i,count,sum_j,sum_j2", _golden_rows())
def test_p5_uniform_keys_closed_form(S, W, i, count, sum_j, sum_j2):
    T = i + 1
    D = 4
    Q = np.random.default_rng(1).standard_normal((1, T, 1, D))
    K = np.zeros((1, T, 1, D))
    V = np.zeros((1, T, 1, D))
    j = np.arange(T, dtype=np.float64)
    V[0, :, 0, 0] = 1.0
    V[0, :, 0, 1] = j
    V[0, :, 0, 2] = j * j
    out = O.attention_layer(Q, K, V, True, S, W, rows=[i])[0, 0, 0]
    assert abs(out[0] - 1.0) < 1e-12
    assert abs(out[1] * count - sum_j) < 1e-6 * max(1, sum_j)
    assert abs(out[2] * count - sum_j2) < 1e-9 * max(1, sum_j2)
    # retrieval: mean over 0..i
    outr = O.attention_layer(Q, K, V, False, S, W, rows=[i])[0, 0, 0]
    assert abs(outr[1] - i / 2.0) < 1e-9 * max(1, i)
    assert abs(outr[2] - i * (2 * i + 1) / 6.0) < 1e-9 * max(1, i * i)


def test_p5_attended_count_is_min_of_context_and_budget():
    S, W = 16, 64
    for i in range(0, 200):
        assert len(O.attended_positions(i, True, S, W)) == min(i + 1, S + W)
        assert len(O.attended_positions(i, False, S, W)) == i + 1


# ---- P6: one dominant key: output = V[j*] iff j* is visible ----------------------

def test_p6_one_hot_key_sweeps_mask_edges():
    S, W, T, D = 4, 8, 40, 16
    i = T - 1
    rng = np.random.default_rng(2)
    qv = rng.standard_normal(D)
    qv *= np.sqrt(D) / np.linalg.norm(qv)          # |q|^2 = D
    for jstar in (0, S - 1, S, S + 1, i - W - 1, i - W, i - W + 1, i - W + 2, i - 1, i):
        Q = np.zeros((1, T, 1, D))
        Q[0, i, 0] = qv
        K = np.zeros((1, T, 1, D))
        K[0, jstar, 0] = 60.0 * qv / np.sqrt(D)     # scale * q.k = 60 with scale 1/sqrt(D)
        V = rng.standard_normal((1, T, 1, D))
        out = O.attention_layer(Q, K, V, True, S, W, rows=[i])[0, 0, 0]
        visible = (jstar < S) or (i - jstar < W)
        if visible:
            assert np.allclose(out, V[0, jstar, 0], atol=1e-12)
        else:
            A = O.attended_positions(i, True, S, W)
            assert np.allclose(out, V[0, A, 0].mean(axis=0), atol=1e-12)
        # retrieval always sees it
        outr = O.attention_layer(Q, K, V, False, S, W, rows=[i])[0, 0, 0]
        assert np.allclose(outr, V[0, jstar, 0], atol=1e-12)


# ---- P7: textbook special cases --------------------------------------------

def test_p7_single_token_and_equal_logits():
    rng = np.random.default_rng(4)
    Q = rng.standard_normal((1, 2, 2, 8))
    K = rng.standard_normal((1, 2, 1, 8))
    V = rng.standard_normal((1, 2, 1, 8))
    out = O.attention_layer(Q, K, V, False, 1, 1)
    assert np.allclose(out[0, 0, 0], V[0, 0, 0], atol=1e-15)
    K[0, 1, 0] = K[0, 0, 0]
    out = O.attention_layer(Q, K, V, False, 1, 2)
    assert np.allclose(out[0, 1, 1], 0.5 * (V[0, 0, 0] + V[0, 1, 0]), atol=1e-15)


def test_p7_two_token_sigmoid_closed_form():
    # two tokens: p_1 = sigmoid(scale (q.k1 - q.k0)); transposed operands or a
    # missing scale change the value.
    q = np.array([1.0, -2.0, 0.5]); k0 = np.array([0.3, 0.1, -1.0]); k1 = np.array([-0.7, 0.2, 2.0])
    v0 = np.array([1.0, 0.0, 0.0]); v1 = np.array([0.0, 1.0, 0.0])
    scale = 0.7
    out = O.attention_row(q, np.stack([k0, k1]), np.stack([v0, v1]), scale)
    p1 = 1.0 / (1.0 + np.exp(-scale * (q @ k1 - q @ k0)))
    assert np.allclose(out, [1 - p1, p1, 0.0], atol=1e-15)
    assert O.default_scale(64) == 0.125


# ---- P8: GQA head -> KV head mapping ------------------------------------------

def test_p8_gqa_equals_mha_with_duplicated_kv_heads():
    T, Hq, Hkv, D = 20, 8, 2, 8
    q, k, v = zz_inputs.make_qkv(6, 2, T, Hq, Hkv, D, bf16=False)
    G = Hq // Hkv
    k_dup = np.repeat(k, G, axis=2)               # head h <- KV head h // G
    v_dup = np.repeat(v, G, axis=2)
    for streaming in (False, True):
        gqa = O.attention_layer(q, k, v, streaming, 2, 5)
        mha = O.attention_layer(q, k_dup, v_dup, streaming, 2, 5)
        assert np.array_equal(gqa, mha)
    # and the mapping is not h % Hkv: swapping that in must change the answer
    k_mod = np.tile(k, (1, 1, G, 1))
    v_mod = np.tile(v, (1, 1, G, 1))
    assert np.abs(O.attention_layer(q, k_mod, v_mod, False, 2, 5) - mha).max() > 1e-3


def test_p8_mixed_heads_follow_their_own_kind():
    T, Hq, Hkv, D = 30, 4, 2, 8
    q, k, v = zz_inputs.make_qkv(8, 1, T, Hq, Hkv, D, bf16=False)
    mixed = O.attention(q, k, v, np.array([True, False]), 3, 4)
    allS = O.attention_layer(q, k, v, True, 3, 4)
    allR = O.attention_layer(q, k, v, False, 3, 4)
    assert np.array_equal(mixed[:, :, :2], allS[:, :, :2])     # q heads 0,1 -> KV head 0 (streaming)
    assert np.array_equal(mixed[:, :, 2:], allR[:, :, 2:])     # q heads 2,3 -> KV head 1 (retrieval)


# ---- P9: invariances ----------------------------------------------------------

def test_p9_logit_shift_and_permutation_invariance():
    rng = np.random.default_rng(9)
    n, D = 50, 8
    q = rng.standard_normal(D); K = rng.standard_normal((n, D)); V = rng.standard_normal((n, D))
    base = O.attention_row(q, K, V, 0.4)
    shifted = O.attention_row(q, K + 3.0 * q / (q @ q), V, 0.4)   # adds 3 to every q.k
    assert np.allclose(base, shifted, rtol=1e-12, atol=1e-13)
    perm = rng.permutation(n)
    assert np.allclose(base, O.attention_row(q, K[perm], V[perm], 0.4), rtol=1e-12, atol=1e-13)


# ---- P10: cache model ------------------------------------------------------------

def simulate_appends(n, streaming, S, W, cap):
    """Brute force: append positions one at a time with the slot rule spelled out."""
    slots = [-1] * cap
    for pos in range(n):
        if not streaming:
            slots[pos] = pos
        elif pos < S:
            slots[pos] = pos
        else:
            slots[S + (pos - S) % W] = pos
    return slots


@pytest.mark.parametrize("S,W", [(4, 8), (0, 5), (3, 1), (16, 64), (1, 2)])
def test_p10_slot_positions_match_sequential_simulation(S, W):
    cap = S + W
    for n in itertools.chain(range(0, 3 * (S + W) + 3), [10 * (S + W) + 1]):
        sim = simulate_appends(n, True, S, W, cap)
        got = [O.slot_position(s, n, True, S, W) for s in range(cap)]
        assert got == sim, (S, W, n)
        occ = [s for s in range(cap) if got[s] >= 0]
        assert occ == list(range(O.n_occupied(n, True, S, W)))       # occupied == prefix
        if n > 0:
            assert set(got) - {-1} == set(O.attended_positions(n - 1, True, S, W).tolist())
        assert O.slot_position(cap, n, True, S, W) == -1


def test_p10_retrieval_slots_and_expected_cache_image():
    n, cap = 13, 20
    assert [O.slot_position(s, n, False, 0, 1) for s in range(cap)] == simulate_appends(n, False, 0, 1, cap)
    X = np.arange(2 * 30 * 3 * 2, dtype=np.float64).reshape(2, 30, 3, 2)
    img, valid = O.expected_cache(X, 27, True, 4, 8, 12)
    sim = simulate_appends(27, True, 4, 8, 12)
    assert valid.all()
    for s, p in enumerate(sim):
        assert np.array_equal(img[:, :, s, :], X[:, p, :, :])
    img, valid = O.expected_cache(X, 5, True, 4, 8, 12)
    assert valid.tolist() == [True] * 5 + [False] * 7
    assert O.cache_capacity(True, 4, 8, 100) == 12 and O.cache_capacity(False, 4, 8, 100) == 100


# ---- bulk helper equals the row definition ------------------------------------------

def test_decode_units_equals_attention_rows_on_attended_sets():
    S, W, T = 4, 8, 60
    q, k, v = zz_inputs.make_qkv(12, 2, T, 4, 2, 16)
    i = T - 1
    scale = O.default_scale(16)
    for streaming in (False, True):
        ref = O.attention_layer(q, k, v, streaming, S, W, rows=[i])[:, 0]      # [B,Hq,D]
        J = O.attended_positions(i, streaming, S, W)
        units = [(q[b, i, 2 * g: 2 * g + 2], k[b, J, g], v[b, J, g]) for b in range(2) for g in range(2)]
        for threads in (1, 3):
            outs = O.decode_units(units, scale, threads=threads)
            got = np.stack(outs).reshape(2, 4, 16)
            assert np.allclose(got, ref, rtol=1e-13, atol=1e-14)


def test_inputs_are_bf16_exact_and_seeded():
    q, k, v = zz_inputs.make_qkv(0, 1, 8, 4, 2, 64)
    q2, _, _ = zz_inputs.make_qkv(0, 1, 8, 4, 2, 64)
    assert np.array_equal(q, q2)
    bits = zz_inputs.bf16_bits(k)
    assert np.array_equal(zz_inputs.bf16_bits_to_f32(bits), k)
    # round-to-nearest-even on a tie: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert zz_inputs.round_to_bf16(np.array([1.0 + 2.0 ** -8], dtype=np.float32))[0] == 1.0
    assert zz_inputs.round_to_bf16(np.array([1.0 + 3 * 2.0 ** -8], dtype=np.float32))[0] == np.float32(1.0 + 2.0 ** -6)
    m = zz_inputs.draw_layer_mask(0, 32, 16)
    assert m.sum() == 16 and np.array_equal(m, zz_inputs.draw_layer_mask(0, 32, 16))
    hm = zz_inputs.draw_kvhead_mask(0, 32, 8, 4)
    assert (hm.sum(axis=1) == 4).all()
