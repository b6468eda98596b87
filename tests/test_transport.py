"""Transport optimisation (Section 2.2, Eq. 5): the enumeration oracle against hand-worked
cases, and the library's closed-form selection against the enumeration."""
import ctypes

import numpy as np
import pytest

from oracle import zz_transport_oracle as TO
from paper_2508_12407_amd import binding as zb


def test_oracle_classification_and_loss_on_a_hand_worked_case():
    # 2 layers x 2 heads, sparsity 0.5: the two smallest alphas (0.1, 0.2) are streaming heads
    alpha = np.array([[0.1, 0.9], [0.2, 0.6]])
    kinds = TO.classify_heads(alpha, 0.5)
    assert kinds.tolist() == [[True, False], [True, False]]
    # layer 0 all-streaming: head (0,1) retrieval->streaming costs 0.9; layer 1 all-retrieval:
    # head (1,0) streaming->retrieval costs -omega*0.2
    assert TO.zigzag_loss(alpha, kinds, (0,), 0.5) == pytest.approx(0.9 - 0.5 * 0.2)
    assert TO.zigzag_loss(alpha, kinds, (1,), 0.5) == pytest.approx(0.6 - 0.5 * 0.1)
    best, loss = TO.solve_by_enumeration(alpha, 0.5, 0.5)
    assert best == (1,) and loss == pytest.approx(0.55)
    # omega = 0: only the retrieval heads that are lost count
    assert TO.solve_by_enumeration(alpha, 0.5, 0.0) == ((1,), pytest.approx(0.6))
    # a layout that is already layer-exclusive costs nothing and is kept
    excl = np.array([[0.05, 0.1], [0.8, 0.9], [0.2, 0.15], [0.7, 0.95]])
    best, loss = TO.solve_by_enumeration(excl, 0.5, 0.3)
    assert best == (0, 2) and loss == 0.0


def test_oracle_loss_is_invariant_to_the_order_of_heads_within_a_layer():
    rng = np.random.default_rng(0)
    alpha = rng.random((6, 4))
    kinds = TO.classify_heads(alpha, 0.5)
    perm = rng.permutation(4)
    for cand in [(0, 1, 2), (1, 3, 5)]:
        assert TO.zigzag_loss(alpha, kinds, cand, 0.4) == pytest.approx(
            TO.zigzag_loss(alpha[:, perm], kinds[:, perm], cand, 0.4))


@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("L,H,s", [(8, 4, 0.5), (10, 8, 0.5), (12, 4, 0.25), (9, 3, 1 / 3), (8, 8, 0.75)])
def test_library_selection_reaches_the_enumerated_minimum(seed, L, H, s):
    rng = np.random.default_rng(100 * seed + L)
    # bimodal importances, as trained gates tend to be, plus a uniform case
    alpha = np.where(rng.random((L, H)) < 0.5, rng.random((L, H)) * 0.2, 0.6 + 0.4 * rng.random((L, H)))
    if seed % 2:
        alpha = rng.random((L, H))
    alpha = alpha.astype(np.float32)
    for omega in (0.0, 0.1, 0.5, 1.0):
        omega = float(np.float32(omega))                     # the C ABI takes omega as a float
        mask, loss = zb.transport_select(alpha, s, omega)
        best, best_loss = TO.solve_by_enumeration(alpha, s, omega)
        assert int(mask.sum()) == len(best) == int(round(s * L))
        kinds = TO.classify_heads(alpha, s)
        chosen = tuple(np.flatnonzero(mask).tolist())
        assert TO.zigzag_loss(alpha, kinds, chosen, omega) == pytest.approx(best_loss, abs=1e-9)
        assert loss == pytest.approx(best_loss, abs=1e-9)


def test_library_selection_at_the_paper_scale_and_error_codes():
    rng = np.random.default_rng(7)
    alpha = rng.random((32, 8)).astype(np.float32)           # Llama-3-8B: 32 layers x 8 KV heads
    w = float(np.float32(0.1))
    mask, loss = zb.transport_select(alpha, 0.5, w)
    assert mask.sum() == 16
    kinds = TO.classify_heads(alpha, 0.5)
    assert TO.zigzag_loss(alpha, kinds, tuple(np.flatnonzero(mask)), w) == pytest.approx(loss, abs=1e-9)
    # no single swap of a chosen and an unchosen layer improves it (local optimality of a global optimum)
    chosen, rest = list(np.flatnonzero(mask)), list(np.flatnonzero(1 - mask))
    for a in chosen[:6]:
        for b in rest[:6]:
            cand = tuple(sorted(set(chosen) - {a} | {b}))
            assert TO.zigzag_loss(alpha, kinds, cand, w) >= loss - 1e-9
    E = zb.ERR
    a = np.zeros((2, 2), np.float32)
    m = np.zeros(2, np.uint8)
    fp, up = ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_uint8)
    f = zb.lib.zz_transport_select
    assert f(None, 2, 2, 0.5, 0.1, m.ctypes.data_as(up), None) == E["EINVAL"]
    assert f(a.ctypes.data_as(fp), 2, 2, 0.5, 0.1, None, None) == E["EINVAL"]
    assert f(a.ctypes.data_as(fp), 0, 2, 0.5, 0.1, m.ctypes.data_as(up), None) == E["EINVAL"]
    assert f(a.ctypes.data_as(fp), 2, 2, 1.5, 0.1, m.ctypes.data_as(up), None) == E["ERANGE"]
    assert f(a.ctypes.data_as(fp), 2, 2, 0.5, -0.1, m.ctypes.data_as(up), None) == E["ERANGE"]
    assert f(a.ctypes.data_as(fp), 2, 2, 0.3, 0.1, m.ctypes.data_as(up), None) == E["ERANGE"]   # 0.3 * 2 layers
    a[0, 0] = 2.0
    assert f(a.ctypes.data_as(fp), 2, 2, 0.5, 0.1, m.ctypes.data_as(up), None) == E["ERANGE"]
