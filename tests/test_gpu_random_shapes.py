"""GPU parity on seeded random configurations: head counts, group sizes, head dim, sink and
window sizes (including 0 and 1), batch, context, chunk boundaries and layout are all drawn
from a seed; every case runs chunked prefill, a few decode steps (fused and two-call) and a
final bit-exact check of the cache against the oracle's cache model.  The hand-picked cases
of the other test files cover the known edges; this one covers combinations nobody picked."""
import numpy as np
import pytest

import zz_inputs
from oracle import zz_oracle as O

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

MAX_ABS, REL_L2 = 2e-2, 5e-3


def _harness():
    from paper_2508_12407_amd import harness, binding
    return harness, binding


def check(got, want, what):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    assert np.isfinite(got).all(), what
    max_abs = np.abs(got - want).max()
    rel = np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-300)
    assert max_abs <= MAX_ABS and rel <= REL_L2, (what, max_abs, rel)


def draw_case(seed):
    r = np.random.default_rng(1000 + seed)
    D = int(r.choice([64, 128]))
    Hkv = int(r.choice([1, 2, 3, 8]))
    G = int(r.choice([1, 2, 3, 4, 8, 16]))
    if Hkv * G > 32:
        G = 32 // Hkv
    B = int(r.choice([1, 2, 3]))
    S = int(r.choice([0, 1, 5, 16, 64]))
    W = int(r.choice([1, 7, 32, 100, 256]))
    T = int(r.integers(1, 520))
    steps = 3
    layout = str(r.choice(["retrieval", "streaming", "mixed"]))
    mask = (r.random(Hkv) < 0.5).astype(np.uint8)
    n_cuts = int(r.integers(0, 5))
    cuts = sorted(set([0, T] + [int(x) for x in r.integers(1, T + 1, size=n_cuts)]))
    q_gain = float(r.choice([1.0, 1.0, 4.0]))
    return dict(D=D, Hkv=Hkv, Hq=Hkv * G, B=B, S=S, W=W, T=T, steps=steps, layout=layout, mask=mask, cuts=cuts,
                q_gain=q_gain)


@pytest.mark.parametrize("seed", range(36))
def test_random_configuration(seed):
    H, zb = _harness()
    c = draw_case(seed)
    D, Hkv, Hq, B, S, W, T, steps = c["D"], c["Hkv"], c["Hq"], c["B"], c["S"], c["W"], c["T"], c["steps"]
    total = T + 2 * steps
    q, k, v = zz_inputs.make_qkv(5000 + seed, B, total, Hq, Hkv, D, q_gain=c["q_gain"])
    max_chunk = max(b - a for a, b in zip(c["cuts"][:-1], c["cuts"][1:]))
    if c["layout"] == "mixed":
        st = H.Stack(1, Hq, Hkv, D, B, total, S, W, max_chunk=max_chunk, layout=zb.ZZ_MIXED,
                     kvhead_is_streaming=c["mask"][None, :], poison_arena=True)
        kinds = c["mask"].astype(bool)
    else:
        st = H.Stack(1, Hq, Hkv, D, B, total, S, W, max_chunk=max_chunk,
                     layer_is_streaming=[int(c["layout"] == "streaming")], poison_arena=True)
        kinds = np.full(Hkv, c["layout"] == "streaming")
    st.workspace.fill_(0xFF)
    qd, kd, vd = H.to_dev_bf16(q), H.to_dev_bf16(k), H.to_dev_bf16(v)
    want = O.attention(q, k, v, kinds, S, W)          # every row of the whole sequence, once
    # chunked prefill
    outs = []
    for a, b in zip(c["cuts"][:-1], c["cuts"][1:]):
        qa, ka, va = qd[:, a:b].contiguous(), kd[:, a:b].contiguous(), vd[:, a:b].contiguous()
        outs.append(H.from_dev(st.prefill(0, qa, ka, va)))
        st.append(0, ka, va)
    got = np.concatenate(outs, axis=1)
    check(got, want[:, :T], ("prefill", c))
    assert np.abs(got - want[:, :T]).reshape(B, T, -1).max(axis=2).max() <= MAX_ABS
    # decode: fused steps, then append + attention
    for t in range(T, T + steps):
        out = st.decode_step(0, qd[:, t].contiguous(), kd[:, t:t + 1].contiguous(), vd[:, t:t + 1].contiguous())
        check(H.from_dev(out), want[:, t], ("decode_step", t, c))
    for t in range(T + steps, total):
        st.append(0, kd[:, t:t + 1].contiguous(), vd[:, t:t + 1].contiguous())
        check(H.from_dev(st.decode(0, qd[:, t].contiguous())), want[:, t], ("append + decode", t, c))
    assert st.ctx.layer_len(0) == total
    # the cache, bit for bit
    arena = st.arena_host()
    for g in sorted({0, Hkv - 1}):
        cap = O.cache_capacity(bool(kinds[g]), S, W, total)
        for which, X in ((0, k), (1, v)):
            img, valid = O.expected_cache(zz_inputs.bf16_bits(X), total, bool(kinds[g]), S, W, cap)
            slots = np.flatnonzero(valid)
            for b in sorted({0, B - 1}):
                assert np.array_equal(st.read_cache_rows(arena, 0, which, b, g, slots), img[b, g, slots]), (c, g, which, b)
