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


def draw_long_case(seed):
    """As draw_case, but one sequence of 600 to 3000 tokens: several query blocks, many cached tiles."""
    c = draw_case(seed)
    r = np.random.default_rng(50000 + seed)
    c["B"] = 1
    c["Hkv"] = int(r.choice([1, 2]))
    c["Hq"] = c["Hkv"] * int(r.choice([1, 2, 4]))
    c["mask"] = (r.random(c["Hkv"]) < 0.5).astype(np.uint8)
    c["T"] = int(r.integers(600, 3000))
    n_cuts = int(r.integers(0, 5))
    c["cuts"] = sorted(set([0, c["T"]] + [int(x) for x in r.integers(1, c["T"] + 1, size=n_cuts)]))
    c["W"] = int(r.choice([1, 7, 32, 100, 256, 700]))
    return c


@pytest.mark.parametrize("seed", range(8))
def test_random_configuration_longer_contexts(seed):
    run_configuration(draw_long_case(seed), 6000 + seed)


@pytest.mark.parametrize("seed", range(36))
def test_random_configuration(seed):
    run_configuration(draw_case(seed), 5000 + seed)


def run_configuration(c, data_seed):
    H, zb = _harness()
    D, Hkv, Hq, B, S, W, T, steps = c["D"], c["Hkv"], c["Hq"], c["B"], c["S"], c["W"], c["T"], c["steps"]
    total = T + 2 * steps
    q, k, v = zz_inputs.make_qkv(data_seed, B, total, Hq, Hkv, D, q_gain=c["q_gain"])
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


def draw_decode_case(seed):
    r = np.random.default_rng(7000 + seed)
    D = int(r.choice([64, 128]))
    Hkv = int(r.choice([1, 2, 4, 8]))
    G = int(r.choice([1, 2, 4, 8, 16]))
    if Hkv * G > 32:
        G = 32 // Hkv
    B = int(r.integers(1, 6))
    S = int(r.choice([0, 1, 16, 64]))
    W = int(r.choice([1, 32, 256, 500]))
    longest = int(r.choice([40, 600, 3000, 6000]))
    if r.random() < 0.35:
        lens = [int(r.integers(1, longest + 1))] * B                 # one common length: the single-length launch
    else:
        lens = [int(r.integers(1, longest + 1)) for _ in range(B)]   # one launch over unequal lengths
    layout = str(r.choice(["retrieval", "streaming", "mixed"]))
    mask = (r.random(Hkv) < 0.5).astype(np.uint8)
    splits = [None, None, 1, 2, 5, 37, 128][int(r.integers(0, 7))]
    cus = [None, None, 8, 64, 1024][int(r.integers(0, 5))]
    return dict(D=D, Hkv=Hkv, Hq=Hkv * G, B=B, S=S, W=W, lens=lens, layout=layout, mask=mask, splits=splits, cus=cus)


@pytest.mark.parametrize("seed", range(40))
def test_random_decode_configuration(seed):
    """Caches of random (equal or unequal) lengths up to 6000 tokens, random split counts and
    compute-unit counts for the split plan; two fused steps and one append + attention."""
    H, zb = _harness()
    c = draw_decode_case(seed)
    D, Hkv, Hq, B, S, W = c["D"], c["Hkv"], c["Hq"], c["B"], c["S"], c["W"]
    G = Hq // Hkv
    lens = list(c["lens"])
    total = max(lens) + 3
    _, k, v = zz_inputs.make_qkv(9000 + seed, B, total, 1, Hkv, D)        # K, V of every sequence
    qs = zz_inputs.make_qkv(9500 + seed, B, 3, Hq, Hkv, D)[0]             # the three queries of every sequence
    if c["layout"] == "mixed":
        st = H.Stack(1, Hq, Hkv, D, B, total, S, W, layout=zb.ZZ_MIXED, kvhead_is_streaming=c["mask"][None, :],
                     poison_arena=True)
        kinds = c["mask"].astype(bool)
    else:
        st = H.Stack(1, Hq, Hkv, D, B, total, S, W, layer_is_streaming=[int(c["layout"] == "streaming")],
                     poison_arena=True)
        kinds = np.full(Hkv, c["layout"] == "streaming")
    st.workspace.fill_(0xFF)
    if c["splits"] is not None:
        st.ctx.tune(zb.TUNE_DECODE_SPLITS, c["splits"])
    if c["cus"] is not None:
        st.ctx.tune(zb.TUNE_NUM_CU, c["cus"])
    kd, vd, qd = H.to_dev_bf16(k), H.to_dev_bf16(v), H.to_dev_bf16(qs)
    sp = st.stream_ptr()
    for b, n in enumerate(lens):
        st.ctx.kv_append_seq(0, b, kd[b:b + 1, :n].contiguous(), vd[b:b + 1, :n].contiguous(), n, sp)
    scale = O.default_scale(D)

    def want_now():
        out = np.zeros((B, Hq, D))
        for b, n in enumerate(lens):
            for g in range(Hkv):
                J = O.attended_positions(n - 1, bool(kinds[g]), S, W)
                out[b, g * G:(g + 1) * G] = O.decode_unit(qs[b, step, g * G:(g + 1) * G], k[b, J, g], v[b, J, g], scale)
        return out

    for step in range(3):
        newk = torch.stack([kd[b, n] for b, n in enumerate(lens)])[:, None].contiguous()
        newv = torch.stack([vd[b, n] for b, n in enumerate(lens)])[:, None].contiguous()
        if step < 2:
            out = st.decode_step(0, qd[:, step].contiguous(), newk, newv)
        else:
            st.ctx.kv_append(0, newk, newv, 1, sp)
            out = st.decode(0, qd[:, step].contiguous())
        lens = [n + 1 for n in lens]
        check(H.from_dev(out), want_now(), ("decode", step, {k_: v_ for k_, v_ in c.items() if k_ != "mask"}))
        assert [st.ctx.seq_len(0, b) for b in range(B)] == lens
    arena = st.arena_host()
    b, g = B - 1, Hkv - 1
    cap = O.cache_capacity(bool(kinds[g]), S, W, total)
    for which, X in ((0, k), (1, v)):
        img, valid = O.expected_cache(zz_inputs.bf16_bits(X[b:b + 1]), lens[b], bool(kinds[g]), S, W, cap)
        slots = np.flatnonzero(valid)
        assert np.array_equal(st.read_cache_rows(arena, 0, which, b, g, slots), img[0, g, slots]), (c, which)


@pytest.mark.parametrize("seed", range(12))
def test_random_unequal_prompts(seed):
    """Prompts of random lengths entering a batch one sequence at a time in random chunks
    (zz_attn_prefill_seq / zz_kv_append_seq), then a batched chunk and a fused decode step on the
    unequal lengths; every sequence against the oracle on its own."""
    H, zb = _harness()
    r = np.random.default_rng(11000 + seed)
    D = int(r.choice([64, 128]))
    Hkv = int(r.choice([1, 2, 4]))
    G = int(r.choice([1, 2, 4, 8]))
    Hq = Hkv * G
    B = int(r.integers(2, 5))
    S = int(r.choice([0, 4, 16, 64]))
    W = int(r.choice([1, 32, 100, 256]))
    lens = [int(r.integers(0, 400)) for _ in range(B)]
    n_batched = int(r.integers(1, 50))
    layout = str(r.choice(["retrieval", "streaming", "mixed"]))
    mask = (r.random(Hkv) < 0.5).astype(np.uint8)
    total = max(lens) + n_batched + 1
    q, k, v = zz_inputs.make_qkv(12000 + seed, B, total, Hq, Hkv, D)
    kw = dict(layout=zb.ZZ_MIXED, kvhead_is_streaming=mask[None, :]) if layout == "mixed" else \
        dict(layer_is_streaming=[int(layout == "streaming")])
    st = H.Stack(1, Hq, Hkv, D, B, total, S, W, max_chunk=max(max(lens), n_batched, 1), poison_arena=True, **kw)
    kinds = mask.astype(bool) if layout == "mixed" else np.full(Hkv, layout == "streaming")
    st.workspace.fill_(0xFF)
    qd, kd, vd = H.to_dev_bf16(q), H.to_dev_bf16(k), H.to_dev_bf16(v)
    sp = st.stream_ptr()
    what = dict(D=D, Hq=Hq, Hkv=Hkv, B=B, S=S, W=W, lens=lens, n_batched=n_batched, layout=layout)

    def want_rows(b, a, e):
        return O.attention(q[b:b + 1, :e], k[b:b + 1, :e], v[b:b + 1, :e], kinds, S, W, rows=list(range(a, e)))

    for b, n in enumerate(lens):
        cuts = sorted(set([0, n] + [int(x) for x in r.integers(0, n + 1, size=int(r.integers(0, 4)))]))
        for a, e in zip(cuts[:-1], cuts[1:]):
            qa, ka, va = qd[b:b + 1, a:e].contiguous(), kd[b:b + 1, a:e].contiguous(), vd[b:b + 1, a:e].contiguous()
            out = torch.empty_like(qa)
            st.ctx.attn_prefill_seq(0, b, qa, ka, va, e - a, out, sp)
            check(H.from_dev(out), want_rows(b, a, e), ("prefill_seq", b, a, e, what))
            st.ctx.kv_append_seq(0, b, ka, va, e - a, sp)
    assert [st.ctx.seq_len(0, b) for b in range(B)] == lens
    qa = torch.stack([qd[b, n:n + n_batched] for b, n in enumerate(lens)]).contiguous()
    ka = torch.stack([kd[b, n:n + n_batched] for b, n in enumerate(lens)]).contiguous()
    va = torch.stack([vd[b, n:n + n_batched] for b, n in enumerate(lens)]).contiguous()
    got = H.from_dev(st.prefill(0, qa, ka, va))
    for b, n in enumerate(lens):
        check(got[b:b + 1], want_rows(b, n, n + n_batched), ("batched prefill", b, what))
    st.append(0, ka, va)
    lens = [n + n_batched for n in lens]
    out = st.decode_step(0, torch.stack([qd[b, n] for b, n in enumerate(lens)]).contiguous(),
                         torch.stack([kd[b, n] for b, n in enumerate(lens)])[:, None].contiguous(),
                         torch.stack([vd[b, n] for b, n in enumerate(lens)])[:, None].contiguous())
    got = H.from_dev(out)
    for b, n in enumerate(lens):
        check(got[b:b + 1], want_rows(b, n, n + 1)[:, 0], ("decode_step", b, what))
    assert [st.ctx.seq_len(0, b) for b in range(B)] == [n + 1 for n in lens]
