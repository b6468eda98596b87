"""GPU parity: every entry point of libzz.so against the fp64 oracle, element by
element, on the same seeded inputs.  Floating point bar (bf16 inputs, fp32
accumulation): max-abs <= 2e-2 and relative L2 <= 5e-3 per call; cache contents
bit-exact."""
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
    return max_abs, rel


def kinds_of(layer_streaming, Hkv):
    return np.full(Hkv, bool(layer_streaming))


# ---------------------------------------------------------------------------
# append / evict: bit-exact cache contents
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("pattern", ["one_by_one", "big_chunks", "straddle"])
def test_append_cache_is_bit_exact(D, pattern):
    H, zb = _harness()
    S, W, B, Hq, Hkv = 16, 64, 2, 4, 2
    T = 300
    _, k, v = zz_inputs.make_qkv(21, B, T, Hq, Hkv, D)
    st = H.Stack(2, Hq, Hkv, D, B, 320, S, W, layer_is_streaming=[0, 1], poison_arena=True)
    kd, vd = H.to_dev_bf16(k), H.to_dev_bf16(v)
    if pattern == "one_by_one":
        cuts = list(range(0, 150)) + [150]
        T = 150
    elif pattern == "big_chunks":          # chunks longer than the ring: only the survivors are written
        cuts = [0, 200, 300]
    else:                                  # chunks that straddle the sink edge and wrap the ring
        cuts = [0, 10, 23, 24, 90, 91, 171, 300]
    for a, b in zip(cuts[:-1], cuts[1:]):
        for layer in (0, 1):
            st.append(layer, kd[:, a:b].contiguous(), vd[:, a:b].contiguous())
        n = b
        arena = st.arena_host()
        for layer, streaming in ((0, False), (1, True)):
            assert st.ctx.layer_len(layer) == n
            cap = O.cache_capacity(streaming, S, W, 320)
            if pattern == "one_by_one" and n % 37 and n not in (1, 16, 17, 80, 81, 150):
                continue
            for which, X in ((0, k), (1, v)):
                img, valid = O.expected_cache(zz_inputs.bf16_bits(X), n, streaming, S, W, cap)
                slots = np.flatnonzero(valid)
                for bb in range(B):
                    for g in range(Hkv):
                        got = st.read_cache_rows(arena, layer, which, bb, g, slots)
                        assert np.array_equal(got, img[bb, g, slots]), (pattern, layer, which, n, bb, g)


# ---------------------------------------------------------------------------
# decode
# ---------------------------------------------------------------------------

def run_decode_case(B, Hq, Hkv, D, S, W, T, seed, streaming, q_gain=1.0, splits=None, one_by_one_tail=0,
                    layout_mixed=None, skew=None):
    """Fill a 1-layer cache with T tokens, decode the newest position, compare."""
    H, zb = _harness()
    q, k, v = zz_inputs.make_qkv(seed, B, T, Hq, Hkv, D, q_gain=q_gain)
    if layout_mixed is None:
        st = H.Stack(1, Hq, Hkv, D, B, T + 8, S, W, layer_is_streaming=[int(streaming)], poison_arena=True)
        kinds = kinds_of(streaming, Hkv)
    else:
        st = H.Stack(1, Hq, Hkv, D, B, T + 8, S, W, layout=zb.ZZ_MIXED,
                     kvhead_is_streaming=np.asarray(layout_mixed, np.uint8)[None, :], poison_arena=True)
        kinds = np.asarray(layout_mixed, bool)
    if splits is not None:
        st.ctx.tune(zb.TUNE_DECODE_SPLITS, splits)
    if skew is not None:
        st.ctx.tune(zb.TUNE_DECODE_XCD_SKEW, skew)
    kd, vd = H.to_dev_bf16(k), H.to_dev_bf16(v)
    bulk = T - one_by_one_tail
    if bulk:
        st.append(0, kd[:, :bulk].contiguous(), vd[:, :bulk].contiguous())
    for t in range(bulk, T):
        st.append(0, kd[:, t:t + 1].contiguous(), vd[:, t:t + 1].contiguous())
    out = st.decode(0, H.to_dev_bf16(q[:, T - 1]))
    got = H.from_dev(out)
    want = O.decode_row(q[:, T - 1], k, v, T - 1, kinds, S, W)
    return check(got, want, dict(B=B, Hq=Hq, Hkv=Hkv, D=D, S=S, W=W, T=T, streaming=streaming, splits=splits))


@pytest.mark.parametrize("streaming", [False, True])
@pytest.mark.parametrize("T", [1, 2, 15, 16, 17, 31, 32, 33, 79, 80, 81, 128, 1000, 1032])
def test_decode_tiny_shape_every_length(streaming, T):
    run_decode_case(1, 4, 2, 64, 16, 64, T, 100 + T, streaming)


@pytest.mark.parametrize("streaming", [False, True])
@pytest.mark.parametrize("splits", [None, 1, 3, 7, 128])
def test_decode_llama_shape_ragged_tail_across_split_counts(streaming, splits):
    # 3333 tokens = 104 full tiles + 5 slots; several tiles per wave and a ragged tail
    run_decode_case(2, 32, 8, 128, 64, 256, 3333, 7, streaming, splits=splits)


@pytest.mark.parametrize("splits", [2, 3, 7, 8, 33])
@pytest.mark.parametrize("skew", [50, 200])
def test_decode_uneven_split_ranges_cover_the_cache_exactly_once(splits, skew):
    """Neighbouring splits may share their two ranges unevenly (the split on an even XCD takes more tiles): odd
    and even split counts, a last split shorter than the others, skews of 5 % and 20 % of a split, odd and
    even numbers of (head, sequence) units before a unit (which decides which neighbour is the long one), a
    ragged last tile, and the fused append landing in a lengthened or a shortened range."""
    for B, T in ((2, 3333), (3, 2048 + 17)):
        run_decode_case(B, 32, 8, 128, 64, 256, T, 70 + splits, False, splits=splits, skew=skew)
    H, zb = _harness()
    B, Hq, Hkv, D, S, W, T = 3, 8, 2, 128, 64, 256, 1500
    q, k, v = zz_inputs.make_qkv(71, B, T + 40, Hq, Hkv, D)
    st = H.Stack(1, Hq, Hkv, D, B, T + 48, S, W, layer_is_streaming=[0], poison_arena=True)
    st.ctx.tune(zb.TUNE_DECODE_SPLITS, splits)
    st.ctx.tune(zb.TUNE_DECODE_XCD_SKEW, skew)
    kd, vd = H.to_dev_bf16(k), H.to_dev_bf16(v)
    st.append(0, kd[:, :T].contiguous(), vd[:, :T].contiguous())
    for t in range(T, T + 40):
        got = H.from_dev(st.decode_step(0, H.to_dev_bf16(q[:, t]), kd[:, t:t + 1].contiguous(), vd[:, t:t + 1].contiguous()))
        check(got, O.decode_row(q[:, t], k, v, t, kinds_of(False, Hkv), S, W), ("uneven ranges, fused append", splits, skew, t))


def test_decode_split_merge_is_race_free_with_far_more_workgroups_than_cus():
    """The workgroup that finishes last merges the split-K partials of its unit.  With
    64 units x 128 splits (8192 workgroups) and fresh queries on every launch, a merge
    that read a partial too early or stale would disagree with the unsplit result."""
    H, zb = _harness()
    B, Hq, Hkv, D, S, W, T = 8, 32, 8, 128, 64, 256, 4096
    q, k, v = zz_inputs.make_qkv(61, B, T, Hq, Hkv, D)
    st = H.Stack(1, Hq, Hkv, D, B, T, S, W, layer_is_streaming=[0], poison_arena=True)
    st.append(0, H.to_dev_bf16(k), H.to_dev_bf16(v))
    qs = H.to_dev_bf16(q[:, :60].transpose(1, 0, 2, 3).copy())          # 60 different query sets [60,B,Hq,D]
    outs = {}
    for splits in (1, 128):
        st.ctx.tune(zb.TUNE_DECODE_SPLITS, splits)
        assert st.ctx.decode_plan(0, 0)[0] == splits
        o = torch.empty_like(qs)
        for rep in range(3):
            for i in range(qs.shape[0]):
                st.decode(0, qs[i], o[i])
        outs[splits] = H.from_dev(o)
    for i in range(qs.shape[0]):
        check(outs[128][i], outs[1][i], ("split merge", i))
    want = O.decode_row(q[:, 7], k, v, T - 1, kinds_of(False, Hkv), S, W)
    check(outs[128][7], want, "split merge vs oracle")


def test_decode_split_merge_stress_every_launch_checked_against_itself_unsplit():
    """Second guard for the ordering of the cross-workgroup merge (partials stored device-coherently,
    each wave waiting for its stores before the workgroup is counted in): 600 launches over changing
    split counts, workgroups per compute unit and queries, on a small cache (so that launches are
    short and the merge is most of each), every output compared on the device with the unsplit result of
    the same query, stopping at the first mismatch.  The merge is deterministic for a given split count,
    and differs from the unsplit sum only by rounding: any larger difference is a stale or early read."""
    H, zb = _harness()
    B, Hq, Hkv, D, S, W, T = 4, 32, 8, 128, 64, 256, 2048
    q, k, v = zz_inputs.make_qkv(62, B, T, Hq, Hkv, D)
    st = H.Stack(1, Hq, Hkv, D, B, T, S, W, layer_is_streaming=[0], poison_arena=True)
    st.append(0, H.to_dev_bf16(k), H.to_dev_bf16(v))
    qs = H.to_dev_bf16(q[:, :200].transpose(1, 0, 2, 3).copy())
    st.ctx.tune(zb.TUNE_DECODE_SPLITS, 1)
    ref = torch.empty_like(qs)
    for i in range(qs.shape[0]):
        st.decode(0, qs[i], ref[i])
    ref = ref.float()
    scale = ref.abs().max().item()
    launches = 0
    for splits, wg_per_cu in ((64, 1), (7, 1), (33, 4), (2, 1), (61, 2), (16, 8)):
        st.ctx.tune(zb.TUNE_DECODE_SPLITS, splits)
        st.ctx.tune(zb.TUNE_DECODE_WG_PER_CU, wg_per_cu)
        o = torch.empty_like(qs[:100])
        for i in range(100):
            st.decode(0, qs[(i * 7 + splits) % 200], o[i])
        torch.cuda.synchronize()
        for i in range(100):
            d = (o[i].float() - ref[(i * 7 + splits) % 200]).abs().max().item()
            assert d <= 2.0 ** -7 * scale, ("first mismatch", splits, wg_per_cu, i, d, scale)
        launches += 100
    assert launches == 600


@pytest.mark.parametrize("D,Hq,Hkv", [(64, 4, 2), (128, 32, 8), (128, 4, 4)])
def test_decode_step_equals_append_then_decode(D, Hq, Hkv):
    """zz_decode_step (append fused into the attention launch) against the two-call
    sequence: same outputs bit for bit, same cache bytes, and both match the oracle.
    Lengths cross a tile start, the sink edge and several ring wraps."""
    H, zb = _harness()
    S, W, B = 16, 64, 2
    T0, steps = 60, 120                       # 60 -> 180 tokens: the ring (64 slots) wraps, tiles start at 64, 96, ...
    T = T0 + steps
    q, k, v = zz_inputs.make_qkv(71 + D, B, T, Hq, Hkv, D)
    qd, kd, vd = H.to_dev_bf16(q), H.to_dev_bf16(k), H.to_dev_bf16(v)
    stacks = [H.Stack(2, Hq, Hkv, D, B, T, S, W, layer_is_streaming=[0, 1], poison_arena=True) for _ in range(2)]
    for st in stacks:
        for layer in (0, 1):
            st.append(layer, kd[:, :T0].contiguous(), vd[:, :T0].contiguous())
    want = {layer: O.attention_layer(q, k, v, bool(layer), S, W, rows=range(T0, T)) for layer in (0, 1)}
    for t in range(T0, T):
        kt, vt, qt = kd[:, t:t + 1].contiguous(), vd[:, t:t + 1].contiguous(), qd[:, t].contiguous()
        for layer in (0, 1):
            fused = H.from_dev(stacks[0].decode_step(layer, qt, kt, vt))
            stacks[1].append(layer, kt, vt)
            two = H.from_dev(stacks[1].decode(layer, qt))
            assert np.array_equal(fused, two), (layer, t)
            check(fused, want[layer][:, t - T0], ("decode_step", layer, t))
            assert stacks[0].ctx.layer_len(layer) == t + 1
        if t in (T0, 63, 64, 79, 80, 81, 143, 144, T - 1):
            a0, a1 = stacks[0].arena_host(), stacks[1].arena_host()
            for layer, streaming in ((0, False), (1, True)):
                cap = O.cache_capacity(streaming, S, W, T)
                slots = np.arange(O.n_occupied(t + 1, streaming, S, W))
                for which, X in ((0, k), (1, v)):
                    img, valid = O.expected_cache(zz_inputs.bf16_bits(X), t + 1, streaming, S, W, cap)
                    for bb in range(B):
                        for g in range(Hkv):
                            got = stacks[0].read_cache_rows(a0, layer, which, bb, g, slots)
                            assert np.array_equal(got, img[bb, g, slots]), (layer, which, t, bb, g)
                            assert np.array_equal(got, stacks[1].read_cache_rows(a1, layer, which, bb, g, slots))


def test_decode_step_from_empty_cache_and_with_many_splits():
    H, zb = _harness()
    B, Hq, Hkv, D, S, W, T = 1, 8, 2, 128, 4, 8, 700
    q, k, v = zz_inputs.make_qkv(81, B, T, Hq, Hkv, D)
    qd, kd, vd = H.to_dev_bf16(q), H.to_dev_bf16(k), H.to_dev_bf16(v)
    st = H.Stack(2, Hq, Hkv, D, B, T, S, W, layer_is_streaming=[0, 1], poison_arena=True)
    st.ctx.tune(zb.TUNE_DECODE_SPLITS, 5)
    for layer in (0, 1):
        want = O.attention_layer(q, k, v, bool(layer), S, W)
        for t in range(T):                      # every token enters through the fused step, the first into an empty layer
            got = H.from_dev(st.decode_step(layer, qd[:, t].contiguous(), kd[:, t:t + 1].contiguous(),
                                            vd[:, t:t + 1].contiguous()))
            if t < 40 or t % 31 == 0 or t == T - 1:
                check(got, want[:, t], ("decode_step from empty", layer, t))


@pytest.mark.parametrize("Hq,Hkv", [(8, 8), (16, 2), (32, 2), (6, 2)])
def test_decode_group_sizes(Hq, Hkv):
    # G = 1 (MHA), 8, 16 (the widest column block) and a non-power-of-two group
    run_decode_case(2, Hq, Hkv, 128, 8, 40, 700, 31, False)
    run_decode_case(2, Hq, Hkv, 64, 8, 40, 700, 32, True, one_by_one_tail=33)


@pytest.mark.parametrize("Hq,Hkv", [(16, 2), (6, 2), (32, 2), (8, 8)])
@pytest.mark.parametrize("S,W", [(32, 100), (256, 256), (256, 288)])
def test_decode_short_caches_around_the_eight_wave_kernel_limits(Hq, Hkv, S, W):
    """Unsplit caches of 5 to 16 tiles and group sizes up to 8 run with eight waves per workgroup
    (one or two tiles per wave); 17 tiles, or a group of 16, fall back to four waves.  Ring caches of
    5 (last one partial), 16 and 17 tiles, and retrieval caches of the same sizes, D = 128 and 64."""
    for D in (128, 64):
        run_decode_case(2, Hq, Hkv, D, S, W, 1000, 90 + D, True, one_by_one_tail=3)
        run_decode_case(1, Hq, Hkv, D, S, W, S + W - 1, 91 + D, False, splits=1)


def test_decode_peaked_softmax_rescales_running_max():
    for streaming in (False, True):
        run_decode_case(1, 8, 2, 128, 64, 256, 2500, 55, streaming, q_gain=8.0)


def test_decode_mixed_layout_matches_per_head_kinds():
    H, zb = _harness()
    for mask in ([1, 0, 0, 1, 1, 0, 1, 0], [0, 0, 0, 0, 0, 0, 0, 1], [1, 1, 1, 1, 1, 1, 1, 1]):
        run_decode_case(2, 32, 8, 128, 64, 256, 2000, 77, None, layout_mixed=mask)


def test_decode_one_hot_key_sees_exactly_the_mask_edges():
    """Section 3.3's two parameters on the GPU: a dominant key is returned iff it is a
    sink token or inside the window (window includes the query's own position)."""
    H, zb = _harness()
    S, W, T, D, Hq, Hkv = 16, 64, 500, 64, 4, 2
    i = T - 1
    rng = np.random.default_rng(3)
    base_q, k, v = zz_inputs.make_qkv(9, 1, T, Hq, Hkv, D)
    qv = zz_inputs.round_to_bf16(np.sign(rng.standard_normal(D)).astype(np.float32))   # |q|^2 = D exactly
    for jstar in (0, S - 1, S, i - W, i - W + 1, i):
        kk = np.zeros_like(k)
        kk[0, jstar, :, :] = 48.0 * qv          # scale * q.k = 48 * 64 / 8 = 384: dominant
        qq = np.zeros((1, Hq, D), np.float32)
        qq[0, :, :] = qv
        st = H.Stack(1, Hq, Hkv, D, 1, T, S, W, layer_is_streaming=[1], poison_arena=True)
        st.append(0, H.to_dev_bf16(kk), H.to_dev_bf16(v))
        got = H.from_dev(st.decode(0, H.to_dev_bf16(qq)))
        visible = jstar < S or i - jstar < W
        want = O.decode_row(qq, kk, v, i, kinds_of(True, Hkv), S, W)
        check(got, want, ("one-hot", jstar))
        for h in range(Hq):
            same = np.array_equal(got[0, h], v[0, jstar, h // 2])
            assert same == visible, (jstar, h)


# ---------------------------------------------------------------------------
# prefill
# ---------------------------------------------------------------------------

def run_prefill_case(B, Hq, Hkv, D, S, W, T, chunks, seed, streaming, q_gain=1.0, layout_mixed=None):
    H, zb = _harness()
    q, k, v = zz_inputs.make_qkv(seed, B, T, Hq, Hkv, D, q_gain=q_gain)
    max_chunk = max(b - a for a, b in zip(chunks[:-1], chunks[1:]))
    if layout_mixed is None:
        st = H.Stack(1, Hq, Hkv, D, B, T, S, W, max_chunk=max_chunk, layer_is_streaming=[int(streaming)],
                     poison_arena=True)
        kinds = kinds_of(streaming, Hkv)
    else:
        st = H.Stack(1, Hq, Hkv, D, B, T, S, W, max_chunk=max_chunk, layout=zb.ZZ_MIXED,
                     kvhead_is_streaming=np.asarray(layout_mixed, np.uint8)[None, :], poison_arena=True)
        kinds = np.asarray(layout_mixed, bool)
    st.workspace.fill_(0xFF)
    qd, kd, vd = H.to_dev_bf16(q), H.to_dev_bf16(k), H.to_dev_bf16(v)
    want = O.attention(q, k, v, kinds, S, W)
    outs = []
    for a, b in zip(chunks[:-1], chunks[1:]):
        qa, ka, va = qd[:, a:b].contiguous(), kd[:, a:b].contiguous(), vd[:, a:b].contiguous()
        outs.append(H.from_dev(st.prefill(0, qa, ka, va)))
        st.append(0, ka, va)
    got = np.concatenate(outs, axis=1)
    res = check(got, want, dict(B=B, Hq=Hq, Hkv=Hkv, D=D, S=S, W=W, T=T, chunks=chunks[:4], streaming=streaming))
    # per-row check too: a wrong row hides inside a whole-tensor norm
    err = np.abs(got - want).reshape(B, T, -1).max(axis=2)
    assert err.max() <= MAX_ABS
    return res


def cuts(T, step):
    c = list(range(0, T, step)) + [T]
    return c


@pytest.mark.parametrize("streaming", [False, True])
@pytest.mark.parametrize("chunk", [1024, 256, 100, 37])
def test_prefill_tiny_shape_one_shot_and_chunked(streaming, chunk):
    run_prefill_case(1, 4, 2, 64, 16, 64, 1024, cuts(1024, chunk), 0, streaming)


@pytest.mark.parametrize("streaming", [False, True])
def test_prefill_llama_shape_chunked_ragged(streaming):
    # chunk boundaries that are not tile multiples; S + W = 320 spans 10 tiles
    run_prefill_case(1, 32, 8, 128, 64, 256, 1500, [0, 7, 450, 451, 963, 1500], 5, streaming)


@pytest.mark.parametrize("streaming", [False, True])
@pytest.mark.parametrize("Hq,Hkv", [(32, 8), (16, 2), (32, 2)])
def test_prefill_eight_wave_and_four_wave_forms_agree_bit_for_bit(streaming, Hq, Hkv):
    """Where a KV head has an even number of head chunks (group sizes 4, 8, 16 at D = 128) the prefill
    launch puts two of them into one workgroup of eight waves that share the K/V ring and alternate
    stages (by default only when that still leaves a workgroup per compute unit; ZZ_TUNE_PREFILL_PAIRING = 2
    forces it); ZZ_TUNE_PREFILL_PAIRING = 0 keeps one chunk per four-wave workgroup.  Every wave does the
    same arithmetic on the same tiles in both forms, so the outputs must be equal bit for bit - across
    chunk sizes that give the pipelined loop 0, 1, 3 and many tiles, ragged tails and a chunk of one."""
    H, zb = _harness()
    B, D, S, W, T = 2, 128, 64, 256, 2400
    chunks = [0, 1, 70, 200, 328, 1100, 1101, 2400]
    q, k, v = zz_inputs.make_qkv(23, B, T, Hq, Hkv, D)
    qd, kd, vd = H.to_dev_bf16(q), H.to_dev_bf16(k), H.to_dev_bf16(v)
    outs = {}
    for pairing in (2, 0):
        st = H.Stack(1, Hq, Hkv, D, B, T, S, W, max_chunk=1300, layer_is_streaming=[int(streaming)], poison_arena=True)
        st.ctx.tune(zb.TUNE_PREFILL_PAIRING, pairing)
        got = []
        for a, b in zip(chunks[:-1], chunks[1:]):
            qa, ka, va = qd[:, a:b].contiguous(), kd[:, a:b].contiguous(), vd[:, a:b].contiguous()
            got.append(st.prefill(0, qa, ka, va).clone())
            st.append(0, ka, va)
        outs[pairing] = torch.cat(got, dim=1)
        del st
    assert torch.equal(outs[2].view(torch.int16), outs[0].view(torch.int16))
    want = O.attention(q, k, v, kinds_of(streaming, Hkv), S, W)
    check(H.from_dev(outs[0]), want, ("four-wave form", streaming, Hq, Hkv))


@pytest.mark.parametrize("Hq,Hkv,D", [(4, 4, 128), (2, 1, 64), (16, 2, 128), (32, 2, 64), (6, 2, 64)])
def test_prefill_group_sizes(Hq, Hkv, D):
    for streaming in (False, True):
        run_prefill_case(2, Hq, Hkv, D, 5, 40, 333, [0, 100, 333], 17, streaming)


def test_prefill_peaked_softmax():
    for streaming in (False, True):
        run_prefill_case(1, 8, 2, 128, 16, 64, 600, [0, 300, 600], 23, streaming, q_gain=8.0)


@pytest.mark.parametrize("W", [1, 7, 40, 100])
def test_prefill_streaming_without_sink_tokens(W):
    """S = 0: nothing but the window.  A query's first visible tile may then show keys to some of
    the four key-group lanes of its column only, and columns next to it may see nothing at all yet."""
    run_prefill_case(2, 4, 1, 128, 0, W, 201, [0, 99, 145, 176, 201], 61, True)
    run_prefill_case(1, 16, 2, 64, 0, W, 137, [0, 137], 62, True)
    run_decode_case(2, 8, 2, 128, 0, W, 150, 63, True, one_by_one_tail=5)


def test_prefill_reference_maximum_is_the_maximum_over_all_key_groups():
    """Keys whose slot falls in key group 0 of a tile score 2^-196 of the others' 2^+196 (log2
    units): a reference maximum taken from one key group instead of the whole column is off by
    2^392 and overflows; the true maximum gives the mean of V over the high-scoring keys."""
    H, zb = _harness()
    D, T = 64, 200
    q = np.zeros((1, T, 1, D), np.float32)
    k = np.zeros((1, T, 1, D), np.float32)
    _, _, v = zz_inputs.make_qkv(77, 1, T, 1, 1, D)
    q[..., 0] = 32.0
    for j in range(T):
        k[0, j, 0, 0] = -34.0 if (j % 16) // 4 == 0 else 34.0      # score * scale * log2(e) = -+196
    for streaming, S, W in ((False, 0, 1), (True, 0, 50), (True, 3, 20)):
        st = H.Stack(1, 1, 1, D, 1, T + 1, S, W, max_chunk=T, layer_is_streaming=[int(streaming)], poison_arena=True)
        qd, kd, vd = H.to_dev_bf16(q), H.to_dev_bf16(k), H.to_dev_bf16(v)
        got = H.from_dev(st.prefill(0, qd[:, :150].contiguous(), kd[:, :150].contiguous(), vd[:, :150].contiguous()))
        want = O.attention(q, k, v, kinds_of(streaming, 1), S, W)
        check(got, want[:, :150], ("prefill", streaming, S, W))
        st.append(0, kd[:, :150].contiguous(), vd[:, :150].contiguous())
        got = H.from_dev(st.prefill(0, qd[:, 150:].contiguous(), kd[:, 150:].contiguous(), vd[:, 150:].contiguous()))
        check(got, want[:, 150:], ("prefill, second chunk", streaming, S, W))
        st.append(0, kd[:, 150:].contiguous(), vd[:, 150:].contiguous())
        check(H.from_dev(st.decode(0, qd[:, T - 1].contiguous())), want[:, T - 1], ("decode", streaming, S, W))


def test_prefill_mixed_layout_equals_zigzag_where_masks_coincide():
    """Section 3.2: the method leaves prefilling unchanged; a mixed layer whose heads
    are all one kind must give what the zigzag layer of that kind gives."""
    run_prefill_case(1, 16, 4, 128, 16, 64, 500, [0, 200, 500], 41, None, layout_mixed=[1, 0, 0, 1])
    H, zb = _harness()
    q, k, v = zz_inputs.make_qkv(43, 1, 400, 8, 2, 64)
    outs = {}
    for name, kw in (("zig", dict(layer_is_streaming=[1])),
                     ("mix", dict(layout=zb.ZZ_MIXED, kvhead_is_streaming=np.ones((1, 2), np.uint8)))):
        st = H.Stack(1, 8, 2, 64, 1, 400, 16, 64, max_chunk=400, **kw)
        outs[name] = H.from_dev(st.prefill(0, H.to_dev_bf16(q), H.to_dev_bf16(k), H.to_dev_bf16(v)))
    assert np.array_equal(outs["zig"], outs["mix"])


# ---------------------------------------------------------------------------
# the tiny stack end to end: prefill 1024, then 8 decode steps, both layers
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("seed", [0, 1, 2])
def test_tiny_stack_prefill_then_decode(seed):
    H, zb = _harness()
    w = zz_inputs.WORKLOADS["c1_tiny"]
    T = w.context + w.decode_steps
    st = H.Stack(w.n_layers, w.n_q_heads, w.n_kv_heads, w.head_dim, w.batch, T, w.sink, w.window,
                 max_chunk=w.chunk, layer_is_streaming=[0, 1], poison_arena=True)
    for layer, streaming in ((0, False), (1, True)):
        q, k, v = zz_inputs.make_qkv(1000 * seed + layer, w.batch, T, w.n_q_heads, w.n_kv_heads, w.head_dim)
        want = O.attention_layer(q, k, v, streaming, w.sink, w.window)
        qd, kd, vd = H.to_dev_bf16(q), H.to_dev_bf16(k), H.to_dev_bf16(v)
        n0 = w.context
        got = [H.from_dev(st.prefill(layer, qd[:, :n0].contiguous(), kd[:, :n0].contiguous(), vd[:, :n0].contiguous()))]
        st.append(layer, kd[:, :n0].contiguous(), vd[:, :n0].contiguous())
        assert st.ctx.layer_launches(layer) == 1
        for t in range(n0, T):
            st.append(layer, kd[:, t:t + 1].contiguous(), vd[:, t:t + 1].contiguous())
            got.append(H.from_dev(st.decode(layer, qd[:, t].contiguous()))[:, None])
            check(got[-1][:, 0], want[:, t], ("decode step", layer, t))      # decode step t == row t
        check(np.concatenate(got, axis=1), want, ("tiny stack", layer, seed))


# ---------------------------------------------------------------------------
# full size, in the launch configuration the benchmark times: sampled units
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("wname", ["c3_llama8b_128k_b4", "c2_llama8b_32k_b1", "c5_mha7b_32k_b8"])
def test_decode_full_size_sampled_units(wname):
    """One retrieval and one streaming layer of each decode workload at its full size (128k /
    batch 4; 32k / batch 1; 32k / batch 8 with 32 KV heads), filled through zz_kv_append, in the
    launch configuration the benchmark times; the oracle recomputes sampled (batch, kv head) units."""
    H, zb = _harness()
    w = zz_inputs.WORKLOADS[wname]
    B, Hq, Hkv, D, N = w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.context
    G = Hq // Hkv
    st = H.Stack(2, Hq, Hkv, D, B, N, w.sink, w.window, layer_is_streaming=[0, 1])
    gen = torch.Generator(device="cuda").manual_seed(1234)
    sample = sorted({(0, 0), (0, 5), (B - 1, Hkv - 1), (B // 2, 3), (min(1, B - 1), 2)})
    kept = {u: ([], []) for u in sample}
    chunk = 8192
    for a in range(0, N, chunk):
        kc = torch.randn((B, chunk, Hkv, D), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        vc = torch.randn((B, chunk, Hkv, D), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        for layer in (0, 1):
            st.append(layer, kc, vc)
        for (b, g) in sample:
            kept[(b, g)][0].append(kc[b, :, g].float().cpu().numpy())
            kept[(b, g)][1].append(vc[b, :, g].float().cpu().numpy())
    q = torch.randn((B, Hq, D), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    qh = q.float().cpu().numpy()
    scale = O.default_scale(D)
    for layer, streaming in ((0, False), (1, True)):
        got = H.from_dev(st.decode(layer, q))
        J = O.attended_positions(N - 1, streaming, w.sink, w.window)
        for (b, g) in sample:
            K = np.concatenate(kept[(b, g)][0])[J]
            V = np.concatenate(kept[(b, g)][1])[J]
            want = O.decode_unit(qh[b, g * G:(g + 1) * G], K, V, scale)
            check(got[b, g * G:(g + 1) * G], want, (wname, layer, b, g))
        assert np.isfinite(got).all()
    if B < 4:
        return
    # The same caches read as sequences of different lengths, in one launch per layer (the
    # configuration `bench.py --workload unequal` times).  A retrieval cache of n tokens is
    # the first n slots of the longer one; a full streaming cache holds S + W tokens whatever
    # the length, and decode attends all of them, so its outputs must not change.
    lens = ([N, N // 2, N // 4 + 5, N // 8] * B)[:B]
    for layer, streaming in ((0, False), (1, True)):
        for b, n in enumerate(lens):
            st.ctx.set_seq_len(layer, b, n)
        got = H.from_dev(st.decode(layer, q))
        for (b, g) in sample:
            J = O.attended_positions(N - 1, True, w.sink, w.window) if streaming else np.arange(lens[b])
            K = np.concatenate(kept[(b, g)][0])[J]
            V = np.concatenate(kept[(b, g)][1])[J]
            want = O.decode_unit(qh[b, g * G:(g + 1) * G], K, V, scale)
            check(got[b, g * G:(g + 1) * G], want, (wname, "unequal lengths", layer, b, g))
        assert np.isfinite(got).all()


def test_prefill_full_size_last_chunk_of_64k_sampled_rows():
    """The chunked-prefill workload's heaviest launch, in the configuration the benchmark
    times: 61440 cached tokens + a 4096-token chunk, Llama-3-8B shape, one retrieval and one
    streaming layer; the oracle recomputes sampled (row, head) outputs."""
    H, zb = _harness()
    w = zz_inputs.WORKLOADS["c4_prefill_64k"]
    B, Hq, Hkv, D, T, C = w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.context, w.chunk
    G = Hq // Hkv
    st = H.Stack(2, Hq, Hkv, D, B, T, w.sink, w.window, max_chunk=C, layer_is_streaming=[0, 1], poison_arena=True)
    gen = torch.Generator(device="cuda").manual_seed(4321)
    kh = np.empty((T, Hkv, D), np.float32)
    vh = np.empty((T, Hkv, D), np.float32)
    n_past = T - C
    for a in range(0, T, C):
        kc = torch.randn((B, C, Hkv, D), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        vc = torch.randn((B, C, Hkv, D), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        kh[a:a + C], vh[a:a + C] = kc[0].float().cpu().numpy(), vc[0].float().cpu().numpy()
        if a < n_past:
            for layer in (0, 1):
                st.append(layer, kc, vc)
    q = torch.randn((B, C, Hq, D), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    qh = q[0].float().cpu().numpy()
    scale = O.default_scale(D)
    rows = [0, 1, 15, 16, 31, 32, 63, 64, 1000, 2047, 2048, 4000, C - 2, C - 1]
    heads = [0, 5, 17, Hq - 1]
    for layer, streaming in ((0, False), (1, True)):
        got = H.from_dev(st.prefill(layer, q, kc, vc))[0]
        assert np.isfinite(got).all()
        for r in rows:
            J = O.attended_positions(n_past + r, streaming, w.sink, w.window)
            for h in heads:
                want = O.attention_row(qh[r, h], kh[J, h // G], vh[J, h // G], scale)
                check(got[r, h], want, ("64k prefill", layer, r, h))


@pytest.mark.parametrize("lengths", ["equal", "unequal"])
def test_decode_step_captured_in_a_hip_graph_replays_identically(lengths):
    """A whole-stack decode step (one zz_decode_step per layer) captured into a HIP graph:
    every replay, with eager launches and synchronisations in between, must reproduce the
    eager result (the library records kernels only: no memset nodes, no allocations).  Also
    with the two sequences at different lengths (the launch over unequal lengths)."""
    H, zb = _harness()
    L, B, Hq, Hkv, D, S, W, T = 4, 2, 8, 2, 128, 16, 64, 900
    st = H.Stack(L, Hq, Hkv, D, B, T + 4, S, W, layer_is_streaming=[0, 1, 1, 0], poison_arena=True)
    q, k, v = zz_inputs.make_qkv(91, B, T + 1, Hq, Hkv, D)
    qd, kd, vd = H.to_dev_bf16(q), H.to_dev_bf16(k), H.to_dev_bf16(v)
    for l in range(L):
        st.append(l, kd[:, :T].contiguous(), vd[:, :T].contiguous())
    qs = torch.stack([qd[:, T].contiguous() for _ in range(L)])
    k1, v1 = kd[:, T:T + 1].contiguous(), vd[:, T:T + 1].contiguous()
    out = torch.zeros_like(qs)

    def step():
        for l in range(L):
            st.ctx.set_layer_len(l, T)
            if lengths == "unequal":
                st.ctx.set_seq_len(l, 1, T - 300)   # a prefix of the same cache
            st.ctx.decode_step(l, qs[l], k1, v1, out[l], st.stream_ptr())

    step()                                   # eager (also clears the split counters outside any capture)
    torch.cuda.synchronize()
    eager = out.clone()
    want0 = O.decode_row(q[:, T], k, v, T, kinds_of(False, Hkv), S, W)
    want1 = O.decode_row(q[:, T], k, v, T, kinds_of(True, Hkv), S, W)
    n_seq = 2 if lengths == "equal" else 1      # sequence 1 of the unequal case is compared with the eager run only
    check(H.from_dev(eager[0])[:n_seq], want0[:n_seq], "eager retrieval layer")
    check(H.from_dev(eager[1])[:n_seq], want1[:n_seq], "eager streaming layer")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    for rep in range(4):
        out.zero_()
        scratch = torch.randn(1 << 20, device="cuda").sum().item()     # the program's own eager work in between
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), rep
        step()                                                          # an eager step between replays
        torch.cuda.synchronize()
        assert torch.equal(out, eager), rep


def test_first_decode_of_a_context_recorded_into_a_graph_then_eager_then_replayed():
    """The split counters sit in caller memory the library has never cleared.  When the very first
    decode call of a context is recorded into a HIP graph, the clear it enqueues runs only on
    replay: an eager call made before any replay must clear them itself.  Workspace filled with
    a non-zero pattern; capture, eager, replay, eager - each against the oracle row."""
    H, zb = _harness()
    B, Hq, Hkv, D, S, W, T = 2, 8, 2, 128, 16, 64, 3000
    q, k, v = zz_inputs.make_qkv(77, B, T, Hq, Hkv, D)
    st = H.Stack(1, Hq, Hkv, D, B, T, S, W, layer_is_streaming=[0], poison_arena=True)
    st.workspace.fill_(0x5A)
    st.append(0, H.to_dev_bf16(k), H.to_dev_bf16(v))
    assert st.ctx.decode_plan(0, 0)[0] > 1          # the launch really merges across workgroups
    qd = H.to_dev_bf16(q[:, T - 1])
    out = torch.zeros_like(qd)
    want = O.decode_row(q[:, T - 1], k, v, T - 1, kinds_of(False, Hkv), S, W)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        st.ctx.attn_decode(0, qd, out, st.stream_ptr())
    for what in ("eager before any replay", "replay", "eager", "replay"):
        out.zero_()
        if what.startswith("eager"):
            st.ctx.attn_decode(0, qd, out, st.stream_ptr())
        else:
            g.replay()
        torch.cuda.synchronize()
        check(H.from_dev(out), want, what)


def test_uniform_keys_give_the_mean_over_exactly_the_attended_set_on_gpu():
    """Closed form on the GPU path itself (no oracle involved): with K = 0 every visible key
    gets the same weight, so the output is the mean of V over the attended set.  V encodes
    the key's position in bf16-exact integers, so the means tell which positions were used:
    streaming: {0..S-1} U {i-W+1..i}; retrieval: {0..i}.  Decode at 32k, prefill rows beside it."""
    H, zb = _harness()
    S, W, B, Hq, Hkv, D, T = 64, 256, 1, 8, 2, 128, 32768
    k = np.zeros((B, T, Hkv, D), np.float32)
    v = np.zeros((B, T, Hkv, D), np.float32)
    j = np.arange(T)
    v[0, :, :, 0] = 1.0
    v[0, :, :, 1] = (j % 256)[:, None]
    v[0, :, :, 2] = (j // 256)[:, None]
    q = zz_inputs.make_qkv(3, B, T, Hq, Hkv, D)[0]
    C = 512
    st = H.Stack(2, Hq, Hkv, D, B, T, S, W, max_chunk=C, layer_is_streaming=[0, 1], poison_arena=True)
    kd, vd, qd = H.to_dev_bf16(k), H.to_dev_bf16(v), H.to_dev_bf16(q)
    n_past = T - C
    for layer in (0, 1):
        st.append(layer, kd[:, :n_past].contiguous(), vd[:, :n_past].contiguous())

    def expect(i, streaming):
        A = np.concatenate([np.arange(min(S, i + 1)), np.arange(max(S, i - W + 1), i + 1)]) if streaming else np.arange(i + 1)
        return np.array([1.0, (A % 256).mean(), (A // 256).mean()])

    for layer, streaming in ((0, False), (1, True)):
        pre = H.from_dev(st.prefill(layer, qd[:, n_past:].contiguous(), kd[:, n_past:].contiguous(),
                                    vd[:, n_past:].contiguous()))
        for r in (0, 1, 31, 32, 255, 256, 300, C - 1):
            want = expect(n_past + r, streaming)
            for h in (0, Hq - 1):
                assert np.allclose(pre[0, r, h, :3], want, rtol=2 ** -7, atol=1e-6), (layer, r, h, pre[0, r, h, :3], want)
        st.append(layer, kd[:, n_past:].contiguous(), vd[:, n_past:].contiguous())
        dec = H.from_dev(st.decode(layer, qd[:, T - 1].contiguous()))
        want = expect(T - 1, streaming)
        assert np.allclose(dec[0, :, :3], want[None, :], rtol=2 ** -7, atol=1e-6), (layer, dec[0, 0, :3], want)
        assert np.abs(dec[0, :, 3:]).max() == 0.0
