"""Rotary position encoding of K at append (zz_set_rope_tables) against the fp64 rotation oracle:
the cache must hold the rotated rows (computed in fp32 on the GPU, in fp64 by the oracle, both
rounded to bf16: at most one bf16 unit apart, and equal almost everywhere), V untouched; prefill
and decode attend the rotated keys.  Tables of random angles (any rotation is a valid input) and,
once, the geometric frequencies a Llama model uses."""
import numpy as np
import pytest

import zz_inputs
from oracle import zz_oracle as O
from oracle import zz_rope_oracle as R

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

MAX_ABS, REL_L2 = 2e-2, 5e-3


def check(got, want, what):
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    assert got.shape == want.shape and np.isfinite(got).all(), what
    max_abs = np.abs(got - want).max()
    rel = np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-300)
    assert max_abs <= MAX_ABS and rel <= REL_L2, (what, max_abs, rel)


def tables(seed, rows, half, llama=False):
    if llama:
        ang = np.arange(rows)[:, None] * (500000.0 ** (-np.arange(half) / half))[None, :]
    else:
        ang = np.random.default_rng(seed).uniform(-np.pi, np.pi, size=(rows, half))
    cos, sin = np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)
    dev = lambda a: torch.from_numpy(a).to("cuda").contiguous()
    return cos, sin, dev(cos), dev(sin)


def bf16_close(got_bits, want_f64, what):
    """got: uint16 bf16 patterns; want: fp64 values.  Equal to the nearest-even rounding of want almost
    everywhere, never more than one bf16 unit away."""
    want_bits = zz_inputs.bf16_bits(zz_inputs.round_to_bf16(want_f64.astype(np.float32)))
    got_f = zz_inputs.bf16_bits_to_f32(got_bits).astype(np.float64)
    ulp = np.maximum(np.abs(want_f64), 2.0 ** -126) * 2.0 ** -7          # one unit of a bf16 at that magnitude (upper bound)
    assert (np.abs(got_f - want_f64) <= ulp).all(), what
    frac = float((got_bits == want_bits).mean())
    assert frac >= 0.995, (what, frac)


@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("llama", [False, True])
def test_appended_keys_are_rotated_by_their_position_and_values_are_not(D, llama):
    from paper_2508_12407_amd import harness as H
    S, W, B, Hq, Hkv, T = 16, 64, 2, 4, 2, 300
    _, k, v = zz_inputs.make_qkv(31, B, T, Hq, Hkv, D)
    cos, sin, cd, sd = tables(1, T, D // 2, llama)
    st = H.Stack(2, Hq, Hkv, D, B, T, S, W, layer_is_streaming=[0, 1], poison_arena=True)
    st.ctx.set_rope_tables(cd, sd, T)
    kd, vd = H.to_dev_bf16(k), H.to_dev_bf16(v)
    cuts = [0, 1, 2, 40, 41, 171, 300]            # single tokens, tile-wise chunks, chunks past the window
    for a, b in zip(cuts[:-1], cuts[1:]):
        for layer in (0, 1):
            st.append(layer, kd[:, a:b].contiguous(), vd[:, a:b].contiguous())
    krot = R.rotate_keys(k, np.arange(T), cos, sin)
    arena = st.arena_host()
    for layer, streaming in ((0, False), (1, True)):
        cap = O.cache_capacity(streaming, S, W, T)
        want_k, valid = O.expected_cache(krot, T, streaming, S, W, cap)
        want_v, _ = O.expected_cache(zz_inputs.bf16_bits(v), T, streaming, S, W, cap)
        slots = np.flatnonzero(valid)
        for bb in range(B):
            for g in range(Hkv):
                bf16_close(st.read_cache_rows(arena, layer, 0, bb, g, slots), want_k[bb, g, slots], (D, layer, bb, g))
                assert np.array_equal(st.read_cache_rows(arena, layer, 1, bb, g, slots), want_v[bb, g, slots])


def test_prefill_and_decode_attend_rotated_keys_at_equal_and_unequal_lengths():
    from paper_2508_12407_amd import harness as H, binding as zb
    S, W, B, Hq, Hkv, D, T, C = 16, 64, 2, 8, 2, 128, 702, 256
    G = Hq // Hkv
    q, k, v = zz_inputs.make_qkv(32, B, T, Hq, Hkv, D)
    cos, sin, cd, sd = tables(2, T, D // 2)
    krot = zz_inputs.round_to_bf16(R.rotate_keys(k, np.arange(T), cos, sin).astype(np.float32))   # what the cache holds
    st = H.Stack(2, Hq, Hkv, D, B, T, S, W, max_chunk=C, layer_is_streaming=[0, 1], poison_arena=True)
    st.ctx.set_rope_tables(cd, sd, T)
    kd, vd, qd = H.to_dev_bf16(k), H.to_dev_bf16(v), H.to_dev_bf16(q)
    for layer, streaming in ((0, False), (1, True)):
        kinds = np.full(Hkv, streaming)
        for a in range(0, 600, C):                      # chunked prefill: the staged chunk is rotated too
            e = min(a + C, 600)
            out = H.from_dev(st.prefill(layer, qd[:, a:e].contiguous(), kd[:, a:e].contiguous(), vd[:, a:e].contiguous()))
            st.append(layer, kd[:, a:e].contiguous(), vd[:, a:e].contiguous())
            want = O.attention(q, krot, v, kinds, S, W, rows=list(range(a, e)))
            check(out, want, ("prefill", layer, a))
        for t in range(600, 640):                       # fused decode steps: the newest row is rotated in registers
            out = H.from_dev(st.decode_step(layer, qd[:, t].contiguous(), kd[:, t:t + 1].contiguous(), vd[:, t:t + 1].contiguous()))
            if t % 13 == 0 or t == 639:
                check(out, O.decode_row(q[:, t], krot, v, t, kinds, S, W), ("decode step", layer, t))
        # sequence 0 goes ahead alone by 30 tokens; then one batched chunk: positions 670.. for it, 640.. for sequence 1
        st.ctx.kv_append_seq(layer, 0, kd[0:1, 640:670].contiguous(), vd[0:1, 640:670].contiguous(), 30, st.stream_ptr())
        k2 = np.stack([k[0, 670:700], k[1, 640:670]])
        v2 = np.stack([v[0, 670:700], v[1, 640:670]])
        q2 = np.stack([q[0, 670:700], q[1, 640:670]])
        out = H.from_dev(st.prefill(layer, H.to_dev_bf16(q2), H.to_dev_bf16(k2), H.to_dev_bf16(v2)))
        st.append(layer, H.to_dev_bf16(k2), H.to_dev_bf16(v2))
        check(out[0:1], O.attention(q[0:1], krot[0:1], v[0:1], kinds, S, W, rows=list(range(670, 700))), ("unequal prefill", layer, 0))
        check(out[1:2], O.attention(q[1:2], krot[1:2], v[1:2], kinds, S, W, rows=list(range(640, 670))), ("unequal prefill", layer, 1))
        # a fused decode step on the unequal batch: position 700 for sequence 0, 670 for sequence 1
        k3 = np.stack([k[0, 700:701], k[1, 670:671]])
        v3 = np.stack([v[0, 700:701], v[1, 670:671]])
        q3 = np.stack([q[0, 700], q[1, 670]])
        out = H.from_dev(st.decode_step(layer, H.to_dev_bf16(q3), H.to_dev_bf16(k3), H.to_dev_bf16(v3)))
        check(out[0:1], O.decode_row(q[0:1, 700], krot[0:1], v[0:1], 700, kinds, S, W), ("unequal decode step", layer, 0))
        check(out[1:2], O.decode_row(q[1:2, 670], krot[1:2], v[1:2], 670, kinds, S, W), ("unequal decode step", layer, 1))
    # a position past the tables: refused before anything is launched; switched off: keys stored as given
    st2 = H.Stack(1, Hq, Hkv, D, B, 64, S, W, layer_is_streaming=[0], poison_arena=True)
    st2.ctx.set_rope_tables(cd, sd, 10)
    with pytest.raises(zb.ZzError) as e:
        st2.append(0, kd[:, :11].contiguous(), vd[:, :11].contiguous())
    assert e.value.code == zb.ERR["ERANGE"] and st2.ctx.layer_len(0) == 0
    st2.ctx.set_rope_tables(None, None, 0)
    st2.append(0, kd[:, :11].contiguous(), vd[:, :11].contiguous())
    img, valid = O.expected_cache(zz_inputs.bf16_bits(k), 11, False, S, W, 64)
    got = st2.read_cache_rows(st2.arena_host(), 0, 0, 1, 1, np.flatnonzero(valid))
    assert np.array_equal(got, img[1, 1, np.flatnonzero(valid)])
