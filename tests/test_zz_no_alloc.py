"""zz_attn_decode_static (split-K scratch in the library's own static device array, nothing
allocated by the call) against zz_attn_decode (scratch in the caller's workspace): same
launches, so the outputs must be identical bit for bit, and both within the oracle's bar.
Two calls in a row share the one array: the second, on a smaller shape, must not be
disturbed by what the first left behind."""
import numpy as np
import pytest

import zz_inputs
from oracle import zz_oracle as O

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

MAX_ABS, REL_L2 = 2e-2, 5e-3


def check(got, want, what):
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    assert got.shape == want.shape and np.isfinite(got).all(), what
    max_abs = np.abs(got - want).max()
    rel = np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-300)
    assert max_abs <= MAX_ABS and rel <= REL_L2, (what, max_abs, rel)


def one_shape(B, Hq, Hkv, D, S, W, T, seed, mixed):
    from paper_2508_12407_amd import harness as H, binding as zb
    q, k, v = zz_inputs.make_qkv(seed, B, T, Hq, Hkv, D)
    if mixed:
        hmask = np.zeros((2, Hkv), np.uint8)
        hmask[:, ::2] = 1
        st = H.Stack(2, Hq, Hkv, D, B, T, S, W, layout=zb.ZZ_MIXED, kvhead_is_streaming=hmask, poison_arena=True)
        kinds = [hmask[0].astype(bool), hmask[1].astype(bool)]
    else:
        st = H.Stack(2, Hq, Hkv, D, B, T, S, W, layer_is_streaming=[0, 1], poison_arena=True)
        kinds = [np.zeros(Hkv, bool), np.ones(Hkv, bool)]
    kd, vd = H.to_dev_bf16(k), H.to_dev_bf16(v)
    qd = H.to_dev_bf16(q[:, T - 1])
    for layer in (0, 1):
        st.append(layer, kd, vd)
    assert st.ctx.decode_plan(0, 0)[0] > 1, "the retrieval launch must really use split-K partials"
    for layer in (0, 1):
        ref = torch.zeros_like(qd)
        got = torch.zeros_like(qd)
        st.ctx.attn_decode(layer, qd, ref, st.stream_ptr())
        before = torch.cuda.memory_allocated()
        st.ctx.attn_decode_static(layer, qd, got, st.stream_ptr())
        assert torch.cuda.memory_allocated() == before
        torch.cuda.synchronize()
        assert torch.equal(got, ref), (B, Hq, Hkv, D, T, layer)
        want = O.decode_row(q[:, T - 1], k, v, T - 1, kinds[layer], S, W)
        check(H.from_dev(got), want, ("static scratch", B, Hq, Hkv, D, T, layer))
    return st


def test_static_scratch_decode_equals_workspace_decode_on_two_calls_in_a_row():
    # Llama-shaped heads, several splits per unit, ragged last tile ...
    one_shape(2, 32, 8, 128, 64, 256, 5003, 5, mixed=False)
    # ... then a smaller shape (other head_dim, fewer rows, shorter cache) in the same array
    one_shape(1, 8, 2, 64, 16, 64, 1500, 6, mixed=False)
    # both head kinds inside a layer: two launches per call share the array in stream order
    one_shape(2, 8, 4, 128, 16, 64, 2100, 7, mixed=True)


def test_static_scratch_decode_refuses_shapes_beyond_its_array():
    from paper_2508_12407_amd import harness as H, binding as zb
    B, Hq, Hkv, D = 9, 32, 8, 128            # 9 * 32 * 128 = 36864 > ZZ_STATIC_MAX_ROW_ELEMS
    st = H.Stack(1, Hq, Hkv, D, B, 256, 16, 64, layer_is_streaming=[0])
    q, k, v = zz_inputs.make_qkv(8, B, 100, Hq, Hkv, D)
    st.append(0, H.to_dev_bf16(k), H.to_dev_bf16(v))
    qd = H.to_dev_bf16(q[:, 99])
    out = torch.full_like(qd, 7.0)
    with pytest.raises(zb.ZzError) as e:
        st.ctx.attn_decode_static(0, qd, out, st.stream_ptr())
    assert e.value.code == zb.ERR["ENOSPC"] and "36864" in str(e.value)
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())            # nothing was launched
    st.ctx.attn_decode(0, qd, out, st.stream_ptr())   # the workspace form still serves the shape
    torch.cuda.synchronize()
    check(H.from_dev(out), O.decode_row(q[:, 99], k, v, 99, np.zeros(Hkv, bool), 16, 64), "workspace form")
