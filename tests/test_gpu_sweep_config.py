"""GPU parity at the setting of the paper's own efficiency experiment (Section 3.2; sink 128 and
window 256 per Section 3.3): Llama-3-8B head shape, batch 1, decode at a context beyond 17k
tokens and a chunked prefill, for (i) a zigzag stack, (ii) the unmodified model (every layer
retrieval) and (iii) mixed layers whose number of streaming heads follows a global quantile of
synthetic importances (2 to 7 of 8 per layer).  Oracle on sampled (layer, KV head) units."""
import numpy as np
import pytest

import zz_inputs
from oracle import zz_oracle as O

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

MAX_ABS, REL_L2 = 2e-2, 5e-3
S, W, Hq, Hkv, D, B = 128, 256, 32, 8, 128, 1
G = Hq // Hkv


def check(got, want, what):
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    assert got.shape == want.shape and np.isfinite(got).all(), what
    max_abs = np.abs(got - want).max()
    rel = np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-300)
    assert max_abs <= MAX_ABS and rel <= REL_L2, (what, max_abs, rel)


def quantile_head_mask(seed, L):
    """The heads of smallest importance stream (half of all heads): a different number in every layer."""
    alpha = zz_inputs.draw_head_importances(seed, L, Hkv)
    order = np.argsort(alpha, axis=None, kind="stable")
    m = np.zeros(L * Hkv, np.uint8)
    m[order[: L * Hkv // 2]] = 1
    return m.reshape(L, Hkv)


def layouts():
    from paper_2508_12407_amd import binding as zb
    full = quantile_head_mask(0, 32)
    counts = full.sum(axis=1)
    picked = [int(np.flatnonzero(counts == c)[0]) for c in (2, 5, 7)]     # the extremes and the middle
    assert sorted(set(counts)) [0] == 2 and sorted(set(counts))[-1] == 7
    return {
        "zigzag": (dict(layout=zb.ZZ_ZIGZAG, layer_is_streaming=[0, 1, 0]), np.array([[0] * Hkv, [1] * Hkv, [0] * Hkv], bool)),
        "all_retrieval": (dict(layout=zb.ZZ_ZIGZAG, layer_is_streaming=[0, 0, 0]), np.zeros((3, Hkv), bool)),
        "mixed_by_quantile": (dict(layout=zb.ZZ_MIXED, kvhead_is_streaming=full[picked]), full[picked].astype(bool)),
    }


@pytest.mark.parametrize("name", ["zigzag", "all_retrieval", "mixed_by_quantile"])
def test_decode_beyond_17k_and_chunked_prefill_at_the_sweep_setting(name):
    from paper_2508_12407_amd import harness as H
    kw, kinds = layouts()[name]
    L, T, C = 3, 17408 + 700, 4096          # 16k prompt + 1k decoded, then a 700-token chunk on top
    n_dec = 17408
    q, k, v = zz_inputs.make_qkv(61, B, T, Hq, Hkv, D)
    st = H.Stack(L, Hq, Hkv, D, B, T, S, W, max_chunk=C, poison_arena=True, **kw)
    kd, vd, qd = H.to_dev_bf16(k), H.to_dev_bf16(v), H.to_dev_bf16(q)
    scale = O.default_scale(D)
    rows = [0, 1, 63, 64, 255, 256, 257, 699]
    for l in range(L):
        for a in range(0, n_dec, C):          # the prompt and the decoded tokens, appended in chunks
            e = min(a + C, n_dec)
            st.append(l, kd[:, a:e].contiguous(), vd[:, a:e].contiguous())
        out = H.from_dev(st.decode(l, qd[:, n_dec - 1].contiguous()))
        for g in range(Hkv):
            J = O.attended_positions(n_dec - 1, bool(kinds[l, g]), S, W)
            want = O.decode_unit(q[0, n_dec - 1, g * G:(g + 1) * G], k[0, J, g], v[0, J, g], scale)
            check(out[0, g * G:(g + 1) * G], want, (name, "decode", l, g))
        # a 700-token chunk in two calls (400 + 300): cached tiles, staged tiles, the window edge inside the chunk
        for a, e in ((n_dec, n_dec + 400), (n_dec + 400, T)):
            pre = H.from_dev(st.prefill(l, qd[:, a:e].contiguous(), kd[:, a:e].contiguous(), vd[:, a:e].contiguous()))
            st.append(l, kd[:, a:e].contiguous(), vd[:, a:e].contiguous())
            for r in rows:
                i = n_dec + r
                if not (a <= i < e):
                    continue
                for h in (0, 5, 14, 23, 31):
                    J = O.attended_positions(i, bool(kinds[l, h // G]), S, W)
                    want = O.attention_row(q[0, i, h], k[0, J, h // G], v[0, J, h // G], scale)
                    check(pre[0, i - a, h], want, (name, "prefill", l, i, h))
