"""GPU parity for batches whose sequences differ in length: prompts enter one
sequence at a time (zz_attn_prefill_seq / zz_kv_append_seq), decode advances all
sequences in one launch per head kind, each attending its own prefix.  Every
sequence is compared on its own with the fp64 oracle (the oracle knows nothing of
batches of unequal length: sequence b is simply a batch of one with T_b tokens).
Same bar as the other parity tests; cache contents bit-exact."""
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


def make_stack(H, zb, kind, Hq, Hkv, D, B, max_ctx, S, W, max_chunk):
    """kind: 'retrieval' | 'streaming' (zigzag layers) or a 0/1 list per kv head (mixed layer)."""
    if isinstance(kind, str):
        st = H.Stack(1, Hq, Hkv, D, B, max_ctx, S, W, max_chunk=max_chunk,
                     layer_is_streaming=[int(kind == "streaming")], poison_arena=True)
        kinds = np.full(Hkv, kind == "streaming")
    else:
        st = H.Stack(1, Hq, Hkv, D, B, max_ctx, S, W, max_chunk=max_chunk, layout=zb.ZZ_MIXED,
                     kvhead_is_streaming=np.asarray(kind, np.uint8)[None, :], poison_arena=True)
        kinds = np.asarray(kind, bool)
    st.workspace.fill_(0xFF)
    return st, kinds


def load_prompts(H, st, lens, chunk, qd, kd, vd, with_attention, q=None, k=None, v=None, kinds=None, S=0, W=1):
    """Sequence b receives its first lens[b] tokens in chunks; returns nothing, checks prefill rows if asked."""
    sp = st.stream_ptr()
    for b, n in enumerate(lens):
        for a in range(0, n, chunk):
            e = min(a + chunk, n)
            ka, va = kd[b:b + 1, a:e].contiguous(), vd[b:b + 1, a:e].contiguous()
            if with_attention:
                qa = qd[b:b + 1, a:e].contiguous()
                out = torch.empty_like(qa)
                st.ctx.attn_prefill_seq(0, b, qa, ka, va, e - a, out, sp)
                want = O.attention(q[b:b + 1, :e], k[b:b + 1, :e], v[b:b + 1, :e], kinds, S, W, rows=list(range(a, e)))
                check(H.from_dev(out), want, ("prefill_seq", b, a, e))
            st.ctx.kv_append_seq(0, b, ka, va, e - a, sp)
        assert st.ctx.seq_len(0, b) == n


def check_caches(H, st, lens, k, v, kinds, S, W, max_ctx):
    arena = st.arena_host()
    for g, streaming in enumerate(kinds):
        cap = O.cache_capacity(bool(streaming), S, W, max_ctx)
        for b, n in enumerate(lens):
            for which, X in ((0, k), (1, v)):
                img, valid = O.expected_cache(zz_inputs.bf16_bits(X[b:b + 1]), n, bool(streaming), S, W, cap)
                slots = np.flatnonzero(valid)
                got = st.read_cache_rows(arena, 0, which, b, g, slots)
                assert np.array_equal(got, img[0, g, slots]), ("cache", b, g, which, n)


@pytest.mark.parametrize("kind", ["retrieval", "streaming", [1, 0]])
def test_prompts_of_different_lengths_then_decode_steps(kind):
    H, zb = _harness()
    B, Hq, Hkv, D, S, W = 4, 8, 2, 128, 16, 64
    lens = [700, 33, 1, 290]
    steps, chunk = 6, 256
    T = max(lens) + steps + 40
    q, k, v = zz_inputs.make_qkv(61, B, T, Hq, Hkv, D)
    st, kinds = make_stack(H, zb, kind, Hq, Hkv, D, B, T, S, W, chunk)
    qd, kd, vd = H.to_dev_bf16(q), H.to_dev_bf16(k), H.to_dev_bf16(v)
    load_prompts(H, st, lens, chunk, qd, kd, vd, True, q, k, v, kinds, S, W)
    assert st.ctx.layer_len(0) == max(lens)
    sp = st.stream_ptr()
    lens = list(lens)

    def gather(xd, offset=0):   # row lens[b] + offset of every sequence -> [B, H, D]
        return torch.stack([xd[b, lens[b] + offset] for b in range(B)]).contiguous()

    def want_rows():            # oracle: sequence b alone, attending from its newest token
        return np.concatenate([O.decode_row(q[b:b + 1, n - 1], k[b:b + 1, :n], v[b:b + 1, :n], n - 1, kinds, S, W)
                               for b, n in enumerate(lens)])

    # fused decode steps: one launch per head kind appends and attends for all four sequences
    for s in range(steps):
        out = st.decode_step(0, gather(qd), gather(kd)[:, None].contiguous(), gather(vd)[:, None].contiguous())
        lens = [n + 1 for n in lens]
        check(H.from_dev(out), want_rows(), ("decode_step", kind, s, lens))
        assert [st.ctx.seq_len(0, b) for b in range(B)] == lens
    # two-call form: batched append of one token (issued per sequence), then attention
    st.ctx.kv_append(0, gather(kd)[:, None].contiguous(), gather(vd)[:, None].contiguous(), 1, sp)
    lens = [n + 1 for n in lens]
    check(H.from_dev(st.decode(0, gather(qd, -1))), want_rows(), ("append + decode", kind, lens))
    # batched prefill of 20 more tokens per sequence on unequal lengths
    n_new = 20
    qa = torch.stack([qd[b, n:n + n_new] for b, n in enumerate(lens)]).contiguous()
    ka = torch.stack([kd[b, n:n + n_new] for b, n in enumerate(lens)]).contiguous()
    va = torch.stack([vd[b, n:n + n_new] for b, n in enumerate(lens)]).contiguous()
    got = H.from_dev(st.prefill(0, qa, ka, va))
    for b, n in enumerate(lens):
        want = O.attention(q[b:b + 1, :n + n_new], k[b:b + 1, :n + n_new], v[b:b + 1, :n + n_new], kinds, S, W,
                           rows=list(range(n, n + n_new)))
        check(got[b:b + 1], want, ("batched prefill on unequal lengths", kind, b))
    st.append(0, ka, va)
    lens = [n + n_new for n in lens]
    assert [st.ctx.seq_len(0, b) for b in range(B)] == lens
    check_caches(H, st, lens, k, v, kinds, S, W, T)


@pytest.mark.parametrize("splits", [None, 5, 128])
@pytest.mark.parametrize("kind", ["retrieval", "streaming"])
def test_decode_llama_shape_unequal_lengths_across_split_counts(kind, splits):
    """Lengths from one tile to hundreds of tiles in one launch: long sequences are split
    over many workgroups and merged, short ones take a single workgroup."""
    H, zb = _harness()
    B, Hq, Hkv, D, S, W = 5, 32, 8, 128, 64, 256
    lens = [5000, 3001, 100, 1025, 31]
    T = max(lens) + 4
    q, k, v = zz_inputs.make_qkv(67, B, T, Hq, Hkv, D)
    st, kinds = make_stack(H, zb, kind, Hq, Hkv, D, B, T, S, W, 0)
    if splits is not None:
        st.ctx.tune(zb.TUNE_DECODE_SPLITS, splits)
    qd, kd, vd = H.to_dev_bf16(q), H.to_dev_bf16(k), H.to_dev_bf16(v)
    load_prompts(H, st, lens, 4096, qd, kd, vd, False)
    for s in range(3):
        qs = torch.stack([qd[b, n] for b, n in enumerate(lens)]).contiguous()
        ks = torch.stack([kd[b, n] for b, n in enumerate(lens)])[:, None].contiguous()
        vs = torch.stack([vd[b, n] for b, n in enumerate(lens)])[:, None].contiguous()
        out = st.decode_step(0, qs, ks, vs)
        lens = [n + 1 for n in lens]
        want = np.concatenate([O.decode_row(q[b:b + 1, n - 1], k[b:b + 1, :n], v[b:b + 1, :n], n - 1, kinds, S, W)
                               for b, n in enumerate(lens)])
        check(H.from_dev(out), want, ("decode_step", kind, splits, s))
    check_caches(H, st, lens, k, v, kinds, S, W, T)


def test_unequal_lengths_that_become_equal_take_the_single_length_path_again():
    """Two sequences at 40 and 41 tokens; the shorter one catches up through zz_kv_append_seq.
    From then on the batched calls are the ordinary ones, and results stay those of the oracle."""
    H, zb = _harness()
    B, Hq, Hkv, D, S, W = 2, 4, 2, 64, 4, 16
    T = 60
    q, k, v = zz_inputs.make_qkv(71, B, T, Hq, Hkv, D)
    for kind in ("retrieval", "streaming"):
        st, kinds = make_stack(H, zb, kind, Hq, Hkv, D, B, T, S, W, 0)
        qd, kd, vd = H.to_dev_bf16(q), H.to_dev_bf16(k), H.to_dev_bf16(v)
        load_prompts(H, st, [40, 41], 64, qd, kd, vd, False)
        got = H.from_dev(st.decode(0, torch.stack([qd[0, 39], qd[1, 40]]).contiguous()))
        want = np.concatenate([O.decode_row(q[b:b + 1, n - 1], k[b:b + 1, :n], v[b:b + 1, :n], n - 1, kinds, S, W)
                               for b, n in enumerate([40, 41])])
        check(got, want, ("unequal", kind))
        st.ctx.kv_append_seq(0, 0, kd[0:1, 40:41].contiguous(), vd[0:1, 40:41].contiguous(), 1, st.stream_ptr())
        assert st.ctx.decode_plan(0, int(kind == "streaming"))[0] >= 1
        out = st.decode_step(0, qd[:, 41].contiguous(), kd[:, 41:42].contiguous(), vd[:, 41:42].contiguous())
        check(H.from_dev(out), O.decode_row(q[:, 41], k[:, :42], v[:, :42], 41, kinds, S, W), ("equal again", kind))
        check_caches(H, st, [42, 42], k, v, kinds, S, W, T)


def test_largest_batch_of_unequal_lengths_and_a_larger_batch_of_equal_ones():
    """256 sequences of different lengths in one decode launch (the most the launch can describe),
    and 300 sequences of one length (no such limit); a sample of sequences against the oracle."""
    H, zb = _harness()
    Hq, Hkv, D, S, W = 4, 2, 64, 8, 40
    for B, unequal in ((zb.ZZ_MAX_RAGGED_BATCH, True), (300, False)):
        rng = np.random.default_rng(B)
        lens = [int(x) for x in rng.integers(1, 400, size=B)] if unequal else [123] * B
        T = max(lens) + 2
        q, k, v = zz_inputs.make_qkv(81, B, T, Hq, Hkv, D)
        for kind in ("retrieval", "streaming"):
            st, kinds = make_stack(H, zb, kind, Hq, Hkv, D, B, T, S, W, 0)
            qd, kd, vd = H.to_dev_bf16(q), H.to_dev_bf16(k), H.to_dev_bf16(v)
            sp = st.stream_ptr()
            if unequal:
                # the whole batch appended once to the longest length, then the lengths declared:
                # a retrieval cache's prefix is the shorter cache; a ring is rebuilt per sequence below
                if kind == "retrieval":
                    st.append(0, kd[:, :T - 2].contiguous(), vd[:, :T - 2].contiguous())
                    for b, n in enumerate(lens):
                        st.ctx.set_seq_len(0, b, n)
                else:
                    for b, n in enumerate(lens):
                        st.ctx.kv_append_seq(0, b, kd[b:b + 1, :n].contiguous(), vd[b:b + 1, :n].contiguous(), n, sp)
            else:
                st.append(0, kd[:, :123].contiguous(), vd[:, :123].contiguous())
            cur = list(lens)
            for step in range(2):
                out = st.decode_step(0, torch.stack([qd[b, n] for b, n in enumerate(cur)]).contiguous(),
                                     torch.stack([kd[b, n] for b, n in enumerate(cur)])[:, None].contiguous(),
                                     torch.stack([vd[b, n] for b, n in enumerate(cur)])[:, None].contiguous())
                cur = [n + 1 for n in cur]
                got = H.from_dev(out)
                assert np.isfinite(got).all()
                for b in (0, 1, B // 2, B - 2, B - 1):
                    n = cur[b]
                    want = O.decode_row(q[b:b + 1, n - 1], k[b:b + 1, :n], v[b:b + 1, :n], n - 1, kinds, S, W)
                    check(got[b:b + 1], want, ("large batch", B, kind, step, b))
            assert [st.ctx.seq_len(0, b) for b in (0, B - 1)] == [cur[0], cur[-1]]
