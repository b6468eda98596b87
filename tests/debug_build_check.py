"""Run by tests/test_gpu_debug_build.py in a process of its own with ZZ_LIBRARY=libzz_debug.so: the
library built with -DZZ_DEBUG_BOUNDS checks every cache-slot write (append kernels, fused append)
against the head's capacity before storing and counts refusals in a workspace word.  Every kind
of write the library makes is exercised here; the word must stay 0 and the caches must be what
the oracle's cache model says."""
import sys

import numpy as np
import torch

import zz_inputs
from oracle import zz_oracle as O
from paper_2508_12407_amd import binding as zb, harness as H


def debug_word(st):
    off = int(zb.lib.zz_debug_word_offset(st.cfg))
    assert off > 0
    torch.cuda.synchronize()
    return int(st.workspace[off:off + 4].view(torch.int32).item()), off


def main():
    assert zb.lib.zz_is_debug_build() == 1, "this check must run against libzz_debug.so"
    S, W, B, Hq, Hkv, D = 16, 64, 3, 8, 2, 128
    T = 400
    q, k, v = zz_inputs.make_qkv(5, B, T, Hq, Hkv, D)
    kd, vd, qd = H.to_dev_bf16(k), H.to_dev_bf16(v), H.to_dev_bf16(q)
    hm = np.array([[0, 1], [1, 0], [0, 0], [1, 1]], np.uint8)
    st = H.Stack(4, Hq, Hkv, D, B, T + 8, S, W, max_chunk=128, layout=zb.ZZ_MIXED, kvhead_is_streaming=hm, poison_arena=True)
    _, off = debug_word(st)
    st.workspace[off:off + 4].zero_()
    # chunks that straddle the sink edge, wrap the ring, exceed the window; single tokens; fused steps;
    # a prefill (staging) before every append of a chunk; the last stretch with the sequences at unequal lengths
    cuts = [0, 10, 23, 24, 90, 91, 171, 300]
    for a, b in zip(cuts[:-1], cuts[1:]):
        for l in range(4):
            if b - a <= 128:
                st.prefill(l, qd[:, a:b].contiguous(), kd[:, a:b].contiguous(), vd[:, a:b].contiguous())
            st.append(l, kd[:, a:b].contiguous(), vd[:, a:b].contiguous())
    for t in range(300, 360):
        for l in range(4):
            st.decode_step(l, qd[:, t].contiguous(), kd[:, t:t + 1].contiguous(), vd[:, t:t + 1].contiguous())
    arena = st.arena_host()
    for l in range(4):
        for g in range(Hkv):
            streaming = bool(hm[l, g])
            cap = O.cache_capacity(streaming, S, W, T + 8)
            for which, X in ((0, k), (1, v)):
                img, valid = O.expected_cache(zz_inputs.bf16_bits(X), 360, streaming, S, W, cap)
                slots = np.flatnonzero(valid)
                for bb in range(B):
                    got = st.read_cache_rows(arena, l, which, bb, g, slots)
                    assert np.array_equal(got, img[bb, g, slots]), (l, g, which, bb)
    for l in range(4):                       # unequal lengths: one launch with per-sequence lengths
        st.ctx.set_seq_len(l, 1, 333)
        st.ctx.set_seq_len(l, 2, 35)
        st.prefill(l, qd[:, 360:400].contiguous(), kd[:, 360:400].contiguous(), vd[:, 360:400].contiguous())
        st.append(l, kd[:, 360:400].contiguous(), vd[:, 360:400].contiguous())
        st.decode_step(l, qd[:, 0].contiguous(), kd[:, 0:1].contiguous(), vd[:, 0:1].contiguous())
    n, _ = debug_word(st)
    print("refused slot writes:", n)
    return 0 if n == 0 else 1


if __name__ == "__main__":
    sys.exit(main())
