"""Third workload of bench.py (--workload unequal): decode over a batch whose sequences
differ in length, Llama-3-8B shape of the 128k workload (32 layers, 16 of them streaming,
sink 64, window 256).  A step is one zz_decode_step per layer for the whole batch: one
launch per layer in the zigzag layout, two in the mixed-head layout, whatever the lengths.
The retrieval-layer launch is compared with the HBM peak on the bytes of the caches it
actually reads (sum over the sequences of 2 * Hkv * len_b * D * 2)."""
from __future__ import annotations

import dataclasses
import time

import numpy as np

LENGTH_MIXES = {
    "b4_128k_to_16k": [131072, 65536, 32768, 16384],
    "b8_128k_to_4k": [131072, 98304, 65536, 49152, 32768, 16384, 8192, 4096],
}


def make_run(base_cls, w, layout, seed, args, lens):
    class UnequalRun(base_cls):
        """DecodeRun whose sequences sit at different lengths (caches drawn in place)."""

        def reset_lengths(self, steps_to_go):
            for l in range(self.w.n_layers):
                for b, n in enumerate(lens):
                    self.st.ctx.set_seq_len(l, b, n - steps_to_go)

        def full_lengths(self):
            for l in range(self.w.n_layers):
                for b, n in enumerate(lens):
                    self.st.ctx.set_seq_len(l, b, n)

        def bytes_per_step(self):
            w = self.w
            total = 0
            for l in range(w.n_layers):
                for g in range(w.n_kv_heads):
                    streaming = bool(self.lmask[l]) if self.layout == "zigzag" else bool(self.hmask[l][g])
                    for n in lens:
                        total += 2 * (min(n, w.sink + w.window) if streaming else n) * w.head_dim * 2
            return total

    return UnequalRun(w, layout, seed, args, fill="random")


def prefill_unequal(args, base, lens, chunk=1024):
    """A chunk of `chunk` new tokens for every sequence of a batch whose sequences hold different
    numbers of tokens: one zz_attn_prefill + zz_kv_append per layer for the whole batch (one
    attention launch per layer) against the same work as one call per sequence."""
    import torch
    from paper_2508_12407_amd import harness
    L, B = 4, len(lens)
    st = harness.Stack(L, base.n_q_heads, base.n_kv_heads, base.head_dim, B, max(lens) + chunk, base.sink, base.window,
                       max_chunk=chunk, layer_is_streaming=[0, 1, 0, 1])
    st.arena.view(torch.bfloat16).normal_()
    q = torch.randn((B, chunk, base.n_q_heads, base.head_dim), device="cuda").to(torch.bfloat16)
    k = torch.randn((B, chunk, base.n_kv_heads, base.head_dim), device="cuda").to(torch.bfloat16)
    v = torch.randn((B, chunk, base.n_kv_heads, base.head_dim), device="cuda").to(torch.bfloat16)
    out = torch.empty_like(q)
    sp, ctx = st.stream_ptr(), st.ctx

    def reset():
        for l in range(L):
            for b, n in enumerate(lens):
                ctx.set_seq_len(l, b, n)

    def batched():
        reset()
        for l in range(L):
            ctx.attn_prefill(l, q, k, v, chunk, out, sp)
            ctx.kv_append(l, k, v, chunk, sp)

    def per_sequence():
        reset()
        for l in range(L):
            for b in range(B):
                ctx.attn_prefill_seq(l, b, q[b:b + 1], k[b:b + 1], v[b:b + 1], chunk, out[b:b + 1], sp)
                ctx.kv_append_seq(l, b, k[b:b + 1], v[b:b + 1], chunk, sp)

    res = {}
    for name, fn in (("one_call_per_layer", batched), ("one_call_per_sequence", per_sequence)):
        fn()
        torch.cuda.synchronize()
        reps = 5
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        res[name + "_ms"] = (time.perf_counter() - t0) / reps * 1e3
    pairs = sum(sum(i + 1 for i in range(n, n + chunk)) for n in lens)      # retrieval layers: every key up to the query
    res.update(layers="2 retrieval + 2 streaming", chunk=chunk, lengths=lens,
               retrieval_flop=2 * pairs * 4 * base.head_dim * base.n_q_heads,
               speedup=res["one_call_per_sequence_ms"] / res["one_call_per_layer_ms"])
    return res


def bench_unequal(args, DecodeRun, HBM_PEAK_GBPS):
    import torch
    import zz_inputs
    base = zz_inputs.WORKLOADS["c3_llama8b_128k_b4"]
    points = {}
    for name, lens in LENGTH_MIXES.items():
        w = dataclasses.replace(base, name="unequal_" + name, batch=len(lens), context=max(lens))
        run = make_run(DecodeRun, w, "zigzag", args.seed, args, lens)
        t = run.timed(args.steps, args.warmup)
        ev = run.per_step_events(args.steps)
        t_launch = run.time_launches(False, max(3, args.steps // 4))
        nbytes = run.bytes_per_step()
        retr = int(np.flatnonzero(run.lmask == 0)[0])
        ns, tps = run.st.ctx.decode_plan(retr, 0)
        per_launch = sum(2 * w.n_kv_heads * n * w.head_dim * 2 for n in lens)
        tiles = [-(-n // 32) for n in lens]
        wgs = sum(-(-t_ // tps) for t_ in tiles) * w.n_kv_heads
        p = {"lengths": lens, "tokens_in_cache": int(sum(lens)), "ms_per_step": t * 1e3,
             "us_per_token": t / len(lens) * 1e6, "step_by_hip_events": ev,
             "algorithmic_bytes_per_step": nbytes, "achieved_GBps": nbytes / t / 1e9,
             "retrieval_launch": {"avg_us": t_launch * 1e6, "bytes": per_launch, "GBps": per_launch / t_launch / 1e9,
                                  "frac_of_hbm_peak": per_launch / t_launch / 1e9 / HBM_PEAK_GBPS,
                                  "tiles_per_split": tps, "workgroups": wgs,
                                  "largest_share_over_even_share": tps / (sum(tiles) * w.n_kv_heads / wgs)}}
        del run
        torch.cuda.empty_cache()
        if not args.no_mixed:
            mixed = make_run(DecodeRun, w, "mixed", args.seed, args, lens)
            tm = mixed.timed(args.steps, args.warmup)
            p["mixed_head_layout"] = {"ms_per_step": tm * 1e3, "us_per_token": tm / len(lens) * 1e6,
                                      "GBps": mixed.bytes_per_step() / tm / 1e9, "zigzag_speedup": tm / t}
            del mixed
            torch.cuda.empty_cache()
        points[name] = p
    first = points["b4_128k_to_16k"]
    return {
        "metric": "decode attention us/token (all layers)", "value": first["us_per_token"], "unit": "us/token",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": first["ms_per_step"],
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "unequal_lengths_llama8b (value: b4_128k_to_16k)", "n_layers": base.n_layers,
                   "n_q_heads": base.n_q_heads, "n_kv_heads": base.n_kv_heads, "head_dim": base.head_dim,
                   "sink": base.sink, "window": base.window, "streaming_layers": base.n_streaming_layers,
                   "launch": "one zz_decode_step per layer for the whole batch, each sequence at its own length"},
        "roofline": {"bound": "hbm", "kernel": "zz_decode_ragged_kernel<128>, one retrieval layer (b4_128k_to_16k)",
                     "achieved": first["retrieval_launch"]["GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": first["retrieval_launch"]["frac_of_hbm_peak"], "traffic": None},
        "cpu_baseline": None,
        "length_mixes": points,
        "prefill_chunk_on_unequal_lengths": {name: prefill_unequal(args, base, lens) for name, lens in LENGTH_MIXES.items()},
    }
