"""Second workload of bench.py (--workload sweep): the shape of the paper's own efficiency
experiment (Section 3.2, Figures 1 and 2) on MI355X.  Llama-3-8B shape, batch 1, 50 % of the
KV budget streaming, sink 128 and window 256 (Section 3.3).
  decode : prompt of 16k, per-token latency after 1k .. 32k decoded tokens
  prefill: per-token latency of prompts of 1k .. 32k (4096-token chunks)
for the zigzag layout, the mixed-head layout and the unmodified model (every layer retrieval)."""
from __future__ import annotations

import time

import numpy as np


def bench_sweep(args):
    import torch
    import zz_inputs
    from paper_2508_12407_amd import binding as zb, harness
    L, Hq, Hkv, D, B, S, W, C = 32, 32, 8, 128, 1, 128, 256, 4096
    max_ctx = 16384 + 32768 + 64
    lmask = zz_inputs.draw_layer_mask(args.seed, L, L // 2)
    hmask = zz_inputs.draw_kvhead_mask(args.seed, L, Hkv, Hkv // 2)
    # The paper's own pipeline on synthetic importances: bimodal alpha per (layer, KV head); the
    # heads of smallest alpha are streaming heads (Section 2.1: a different number in every
    # layer), and the transport optimisation (Section 2.2) turns that into whole layers.
    alpha = zz_inputs.draw_head_importances(args.seed, L, Hkv)
    order = np.argsort(alpha, axis=None, kind="stable")
    hmask_q = np.zeros(L * Hkv, np.uint8)
    hmask_q[order[: L * Hkv // 2]] = 1
    hmask_q = hmask_q.reshape(L, Hkv)
    lmask_t, _ = zb.transport_select(alpha, 0.5, float(np.float32(0.1)))
    layouts = {
        "zigzag": dict(layout=zb.ZZ_ZIGZAG, layer_is_streaming=lmask),
        "mixed": dict(layout=zb.ZZ_MIXED, kvhead_is_streaming=hmask),
        "all_retrieval": dict(layout=zb.ZZ_ZIGZAG, layer_is_streaming=np.zeros(L, np.uint8)),
        "mixed_by_quantile": dict(layout=zb.ZZ_MIXED, kvhead_is_streaming=hmask_q),
        "zigzag_by_transport": dict(layout=zb.ZZ_ZIGZAG, layer_is_streaming=lmask_t),
    }
    gen = torch.Generator(device="cuda").manual_seed(args.seed + 1)
    q1 = torch.randn((L, B, Hq, D), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    k1 = torch.randn((L, B, 1, Hkv, D), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    v1 = torch.randn((L, B, 1, Hkv, D), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    o1 = torch.empty_like(q1)
    qc = torch.randn((B, C, Hq, D), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    kc = torch.randn((B, C, Hkv, D), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    vc = torch.randn((B, C, Hkv, D), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    oc = torch.empty_like(qc)
    decode_lengths = [1024, 2048, 4096, 8192, 16384, 32768]
    prefill_lengths = [1024, 2048, 4096, 8192, 16384, 32768]
    res = {"decode_us_per_token": {}, "prefill_us_per_token": {}, "decode_us_per_token_both_orders": {},
           "prefill_us_per_token_both_orders": {}, "warmup_rounds": {}}
    TOL = 0.02      # a longer context may not be faster than a shorter one by more than this (run-to-run spread is about 1 %)

    def settle(fn, label):
        """Runs fn (which returns a time) until two consecutive results agree within 2 %: the first
        launches after an arena fill and a context creation are not representative."""
        prev = fn()
        for rounds in range(1, 12):
            cur = fn()
            if abs(cur - prev) <= 0.02 * prev:
                res["warmup_rounds"][label] = rounds
                return
            prev = cur
        raise RuntimeError("timings of %s do not settle" % label)

    def both_orders(lengths, fn, label):
        """fn(length) -> time; every length measured in ascending and then in descending order.  A point
        that comes out more than TOL below its predecessor is measured again with that predecessor
        (twice at most, the new pair replacing the old); if it stays below, the run stops with an error."""
        up = [fn(x) for x in lengths]
        down = [fn(x) for x in reversed(lengths)][::-1]
        mean = [(a + b) / 2 for a, b in zip(up, down)]
        for i in range(1, len(mean)):
            for _ in range(2):
                if mean[i] >= mean[i - 1] * (1 - TOL):
                    break
                res.setdefault("remeasured", []).append("%s at %d and %d tokens" % (label, lengths[i - 1], lengths[i]))
                a0, b0 = fn(lengths[i - 1]), fn(lengths[i])
                b1, a1 = fn(lengths[i]), fn(lengths[i - 1])
                up[i - 1], up[i], down[i - 1], down[i] = a0, b0, a1, b1
                mean[i - 1], mean[i] = (a0 + a1) / 2, (b0 + b1) / 2
            if mean[i] < mean[i - 1] * (1 - TOL):
                raise RuntimeError("%s: latency falls from %.2f to %.2f between %d and %d tokens (ascending %s, descending %s)"
                                   % (label, mean[i - 1], mean[i], lengths[i - 1], lengths[i], up, down))
        return mean, {"ascending": up, "descending": down}

    point = getattr(args, "sweep_point", None)
    if point:            # one decode point of one layout (what a kernel trace of a single layout needs)
        layouts = {point: layouts[point]}
        decode_lengths = [1024]
    for name, kw in layouts.items():
        st = harness.Stack(L, Hq, Hkv, D, B, max_ctx, S, W, max_chunk=C, **kw)
        view = st.arena.view(torch.bfloat16)
        step = 1 << 28
        for a in range(0, view.numel(), step):
            n = min(step, view.numel() - a)
            view[a:a + n] = torch.randn(n, generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        sp = st.stream_ptr()
        ctx = st.ctx

        def decode_time(d, steps=args.steps, warmup=args.warmup):
            """us per token at context 16k + d: the caches grow by one token per step and reach that
            context at the last timed step; nothing but zz_decode_step calls inside the timed loop."""
            n_ctx = 16384 + d
            for l in range(L):
                ctx.set_layer_len(l, n_ctx - steps - warmup)

            def one():
                for l in range(L):
                    ctx.decode_step(l, q1[l], k1[l], v1[l], o1[l], sp)
            for _ in range(warmup):
                one()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                one()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) / steps * 1e6

        def prefill_time(T, reps=max(1, min(args.steps, 3))):
            def prompt():
                ctx.reset()
                for a in range(0, T, C):
                    n = min(C, T - a)
                    for l in range(L):
                        ctx.attn_prefill(l, qc, kc, vc, n, oc, sp)
                        ctx.kv_append(l, kc, vc, n, sp)
            prompt()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                prompt()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) / reps / T * 1e6

        settle(lambda: decode_time(decode_lengths[0]), name + " decode")
        res["decode_us_per_token"][name], res["decode_us_per_token_both_orders"][name] = \
            both_orders(decode_lengths, decode_time, name + " decode")
        if point:
            return {"metric": "per-token decode latency after a 16k prompt and 1k decoded tokens, %s layout" % point,
                    "value": res["decode_us_per_token"][name][0], "unit": "us/token", "n_gpus": 1, "steps": args.steps,
                    "warmup": args.warmup, "higher_is_better": False, "dtype": "bf16", "data": "synthetic",
                    "config": {"workload": "paper_efficiency_sweep, one point", "layout": point, "context": 16384 + 1024,
                               "sink": S, "window": W, "streaming_heads_per_layer": (
                                   hmask_q.sum(axis=1).tolist() if point == "mixed_by_quantile" else None)}}
        settle(lambda: prefill_time(prefill_lengths[0]), name + " prefill")
        pre, res["prefill_us_per_token_both_orders"][name] = both_orders(prefill_lengths, lambda T: prefill_time(T) * T, name + " prefill")
        res["prefill_us_per_token"][name] = [t / T for t, T in zip(pre, prefill_lengths)]   # (monotone in total time, reported per token)
        del st
        torch.cuda.empty_cache()

    # roofline, CPU baseline and parity at the longest decode point of the zigzag layout (same seeded layer mask):
    # a cache the library built by appending, units sampled as in the default benchmark
    import bench as B_
    w_long = zz_inputs.Workload("sweep_longest_point", L, Hq, Hkv, D, B, 16384 + decode_lengths[-1], S, W, L // 2)
    retr = [l for l in range(L) if not lmask[l]]
    strm = [l for l in range(L) if lmask[l]]
    sample = [(l, 0, g) for l in retr[:2] + strm[:2] for g in range(Hkv)]
    run = B_.DecodeRun(w_long, "zigzag", args.seed, args, fill="append", sample=sample if not args.no_cpu else ())
    cpu = parity = None
    if not args.no_cpu:
        run.step()
        torch.cuda.synchronize()
        cpu, parity = B_.cpu_baseline_and_parity(run, args.seed)
    t_launch = run.time_launches(False, 5)
    per_launch = B_.layer_bytes(w_long, False, w_long.context)
    roofline = {"bound": "hbm", "kernel": "zz_decode_kernel<128>, one retrieval layer at the longest sweep point (context %d, batch 1)" % w_long.context,
                "achieved": per_launch / t_launch / 1e9, "peak": B_.HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": per_launch / t_launch / 1e9 / B_.HBM_PEAK_GBPS, "bytes_per_launch": per_launch,
                "avg_launch_us": t_launch * 1e6, "traffic": None}
    del run
    torch.cuda.empty_cache()
    z, m, r = (np.array(res["decode_us_per_token"][k]) for k in ("zigzag", "mixed", "all_retrieval"))
    return {
        "metric": "per-token decode latency after a 16k prompt, zigzag layout (paper's efficiency experiment shape)",
        "value": float(z[0]), "unit": "us/token", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": float(z[0]) / 1e3, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "paper_efficiency_sweep", "n_layers": L, "n_q_heads": Hq, "n_kv_heads": Hkv,
                   "head_dim": D, "batch": B, "sink": S, "window": W, "streaming_fraction": 0.5, "prompt": 16384,
                   "decode_lengths": decode_lengths, "prefill_lengths": prefill_lengths, "prefill_chunk": C,
                   "value_is": "zigzag, 1k tokens decoded (context 17408)",
                   "protocol": "each layout warmed after its arena fill until two consecutive timings agree within 2 %, every "
                               "length measured in ascending and in descending order (mean reported), monotone growth checked"},
        "sweep": res, "roofline": roofline, "cpu_baseline": cpu, "parity_sample": parity,
        "zigzag_speedup_over_mixed": (m / z).tolist(), "zigzag_speedup_over_all_retrieval": (r / z).tolist(),
        "transport_zigzag_speedup_over_quantile_mixed":
            (np.array(res["decode_us_per_token"]["mixed_by_quantile"]) /
             np.array(res["decode_us_per_token"]["zigzag_by_transport"])).tolist(),
        "streaming_heads_per_layer_quantile_mixed": hmask_q.sum(axis=1).tolist(),
        "paper_context": "the paper reports up to 37 % acceleration at 1k decoded tokens, shrinking with length, "
                         "and equal prefill latency; its hardware, precision and baseline are not stated",
    }
