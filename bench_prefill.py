"""Chunked-prefill leg of bench.py (workload c4): a 64k-token prompt fed in 4096-token
chunks through all 32 layers (16 retrieval + 16 streaming).  A step is the whole prompt."""
from __future__ import annotations

import os
import time

import numpy as np

MFMA_BF16_PEAK_TFLOPS = 2500.0


def attended_pairs(T, streaming, S, W):
    """Number of (query, key) pairs the mask keeps for one head over a T-token prompt."""
    if not streaming:
        return T * (T + 1) // 2
    n = S + W
    if T <= n:
        return T * (T + 1) // 2
    return n * (n + 1) // 2 + (T - n) * n


def bench_prefill(args, wname, steps=None, warmup=None):
    import torch
    import zz_inputs
    from paper_2508_12407_amd import binding as zb, harness
    steps = steps or args.steps
    warmup = args.warmup if warmup is None else warmup
    w = zz_inputs.WORKLOADS[wname]
    B, Hq, Hkv, D, L, T, C = w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.n_layers, w.context, w.chunk
    lmask = zz_inputs.draw_layer_mask(args.seed, L, w.n_streaming_layers)
    st = harness.Stack(L, Hq, Hkv, D, B, T, w.sink, w.window, max_chunk=C, layer_is_streaming=lmask)
    gen = torch.Generator(device="cuda").manual_seed(args.seed + 1)
    n_chunks = T // C
    # one set of chunk tensors per chunk index, shared by all layers (values do not affect timing)
    q = torch.randn((n_chunks, B, C, Hq, D), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    k = torch.randn((n_chunks, B, C, Hkv, D), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    v = torch.randn((n_chunks, B, C, Hkv, D), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    out = torch.empty_like(q[0])
    keep_out = {}
    sp = st.stream_ptr()

    kind_counts = {False: [0, 0], True: [0, 0]}

    def one_prompt(record=False):
        st.ctx.reset()
        vis = cau = 0
        for c in range(n_chunks):
            for l in range(L):
                if record:
                    a, b_ = st.ctx.prefill_tile_counts(l, C)
                    vis += a
                    cau += b_
                    kind_counts[bool(lmask[l])][0] += a
                    kind_counts[bool(lmask[l])][1] += b_
                st.ctx.attn_prefill(l, q[c], k[c], v[c], C, out, sp)
                if record and (c, l) in keep_out:
                    keep_out[(c, l)] = out.float().cpu().numpy()
                st.ctx.kv_append(l, k[c], v[c], C, sp)
        return vis, cau

    retr = [l for l in range(L) if not lmask[l]]
    strm = [l for l in range(L) if lmask[l]]
    last = n_chunks - 1
    if not args.no_cpu:
        keep_out[(last, retr[0])] = None
        keep_out[(last, strm[0])] = None
    vis, cau = one_prompt(record=True)
    torch.cuda.synchronize()
    for _ in range(max(0, warmup - 1)):      # the recording pass above was the first warm-up prompt
        one_prompt()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        one_prompt()
    torch.cuda.synchronize()
    t_step = (time.perf_counter() - t0) / steps

    # dominant kernel: the last chunk of a retrieval layer (n_past = T - C), HIP events on the launch stream
    # (every retrieval layer's last-chunk call is the same launch: all of them are timed, in one more prompt)
    st.ctx.reset()
    evs = []
    for c in range(n_chunks):
        for l in range(L):
            if c == last and not lmask[l]:
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                st.ctx.attn_prefill(l, q[c], k[c], v[c], C, out, sp)
                e1.record()
                evs.append((e0, e1))
            else:
                st.ctx.attn_prefill(l, q[c], k[c], v[c], C, out, sp)
            st.ctx.kv_append(l, k[c], v[c], C, sp)
    torch.cuda.synchronize()
    t_kernel = float(np.mean([a.elapsed_time(b) for a, b in evs])) * 1e-3
    pairs_last = sum(i + 1 for i in range(T - C, T))            # retrieval, last chunk, per head
    flop_last = pairs_last * 4 * D * Hq * B

    flop = sum(attended_pairs(T, bool(lmask[l]), w.sink, w.window) for l in range(L)) * 4 * D * Hq * B
    parity = None
    cpu = None
    if not args.no_cpu:
        from oracle import zz_oracle as O
        # oracle on sampled query rows of the last chunk (same launch configuration as timed)
        kh = k.float().cpu().numpy().transpose(1, 0, 2, 3, 4).reshape(B, T, Hkv, D)
        vh = v.float().cpu().numpy().transpose(1, 0, 2, 3, 4).reshape(B, T, Hkv, D)
        qh = q[last].float().cpu().numpy()
        rows = [0, 1, 17, C // 2, C - 2, C - 1]
        heads = [0, Hq // 2 + 1, Hq - 1]
        G = Hq // Hkv
        scale = O.default_scale(D)
        max_abs, num, den = 0.0, 0.0, 0.0
        # one (query row, head) per unit, spread over the host threads the way the decode baseline is
        threads, host_cores = min(os.cpu_count() or 1, 16), os.cpu_count() or 1
        units, meta = [], []
        for (c, l), got in keep_out.items():
            streaming = bool(lmask[l])
            for r in rows:
                i = c * C + r
                J = O.attended_positions(i, streaming, w.sink, w.window)
                for h in heads:
                    units.append((qh[0, r, h][None, :], kh[0, J, h // G], vh[0, J, h // G]))
                    meta.append((got, r, h))
        t1 = time.perf_counter()
        wants = O.decode_units(units, scale, threads=threads)
        t_cpu = time.perf_counter() - t1
        n_rows = len(units)
        for (got, r, h), want in zip(meta, wants):
            d = got[0, r, h].astype(np.float64) - want[0]
            max_abs = max(max_abs, float(np.abs(d).max()))
            num += float((d ** 2).sum())
            den += float((want ** 2).sum())
        parity = dict(max_abs=max_abs, rel_l2=float(np.sqrt(num / den)), rows=n_rows)
        # CPU baseline: the oracle's time per sampled row, extrapolated by attended pairs
        pairs_sample = sum(len(O.attended_positions(c * C + r, bool(lmask[l]), w.sink, w.window))
                           for (c, l) in keep_out for r in rows) * len(heads)
        total_pairs = flop / (4 * D)
        t_cpu_prompt = total_pairs / pairs_sample * t_cpu     # seconds the oracle would need for the whole prompt
        cpu = dict(value=flop / t_cpu_prompt / 1e12, unit="TFLOP/s", ms_per_prompt_token=t_cpu_prompt * 1e3 / (T * B),
                   cores=threads, host_cores_visible=host_cores, kind="oracle", measured_on_sample_s=t_cpu,
                   extrapolated=True,
                   sample=f"{n_rows} (query row, head) pairs of the last chunk of one retrieval and one streaming "
                          f"layer, {t_cpu:.2f} s wall on {threads} threads (the host shows {host_cores} cores; a "
                          f"one-GPU box's share is 16), extrapolated by attended (query,key) pairs")
    import bench as B_
    traffic, traffic_source = B_.profiled_traffic("prefill_c4_64k_chunked.txt") if wname == "c4_prefill_64k" else (None, None)
    return {
        "metric": "chunked prefill attention TFLOP/s (all layers)", "value": flop / t_step / 1e12, "unit": "TFLOP/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": t_step * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wname, "layout": "zigzag", "n_layers": L, "n_q_heads": Hq, "n_kv_heads": Hkv,
                   "head_dim": D, "batch": B, "prompt": T, "chunk": C, "sink": w.sink, "window": w.window,
                   "streaming_layers": w.n_streaming_layers, "step": "whole prompt: attention + append per chunk per layer"},
        "algorithmic_flop_per_step": flop, "us_per_prompt_token": t_step / (T * B) * 1e6,
        "skipped_tile_fraction": 1.0 - vis / cau,
        "skipped_tile_fraction_by_kind": {"retrieval": 1.0 - kind_counts[False][0] / max(kind_counts[False][1], 1),
                                          "streaming": 1.0 - kind_counts[True][0] / max(kind_counts[True][1], 1)},
        "tile": "32 keys x 64 query positions x 2 heads (the share of a KV tile that four waves work on)",
        # every visited (workgroup, tile) pair is computed in full: scores and P V for 64 x 2 x 32 pairs
        "tile_granular_flop_per_step": vis * 64 * 2 * 32 * 4 * D,
        "roofline": {"bound": "mfma", "kernel": "zz_prefill_kernel<128, 2, paired>, retrieval layer, last 4096-token chunk of 65536 (chunk staging included)",
                     "achieved": flop_last / t_kernel / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": flop_last / t_kernel / 1e12 / MFMA_BF16_PEAK_TFLOPS, "flop_per_launch": flop_last,
                     "avg_launch_us": t_kernel * 1e6, "traffic": traffic, "traffic_source": traffic_source},
        "cpu_baseline": cpu, "parity_sample": parity,
    }
