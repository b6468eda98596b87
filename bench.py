#!/usr/bin/env python3
"""Benchmark of the ZigzagAttention hot path on one MI355X.

A step is one pass of the whole hot path over one batch: for every layer, append
the new token's K/V (ring evict in streaming layers) and run that layer's single
attention launch.  Prints ONE JSON line:
  value            us per generated token = step time / batch, inputs resident in HBM
  achieved_GBps    algorithmic K+V bytes of the step / step time
  roofline         the retrieval-layer attention launch alone (HIP events) against the HBM peak
  cpu_baseline     the fp64 oracle on a sample of the same workload, host threads stated
  parity_sample    the GPU output of that sample against the oracle
  mixed_head_layout, separate_append, attention_only, hip_graph_replay: the same step in the
                   comparison layout / with the append as its own launch / without the append /
                   replayed from a HIP graph
  at_32k_batch1, mha_32k_batch8, prefill_64k_chunked (default workload only): the other
                   configurations, each measured briefly in the same run with its own
                   roofline, cpu_baseline and parity_sample

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c3|c2|c5|c4|sweep|unequal]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0        # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0

ALIASES = {"c2": "c2_llama8b_32k_b1", "c3": "c3_llama8b_128k_b4", "c5": "c5_mha7b_32k_b8", "c4": "c4_prefill_64k"}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c3")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-mixed", action="store_true", help="skip the mixed-head layout comparison")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline and parity sample")
    ap.add_argument("--no-graph", action="store_true", help="do not also time a HIP-graph replay of the step")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 1 GiB device copy (a known-size kernel to scale rocprofv3 byte counters by)")
    ap.add_argument("--no-32k", action="store_true",
                    help="with the default workload: skip the extra measurement at 32k context, batch 1")
    ap.add_argument("--no-legs", action="store_true",
                    help="with the default workload: skip the MHA 32k/batch-8 and the chunked-prefill legs")
    ap.add_argument("--sweep-point", default=None,
                    choices=["zigzag", "mixed", "all_retrieval", "mixed_by_quantile", "zigzag_by_transport"],
                    help="with --workload sweep: only this layout's decode at 1k decoded tokens (for a kernel trace)")
    ap.add_argument("--wg-per-cu", type=int, default=0)
    ap.add_argument("--splits", type=int, default=0)
    return ap.parse_args()


def profiled_traffic(fname):
    """(bytes, source): HBM bytes per launch of the dominant kernel as rocprofv3's FETCH_SIZE /
    WRITE_SIZE counters measured them (two --pmc runs of this program, scaled by a known-size
    copy).  Counters cannot be read from inside the run: the figure comes from the summary
    kept under profiles/, and the source string names the file and the commit it was measured
    at.  (None, None) without a summary."""
    try:
        nbytes, commit = None, "unknown commit"
        for line in open(os.path.join(ROOT, "profiles", fname)):
            if line.startswith("traffic_bytes_per_launch:"):
                nbytes = int(float(line.split(":")[1]))
            elif line.startswith("measured at commit "):
                commit = line.split()[3].rstrip(";,.")
        if nbytes is not None:
            return nbytes, "profiles/%s @ %s (rocprofv3 --pmc FETCH_SIZE, WRITE_SIZE; not measured in this run)" % (fname, commit)
    except OSError:
        pass
    return None, None


def calibrate_copy():
    """Three 1 GiB device-to-device copies: a kernel of known size to scale rocprofv3's byte counters by."""
    import torch
    src = torch.ones(1 << 28, dtype=torch.int32, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)          # reads 1 GiB, writes 1 GiB
    torch.cuda.synchronize()


def host_threads():
    """(threads the oracle is given, cores the host shows).  A one-GPU machine's share of its host is
    16 cores whatever the machine shows."""
    seen = os.cpu_count() or 1
    return min(seen, 16), seen


def layer_bytes(w, streaming, n_ctx):
    n_valid = min(n_ctx, w.sink + w.window) if streaming else n_ctx
    return 2 * w.batch * w.n_kv_heads * n_valid * w.head_dim * 2


class DecodeRun:
    """One layout of one decode workload, resident in HBM.  `n_arenas` > 1 keeps that many
    independent copies of the whole cache and lets consecutive steps rotate over them."""

    def __init__(self, w, layout, seed, args, fill="append", sample=(), n_arenas=1):
        import torch
        import zz_inputs
        from paper_2508_12407_amd import binding as zb, harness
        self.torch, self.zb, self.w = torch, zb, w
        self.lmask = zz_inputs.draw_layer_mask(seed, w.n_layers, w.n_streaming_layers)
        kw = {}
        if layout == "zigzag":
            kw = dict(layout=zb.ZZ_ZIGZAG, layer_is_streaming=self.lmask)
        else:
            frac = w.n_streaming_layers / w.n_layers
            per_layer = int(round(frac * w.n_kv_heads))
            self.hmask = zz_inputs.draw_kvhead_mask(seed, w.n_layers, w.n_kv_heads, per_layer)
            kw = dict(layout=zb.ZZ_MIXED, kvhead_is_streaming=self.hmask)
        self.layout = layout
        self.N = w.context
        self.stacks = [harness.Stack(w.n_layers, w.n_q_heads, w.n_kv_heads, w.head_dim, w.batch, self.N,
                                     w.sink, w.window, **kw) for _ in range(n_arenas)]
        self.st = self.stacks[0]
        self.turn = 0
        for st in self.stacks:
            if args.wg_per_cu:
                st.ctx.tune(zb.TUNE_DECODE_WG_PER_CU, args.wg_per_cu)
            if args.splits:
                st.ctx.tune(zb.TUNE_DECODE_SPLITS, args.splits)
        gen = torch.Generator(device="cuda").manual_seed(seed + 1)
        B, Hq, Hkv, D, L = w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.n_layers
        self.kept = {}
        n_pre = self.N - 1
        for i, st in enumerate(self.stacks):
            if fill == "append" and i == 0:
                # the measured cache is one the library built: N-1 tokens appended in chunks
                chunk = 8192
                for l in range(L):
                    streaming = layout == "zigzag" and bool(self.lmask[l])
                    # a streaming layer keeps the sink tokens and the newest W: appending the first
                    # chunk and the last one (positions in between skipped) builds the same cache
                    starts = list(range(0, n_pre, chunk))
                    if streaming and len(starts) > 2:
                        starts = [0, n_pre - chunk]
                    for a in starts:
                        n = min(chunk, n_pre - a)
                        st.ctx.set_layer_len(l, a)
                        kc = torch.randn((B, n, Hkv, D), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
                        vc = torch.randn((B, n, Hkv, D), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
                        st.append(l, kc, vc)
                        if any(sl == l for (sl, _, _) in sample):
                            kh, vh = kc.float().cpu().numpy(), vc.float().cpu().numpy()
                            for (sl, b, g) in sample:
                                if sl == l:
                                    self.kept.setdefault((sl, b, g), []).append((a, kh[b, :, g], vh[b, :, g]))
            else:
                # any bit pattern of the arena is some cache (the tile layout is a bijection):
                # draw it directly, N(0,1) in bf16, and declare the lengths
                view = st.arena.view(torch.bfloat16)
                step = 1 << 28
                for a in range(0, view.numel(), step):
                    n = min(step, view.numel() - a)
                    view[a:a + n] = torch.randn(n, generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        self.q = torch.randn((L, B, Hq, D), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        self.k1 = torch.randn((L, B, 1, Hkv, D), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        self.v1 = torch.randn((L, B, 1, Hkv, D), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        self.out = torch.empty_like(self.q)
        self.reset_lengths(1)
        torch.cuda.synchronize()

    def reset_lengths(self, steps_to_go):
        """Every cache at N - steps_to_go tokens, so that the last of that many decode steps attends
        to N tokens (host bookkeeping only; outside every timed region).  The caches are not
        restored: slots past the declared length are simply not read."""
        for st in self.stacks:
            for l in range(self.w.n_layers):
                st.ctx.set_layer_len(l, self.N - steps_to_go)

    def full_lengths(self):
        """Every cache at N tokens: what zz_attn_decode alone (no append) attends to."""
        for st in self.stacks:
            for l in range(self.w.n_layers):
                st.ctx.set_layer_len(l, self.N)

    def step(self, mode="fused", rotate=False):
        """One decode step of the whole stack.  fused: zz_decode_step (append inside the
        attention launch); separate: zz_kv_append then zz_attn_decode; attention: only
        zz_attn_decode on the cache as it stands.  The caches grow by one token per step, as
        they do when a model decodes; a timed phase of K steps starts K tokens short of N."""
        st = self.st
        if rotate:
            self.turn = (self.turn + 1) % len(self.stacks)
            st = self.stacks[self.turn]
        ctx, sp = st.ctx, st.stream_ptr()
        for l in range(self.w.n_layers):
            if mode == "fused":
                ctx.decode_step(l, self.q[l], self.k1[l], self.v1[l], self.out[l], sp)
            else:
                if mode == "separate":
                    ctx.kv_append(l, self.k1[l], self.v1[l], 1, sp)
                ctx.attn_decode(l, self.q[l], self.out[l], sp)

    def timed(self, steps, warmup, mode="fused", rotate=False):
        torch = self.torch
        if mode == "attention":
            self.full_lengths()
        else:
            self.reset_lengths(steps + warmup)
        for _ in range(warmup):
            self.step(mode, rotate)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            self.step(mode, rotate)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps

    def per_step_events(self, steps):
        """Median and minimum step time from HIP events around each step (same stream)."""
        torch = self.torch
        self.reset_lengths(steps)
        evs = []
        for _ in range(steps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            self.step()
            e1.record()
            evs.append((e0, e1))
        torch.cuda.synchronize()
        ms = sorted(a.elapsed_time(b) for a, b in evs)
        return {"median_ms": ms[len(ms) // 2], "min_ms": ms[0], "max_ms": ms[-1]}

    def timed_graph(self, steps, warmup):
        """The same step captured once into a HIP graph and replayed (a replay repeats the
        recorded launches: the same slot is rewritten, the same number of tokens attended)."""
        torch = self.torch
        self.reset_lengths(1)
        s = torch.cuda.Stream()
        s.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(s):
            self.step()
        torch.cuda.current_stream().wait_stream(s)
        torch.cuda.synchronize()
        self.reset_lengths(1)
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            self.step()
        for _ in range(warmup):
            g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            g.replay()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps

    def time_launches(self, streaming, reps):
        """Average duration of the attention launch of one layer kind (retrieval: the dominant
        kernel), HIP events on the launch stream around each pass over all layers of that kind
        (back-to-back launches, so a launch's share includes the gap to the next one)."""
        torch = self.torch
        if self.layout != "zigzag":
            return None
        layers = [l for l in range(self.w.n_layers) if bool(self.lmask[l]) == streaming]
        if not layers:
            return None
        self.full_lengths()
        sp = self.st.stream_ptr()
        evs = []
        for r in range(reps + 1):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for l in layers:
                self.st.ctx.attn_decode(l, self.q[l], self.out[l], sp)
            e1.record()
            if r:
                evs.append((e0, e1))
        torch.cuda.synchronize()
        ms = [a.elapsed_time(b) / len(layers) for a, b in evs]
        return float(np.mean(ms)) * 1e-3

    def read_ceiling(self, nbytes=1 << 31, reps=5):
        """GB/s of a pure streaming read of the arena with the decode kernel's access pattern
        (default-policy and non-temporal loads): the practical ceiling beside the 8 TB/s peak."""
        torch = self.torch
        nbytes = min(nbytes, self.st.arena_nbytes)
        out = {}
        for name, nt in (("default_loads", 0), ("nontemporal_loads", 1)):
            sp = self.st.stream_ptr()
            self.st.ctx.probe_read(self.st.arena, nbytes, nt, sp)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                self.st.ctx.probe_read(self.st.arena, nbytes, nt, sp)
            e1.record()
            torch.cuda.synchronize()
            out[name] = nbytes / (e0.elapsed_time(e1) * 1e-3 / reps) / 1e9
        return out

    def bytes_per_step(self, n_ctx=None):
        """Algorithmic K+V bytes of one step at context n_ctx (default N)."""
        w = self.w
        n_ctx = self.N if n_ctx is None else n_ctx
        total = 0
        for l in range(w.n_layers):
            if self.layout == "zigzag":
                total += layer_bytes(w, bool(self.lmask[l]), n_ctx)
            else:
                ns = int(self.hmask[l].sum())
                total += layer_bytes(w, True, n_ctx) * ns // w.n_kv_heads
                total += layer_bytes(w, False, n_ctx) * (w.n_kv_heads - ns) // w.n_kv_heads
        return total


def cpu_baseline_and_parity(run, seed):
    """Times the fp64 oracle on a bounded sample of (layer, batch, kv head) units of the
    same workload and checks the GPU output of those units against it."""
    import torch
    from oracle import zz_oracle as O
    w = run.w
    G = w.n_q_heads // w.n_kv_heads
    scale = O.default_scale(w.head_dim)
    qh = run.q.float().cpu().numpy()
    k1 = run.k1.float().cpu().numpy()
    v1 = run.v1.float().cpu().numpy()
    out = run.out.float().cpu().numpy()
    threads, host_cores = host_threads()
    units, meta = [], []
    for (l, b, g), parts in run.kept.items():
        streaming = bool(run.lmask[l])
        pos = np.concatenate([np.arange(a, a + len(kc)) for (a, kc, vc) in parts] + [np.array([run.N - 1])])
        K = np.concatenate([kc for (a, kc, vc) in parts] + [k1[l, b, :, g]])
        V = np.concatenate([vc for (a, kc, vc) in parts] + [v1[l, b, :, g]])
        J = O.attended_positions(run.N - 1, streaming, w.sink, w.window)
        idx = np.searchsorted(pos, J)
        assert np.array_equal(pos[idx], J), "a position the oracle attends to was never appended"
        units.append((qh[l, b, g * G:(g + 1) * G], K[idx], V[idx]))
        meta.append((l, b, g, streaming))
    res = [None] * len(units)
    t_kind, n_kind = {}, {}
    for kind in (False, True):
        ids = [i for i, mm in enumerate(meta) if mm[3] == kind]
        if not ids:
            continue
        t0 = time.perf_counter()
        outs = O.decode_units([units[i] for i in ids], scale, threads=threads)
        t_kind[kind] = time.perf_counter() - t0
        n_kind[kind] = len(ids)
        for i, o in zip(ids, outs):
            res[i] = o
    max_abs, num, den = 0.0, 0.0, 0.0
    for (l, b, g, streaming), want in zip(meta, res):
        got = out[l, b, g * G:(g + 1) * G].astype(np.float64)
        max_abs = max(max_abs, float(np.abs(got - want).max()))
        num += float(((got - want) ** 2).sum())
        den += float((want ** 2).sum())
    # extrapolate by unit count per layer kind (same thread count, same unit size)
    n_units = {True: int(run.lmask.sum()) * w.batch * w.n_kv_heads,
               False: int((1 - run.lmask).sum()) * w.batch * w.n_kv_heads}
    step_s = sum(t_kind[k] / n_kind[k] * n_units[k] for k in t_kind)
    t_cpu = sum(t_kind.values())
    return dict(value=step_s / w.batch * 1e6, unit="us/token", cores=threads, host_cores_visible=host_cores,
                kind="oracle", measured_on_sample_s=t_cpu, extrapolated=True,
                sample=f"{len(units)} (layer,batch,kv-head) units of this workload "
                       f"({n_kind.get(False, 0)} retrieval, {n_kind.get(True, 0)} streaming: every unit of the "
                       f"sampled layers), {t_cpu:.2f} s wall on {threads} threads (the host shows {host_cores} "
                       f"cores; a one-GPU box's share is 16), extrapolated by unit count "
                       f"to the {n_units[False] + n_units[True]} units of one step"), \
        dict(max_abs=max_abs, rel_l2=float(np.sqrt(num / max(den, 1e-300))), units=len(units))


def bench_decode(args, wname, steps=None, warmup=None, mixed=True, rotate_arenas=0, sample_seconds_cap=None):
    import torch
    import zz_inputs
    steps = steps or args.steps
    warmup = args.warmup if warmup is None else warmup
    w = zz_inputs.WORKLOADS[wname]
    lmask = zz_inputs.draw_layer_mask(args.seed, w.n_layers, w.n_streaming_layers)
    retr = [l for l in range(w.n_layers) if not lmask[l]]
    strm = [l for l in range(w.n_layers) if lmask[l]]
    sample = []
    if not args.no_cpu:
        # every (batch, kv head) unit of one or two retrieval and two streaming layers
        B, Hkv = w.batch, w.n_kv_heads
        n_r = 2 if B * Hkv <= 32 else 1
        picked = retr[:n_r] + strm[:2]
        units = [(b, g) for b in range(B) for g in range(Hkv)]
        if B * Hkv > 64:           # bounded sample: first and last sequence, every KV head
            units = [(b, g) for b in (0, B - 1) for g in range(Hkv)]
        for l in picked:
            sample += [(l, b, g) for (b, g) in units]
    run = DecodeRun(w, "zigzag", args.seed, args, fill="append", sample=sample)
    cpu, parity = (None, None)
    if not args.no_cpu:
        # before anything else grows the caches: the step from N-1 to N tokens, checked against the oracle
        run.step()
        torch.cuda.synchronize()
        cpu, parity = cpu_baseline_and_parity(run, args.seed)
    t_step = run.timed(steps, warmup)
    step_events = run.per_step_events(steps)
    t_sep = run.timed(steps, warmup, mode="separate")
    t_attn = run.timed(steps, warmup, mode="attention")
    t_graph = None if args.no_graph else run.timed_graph(steps, warmup)
    t_launch = run.time_launches(False, max(3, steps // 4))
    t_launch_s = run.time_launches(True, max(3, steps // 4))
    nbytes = run.bytes_per_step()
    ceiling = run.read_ceiling()
    ns, tps = run.st.ctx.decode_plan(retr[0], 0) if retr else (0, 0)
    per_launch = layer_bytes(w, False, w.context)
    per_launch_s = layer_bytes(w, True, w.context)
    traffic, traffic_source = profiled_traffic("decode_retrieval_%s.txt" % wname)
    out = {
        "metric": "decode attention us/token (all layers)",
        "value": t_step / w.batch * 1e6, "unit": "us/token", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": t_step * 1e3, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wname, "layout": "zigzag", "n_layers": w.n_layers, "n_q_heads": w.n_q_heads,
                   "n_kv_heads": w.n_kv_heads, "head_dim": w.head_dim, "batch": w.batch, "context": w.context,
                   "sink": w.sink, "window": w.window, "streaming_layers": w.n_streaming_layers,
                   "launch": "plain stream launches, one zz_decode_step (append fused into the attention launch) per "
                             "layer; nothing but those calls inside the timed loop (the caches grow by one token per step "
                             "and reach `context` tokens at the last timed step; bytes are counted at `context`, at most "
                             "steps/context more than what was read)",
                   "retrieval_split_k": {"splits": ns, "tiles_per_split": tps}},
        "achieved_GBps": nbytes / t_step / 1e9, "frac_of_hbm_peak": nbytes / t_step / 1e9 / HBM_PEAK_GBPS,
        "algorithmic_bytes_per_step": nbytes,
        "step_by_hip_events": step_events,
        "attention_only": {"us_per_token": t_attn / w.batch * 1e6, "GBps": nbytes / t_attn / 1e9},
        "separate_append": {"us_per_token": t_sep / w.batch * 1e6, "GBps": nbytes / t_sep / 1e9,
                            "note": "zz_kv_append + zz_attn_decode per layer (two launches)"},
        "roofline": {"bound": "hbm", "kernel": "zz_decode_kernel<128>, one retrieval layer (split-K merge included)",
                     "achieved": per_launch / t_launch / 1e9 if t_launch else None, "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": per_launch / t_launch / 1e9 / HBM_PEAK_GBPS if t_launch else None,
                     "bytes_per_launch": per_launch, "avg_launch_us": t_launch * 1e6 if t_launch else None,
                     "traffic": traffic, "traffic_source": traffic_source,
                     "streaming_read_GBps": ceiling,
                     "frac_of_streaming_read": per_launch / t_launch / 1e9 / ceiling["nontemporal_loads"] if t_launch else None},
        "streaming_layer_launch": {"avg_launch_us": t_launch_s * 1e6 if t_launch_s else None, "bytes_per_launch": per_launch_s,
                                   "GBps": per_launch_s / t_launch_s / 1e9 if t_launch_s else None},
        "cpu_baseline": cpu, "parity_sample": parity,
    }
    if t_graph is not None:
        out["hip_graph_replay"] = {"us_per_token": t_graph / w.batch * 1e6, "GBps": nbytes / t_graph / 1e9,
                                   "frac_of_hbm_peak": nbytes / t_graph / 1e9 / HBM_PEAK_GBPS}
    del run
    torch.cuda.empty_cache()
    if rotate_arenas > 1:
        # Cache residency: the same step rotating over independent copies of the whole cache, so
        # that no byte (in particular the few MB of the streaming layers) is read again before
        # rotate_arenas - 1 other caches have passed through the memory-side cache.
        rot = DecodeRun(w, "zigzag", args.seed, args, fill="random", n_arenas=rotate_arenas)
        t_one = rot.timed(steps, warmup)
        t_rot = rot.timed(steps, warmup, rotate=True)
        streaming_bytes = sum(layer_bytes(w, True, w.context) for l in strm)
        out["cache_rotation"] = {"arenas": rotate_arenas, "us_per_token_one_arena": t_one / w.batch * 1e6,
                                 "us_per_token_rotating": t_rot / w.batch * 1e6,
                                 "streaming_bytes_per_step": streaming_bytes,
                                 "bytes_between_two_reads_of_a_line": nbytes * rotate_arenas,
                                 "streaming_bytes_of_all_arenas": streaming_bytes * rotate_arenas}
        del rot
        torch.cuda.empty_cache()
    if mixed and not args.no_mixed:
        mx = DecodeRun(w, "mixed", args.seed, args, fill="random")
        tm = mx.timed(steps, warmup)
        tma = mx.timed(steps, warmup, mode="attention")
        tmg = None if args.no_graph else mx.timed_graph(steps, warmup)
        out["mixed_head_layout"] = {"us_per_token": tm / w.batch * 1e6, "ms_per_step": tm * 1e3,
                                    "attention_only_us_per_token": tma / w.batch * 1e6,
                                    "GBps": mx.bytes_per_step() / tm / 1e9,
                                    "algorithmic_bytes_per_step": mx.bytes_per_step(),
                                    "attention_launches_per_step": sum(mx.st.ctx.layer_launches(l) for l in range(w.n_layers)),
                                    "zigzag_speedup": tm / t_step, "zigzag_speedup_attention_only": tma / t_attn}
        if tmg is not None and t_graph is not None:
            out["mixed_head_layout"]["hip_graph_replay_us_per_token"] = tmg / w.batch * 1e6
            out["mixed_head_layout"]["zigzag_speedup_hip_graph_replay"] = tmg / t_graph
        out["config"]["attention_launches_per_step"] = w.n_layers
        del mx
        torch.cuda.empty_cache()
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives are part of the path); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the hot path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    if not os.path.exists(os.path.join(ROOT, "paper_2508_12407_amd", "libzz.so")):
        import __graft_entry__
        __graft_entry__.build()       # only when nothing is built; otherwise the library is used as it is
    wname = ALIASES.get(args.workload, args.workload)
    if args.calibrate_copy:
        calibrate_copy()
    if wname == "sweep":
        from bench_sweep import bench_sweep
        out = bench_sweep(args)
    elif wname == "unequal":
        from bench_unequal import bench_unequal
        out = bench_unequal(args, DecodeRun, HBM_PEAK_GBPS)
    elif wname == "c4_prefill_64k":
        from bench_prefill import bench_prefill
        out = bench_prefill(args, wname)
    else:
        out = bench_decode(args, wname, rotate_arenas=16 if wname == "c2_llama8b_32k_b1" else 0)
        if wname == "c3_llama8b_128k_b4":
            # the other configurations, briefly, in the same run (each leg frees its memory before the next)
            if not args.no_32k:
                out["at_32k_batch1"] = bench_decode(args, "c2_llama8b_32k_b1", rotate_arenas=16)
            if not args.no_legs:
                out["mha_32k_batch8"] = bench_decode(args, "c5_mha7b_32k_b8", steps=min(args.steps, 10),
                                                     warmup=min(args.warmup, 3), mixed=False)
                from bench_prefill import bench_prefill
                out["prefill_64k_chunked"] = bench_prefill(args, "c4_prefill_64k", steps=2, warmup=1)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
