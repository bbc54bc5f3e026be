#!/usr/bin/env python3
"""Benchmark of the relay decode-attention hot path on one MI355X.

A "step" is one decode step of one attention layer for one batch: system attention over the
shared prompt, paged context attention, relay fusion (Alg. 1), through the C ABI.  Inputs are
synthetic (N(0,1) bf16, random block placement) and resident in HBM before the timed region.
The timed steps rotate over several independent copies of the inputs whose total size exceeds
the last-level cache, so every step streams its keys/values from HBM ("cold").

Prints ONE JSON line: the headline workload's attention tokens/s, the roofline of the dominant
kernel (algorithmic bytes / measured kernel time vs the 8 TB/s HBM peak), the system-prompt
length sweep with the per-request ("naive") kernel beside it, and the CPU oracle's throughput.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

COLD_FOOTPRINT_BYTES = 640 << 20     # rotate over at least this much input data

# HBM traffic of one launch of the dominant kernel (relay_tile_kernel), from rocprofv3 counter
# runs of this script (FETCH_SIZE, then WRITE_SIZE, each scaled by what the same counter reads for
# the 512 MiB copy of --calibrate-copy).  A constant copied from that profile, not something this
# run measures: the bench line says so in `traffic_source`.
TRAFFIC_PROFILE = "profiles/relay_tile_kernel_llama30b_s2048_hbm_traffic.md"
MEASURED_TRAFFIC_BYTES = {"llama30b_s2048": 165.08e6 + 4.14e6}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=300)
    ap.add_argument("--workload", default="llama30b_s2048",
                    help="llama7b | llama30b_s<len> | llama3_8b_gqa | tiny")
    ap.add_argument("--no-sweep", action="store_true", help="skip the system-prompt-length sweep")
    ap.add_argument("--no-naive", action="store_true", help="skip the per-request comparison kernel")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP-graph replay timing")
    ap.add_argument("--warm", action="store_true", help="reuse one input set (cache-resident)")
    ap.add_argument("--sys-layout", default="padded", choices=["padded", "token", "head"],
                    help="storage of the system cache: [s][Hkv][d] with the row stride the library\n"
                         "recommends (relay_attn_system_cache_layout), dense [s][Hkv][d], or [Hkv][s][d]")
    ap.add_argument("--timeline", action="store_true",
                    help="per-wavefront begin/end times of the partial-attention launch of --workload\n"
                         "(and of the prompt-phase launch), summarised")
    ap.add_argument("--speedup-grid", action="store_true",
                    help="measured vs theoretical speedup over per-request attention for batch sizes\n"
                         "{4,8,16,32} x context {128,256} x the prompt-length sweep (Sec. 3.4, Fig. 5's grid)")
    ap.add_argument("--decode-loop", action="store_true",
                    help="generation loops with growing contexts (cache append + decode attention per\n"
                         "step) at fixed user-prompt / generation lengths (App. C's synthetic workloads)")
    ap.add_argument("--multi-prefix", action="store_true",
                    help="several system prompts in one batch: one grouped call vs one call per group")
    ap.add_argument("--prefill", action="store_true",
                    help="time only the prompt-phase kernel at the Llama-13B shape (for profiling it)")
    ap.add_argument("--stream-probe", action="store_true",
                    help="only the memory-system yardsticks: read-only streaming kernels (ordinary and\n"
                         "non-temporal loads) and the cost of an empty launch")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the other shapes, the reduced speedup grid and the generation-loop row")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 512 MiB device copy (counter calibration for profiling)")
    ap.add_argument("--sys-chunk", type=int, default=0)
    ap.add_argument("--ctx-part", type=int, default=0)
    return ap.parse_args()


def workload_config(name):
    import workloads as W
    if name == "llama7b":
        return W.LLAMA7B
    if name == "tiny":
        return W.TINY
    if name == "llama3_8b_gqa":
        return W.LLAMA3_8B_GQA
    if name.startswith("llama30b_s"):
        return W.llama30b(int(name[len("llama30b_s"):]))
    raise SystemExit("unknown workload " + name)


def system_cache(dense):
    """The [s, Hkv, d] tensor copied into a buffer with the layout the library recommends for the
    system cache (padded token rows; relay_attn_system_cache_layout)."""
    import torch
    import paper_2402_14808_amd as ra
    s, Hkv, d = dense.shape
    if s == 0:
        return dense
    _, _, nbytes = ra.relay_attn_system_cache_layout(s, Hkv, d)
    view = ra.system_cache_view(torch.zeros(nbytes // 2, dtype=dense.dtype, device=dense.device), s, Hkv, d)
    view.copy_(dense)
    return view


class DeviceInputs:
    """One independent copy of a batch's inputs, generated on the GPU from a seed."""

    def __init__(self, cfg, seed, dev, with_naive, sys_layout="padded"):
        import torch
        g = torch.Generator(device=dev)
        g.manual_seed(seed)
        B, Hq, Hkv, d, s, bs = (cfg.batch, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim,
                                cfg.sys_len, cfg.block_size)

        def normal(*shape):
            return torch.randn(*shape, generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)

        self.cfg = cfg
        self.q = normal(B, Hq, d)
        self.k_sys, self.v_sys = normal(s, Hkv, d), normal(s, Hkv, d)
        if sys_layout == "head":      # same logical [s, Hkv, d] tensors, stored head-major
            self.k_sys = self.k_sys.permute(1, 0, 2).contiguous().permute(1, 0, 2)
            self.v_sys = self.v_sys.permute(1, 0, 2).contiguous().permute(1, 0, 2)
        lens = torch.randint(cfg.ctx_lo, cfg.ctx_hi + 1, (B,), generator=g, device=dev,
                             dtype=torch.int32)
        self.context_lens = lens
        lens_h = lens.cpu()
        need = (lens_h + bs - 1) // bs
        total = int(need.sum())
        nsb = s // bs if with_naive else 0          # shared system pages for the naive view
        pool = int(math.ceil(total * 1.1)) + 1
        self.k_cache, self.v_cache = normal(pool + nsb, Hkv, bs, d), normal(pool + nsb, Hkv, bs, d)
        order = torch.randperm(pool, generator=g, device=dev).to(torch.int32).cpu()
        width = max(int(need.max()), 1)
        tables = torch.full((B, width), 0x7FFFFFF0, dtype=torch.int32)
        at = 0
        for i in range(B):
            n = int(need[i])
            tables[i, :n] = order[at:at + n]
            at += n
        self.block_tables = tables.to(dev)
        self.max_ctx = int(lens_h.max())
        self.total_ctx = int(lens_h.sum())
        self.out = torch.empty(B, Hq, d, device=dev, dtype=torch.bfloat16)
        if with_naive:
            # the same batch as a per-request kernel sees it: system pages first in every table
            assert s % bs == 0
            self.k_cache[pool:] = self.k_sys.reshape(nsb, bs, Hkv, d).permute(0, 2, 1, 3)
            self.v_cache[pool:] = self.v_sys.reshape(nsb, bs, Hkv, d).permute(0, 2, 1, 3)
        if sys_layout == "padded":
            self.k_sys, self.v_sys = system_cache(self.k_sys), system_cache(self.v_sys)
            nt = torch.full((B, nsb + width), 0x7FFFFFF0, dtype=torch.int32)
            nt[:, :nsb] = pool + torch.arange(nsb, dtype=torch.int32)[None, :]
            nt[:, nsb:] = tables
            self.naive_tables = nt.to(dev)
            self.naive_lens = (lens + s).to(torch.int32)

    def nbytes(self):
        n = 0
        for t in (self.q, self.k_sys, self.v_sys, self.k_cache, self.v_cache):
            n += t.numel() * t.element_size()
        return n


class Runner:
    def __init__(self, cfg, dev, args, with_naive, warm):
        import torch
        import paper_2402_14808_amd as ra
        from paper_2402_14808_amd import io_model
        self.ra, self.torch, self.cfg = ra, torch, cfg
        first = DeviceInputs(cfg, 1000, dev, with_naive, args.sys_layout)
        n_sets = 1 if warm else max(2, int(math.ceil(COLD_FOOTPRINT_BYTES / first.nbytes())))
        self.sets = [first] + [DeviceInputs(cfg, 1000 + i, dev, with_naive, args.sys_layout) for i in range(1, n_sets)]
        self.calls, self.naive_calls, self.partial_calls = [], [], []
        self.keep = []
        for st in self.sets:
            tune = dict(sys_chunk_tokens=args.sys_chunk, ctx_part_tokens=args.ctx_part)
            p = ra.make_params(st.q, st.out, st.k_sys, st.k_cache, st.block_tables,
                               batch=cfg.batch, softmax_scale=cfg.scale,
                               max_context_len=st.max_ctx, **tune)
            ws = torch.empty(ra.relay_attn_workspace_bytes(p, cfg.batch), dtype=torch.uint8, device=dev)
            self.keep += [p, ws]
            args_ = (st.q, st.k_sys, st.v_sys, st.k_cache, st.v_cache, st.block_tables,
                     st.context_lens, st.out, None, ws)
            self.calls.append((p, args_))
            self.partial_calls.append((p, (1,) + args_))
            if with_naive:
                pn = ra.make_params(st.q, st.out, None, st.k_cache, st.naive_tables,
                                    batch=cfg.batch, softmax_scale=cfg.scale,
                                    max_context_len=st.max_ctx + cfg.sys_len,
                                    ctx_part_tokens=args.ctx_part)
                wn = torch.empty(ra.relay_attn_workspace_bytes(pn, cfg.batch), dtype=torch.uint8,
                                 device=dev)
                self.keep += [pn, wn]
                self.naive_calls.append((pn, (st.q, st.k_cache, st.v_cache, st.naive_tables,
                                              st.naive_lens, st.out, None, wn)))
        total_ctx = sum(s.total_ctx for s in self.sets) / len(self.sets)
        shape = (cfg.batch, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.sys_len, total_ctx)
        self.relay_bytes = io_model.relay_decode_bytes(*shape)
        self.naive_bytes = io_model.naive_decode_bytes(*shape)

    def _loop(self, fn, calls, steps, first=0):
        n = len(calls)
        for i in range(steps):
            p, a = calls[(first + i) % n]
            fn(p, *a)

    def time_steps(self, kind, steps, warmup):
        """Returns (wall ms/step, event ms/step): exactly `steps` steps between two syncs."""
        torch = self.torch
        fn, calls = {"relay": (self.ra.relay_attn_decode, self.calls),
                     "partial": (self.ra.relay_attn_debug_decode_phases, self.partial_calls),
                     "naive": (self.ra.paged_attn_decode_naive, self.naive_calls)}[kind]
        self._loop(fn, calls, warmup)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0.record()
        self._loop(fn, calls, steps, warmup)
        e1.record()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) * 1e3 / steps
        return wall, e0.elapsed_time(e1) / steps


def time_spread(run, kind="relay", chunks=25, per=40):
    """Spread of the step time: `chunks` groups of `per` back-to-back steps, each bracketed by its
    own pair of events; returns the 10th / 50th / 90th percentile of the per-step time in us."""
    torch = run.torch
    fn, calls = {"relay": (run.ra.relay_attn_decode, run.calls),
                 "naive": (run.ra.paged_attn_decode_naive, run.naive_calls)}[kind]
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
             for _ in range(chunks)]
    run._loop(fn, calls, 10)
    torch.cuda.synchronize()
    at = 10
    for e0, e1 in pairs:
        e0.record()
        run._loop(fn, calls, per, at)
        e1.record()
        at += per
    torch.cuda.synchronize()
    us = sorted(e0.elapsed_time(e1) / per * 1e3 for e0, e1 in pairs)
    pick = lambda q: us[min(len(us) - 1, int(q * len(us)))]
    return {"p10": pick(0.10), "p50": pick(0.50), "p90": pick(0.90), "groups": chunks, "steps_per_group": per}


def time_graph(run, steps):
    """The same steps replayed from a captured HIP graph (60 steps per graph, rotating over the
    input sets): what a serving loop that captures its decode step pays per step."""
    torch = run.torch
    per_graph = 60
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):
        run._loop(run.ra.relay_attn_decode, run.calls, per_graph)
    replays = max(steps // per_graph, 1)
    for _ in range(2):
        graph.replay()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(replays):
        graph.replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / (replays * per_graph)


def time_prefill(dev, steps=40, with_timeline=False):
    """Relay prefill at the Llama-13B shape (batch 16, 40 heads, system prompt 4096, 64..512 new
    tokens per request attending causally to themselves): the matrix-unit-bound row of the path.
    with_timeline: also one call through relay_attn_debug_timeline, summarised per workgroup."""
    import numpy as np
    import torch
    import workloads as W
    import paper_2402_14808_amd as ra
    from paper_2402_14808_amd import io_model
    cfg = W.LLAMA13B_PREFILL
    g = torch.Generator(device=dev)
    g.manual_seed(77)
    B, Hq, Hkv, d, s, bs = cfg.batch, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.sys_len, cfg.block_size

    def normal(*shape):
        return torch.randn(*shape, generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)

    m = torch.randint(cfg.q_lo, cfg.q_hi + 1, (B,), generator=g, device=dev, dtype=torch.int32).cpu()
    cu = torch.zeros(B + 1, dtype=torch.int32)
    cu[1:] = torch.cumsum(m, 0)
    total_q, max_q = int(cu[-1]), int(m.max())
    need = (m + bs - 1) // bs
    pool = int(need.sum()) + 8
    order = torch.randperm(pool, generator=g, device=dev).to(torch.int32).cpu()
    tables = torch.full((B, int(need.max())), 0x7FFFFFF0, dtype=torch.int32)
    at = 0
    for i in range(B):
        n = int(need[i])
        tables[i, :n] = order[at:at + n]
        at += n
    q, out = normal(total_q, Hq, d), torch.empty(total_q, Hq, d, device=dev, dtype=torch.bfloat16)
    k_sys, v_sys = system_cache(normal(s, Hkv, d)), system_cache(normal(s, Hkv, d))
    k_cache, v_cache = normal(pool, Hkv, bs, d), normal(pool, Hkv, bs, d)
    tables_d, lens_d, cu_d = tables.to(dev), m.to(dev), cu.to(dev)
    p = ra.make_params(q, out, k_sys, k_cache, tables_d, batch=B, softmax_scale=cfg.scale,
                       max_context_len=max_q)
    ws = torch.empty(ra.relay_attn_workspace_bytes(p, total_q), dtype=torch.uint8, device=dev)

    def step():
        ra.relay_attn_prefill(p, q, cu_d, total_q, max_q, k_sys, v_sys, k_cache, v_cache, tables_d,
                              lens_d, out, None, ws)
    for _ in range(20):                      # (the first calls after idle run slower)
        step()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    mm = m.numpy().astype(np.float64)
    flops = 4.0 * Hq * d * (total_q * s + float((mm * (mm + 1) / 2).sum()))
    extra = {}
    if with_timeline:
        tl = torch.zeros(2 * 4 * 8192, dtype=torch.int64, device=dev)
        ra.relay_attn_debug_timeline(p, q, cu_d, total_q, max_q, k_sys, v_sys, k_cache, v_cache, tables_d,
                                     lens_d, out, None, ws, tl)
        torch.cuda.synchronize()
        t = tl.cpu().numpy().reshape(-1, 2).astype(np.float64)
        t = t[t[:, 0] > 0]
        t0 = t[:, 0].min()
        b = (t[:, 0] - t0).reshape(-1, 4).min(axis=1) / 100.0       # per workgroup, us
        e = (t[:, 1] - t0).reshape(-1, 4).max(axis=1) / 100.0
        pct = lambda x: [round(float(v), 1) for v in np.percentile(x, [0, 10, 50, 90, 100])]
        every = 20.0
        extra["timeline"] = {
            "workgroups": int(len(b)), "launch_span_us": round(float(e.max()), 1),
            "percentiles": "min, 10 %, median, 90 %, max",
            "workgroup_duration_us": pct(e - b),
            "duration_of_the_first_256_us": pct((e - b)[:256]), "duration_of_the_next_256_us": pct((e - b)[256:512]),
            "active_workgroups_every_20_us": [int(((b <= x) & (e > x)).sum()) for x in np.arange(0, e.max(), every)]}
    return {**extra, "workload": "llama13b_prefill: batch %d, %d heads, head_dim %d, system prompt %d, %d new "
                        "tokens in all (%d..%d per request)" % (B, Hq, d, s, total_q, cfg.q_lo, cfg.q_hi),
            "gpu_ms": ms, "query_tokens_s": total_q / (ms * 1e-3),
            "roofline": {"bound": "mfma", "achieved": flops / (ms * 1e-3) / 1e12,
                         "peak": io_model.MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                         "frac": flops / (ms * 1e-3) / 1e12 / io_model.MFMA_BF16_PEAK_TFLOPS,
                         "flops": flops}}


def speedup_grid(dev, args, batches=(4, 8, 16, 32), contexts=(128, 256), sys_lens=None, steps=200):
    """Relay vs per-request attention on the grid of the paper's standalone-attention experiment
    (Llama-30B attention: 52 heads, head_dim 128; batch 4/8/16/32; context 128/256; system prompt
    512..16384), next to Eq. 10 and to the byte-count ratio of this implementation."""
    import torch
    import workloads as W
    import paper_2402_14808_amd as ra
    from paper_2402_14808_amd import io_model
    rows = []
    for c in contexts:
        for b in batches:
            for s in (sys_lens or W.LLAMA30B_SWEEP):
                cfg = W.AttnConfig("grid_b%d_c%d_s%d" % (b, c, s), b, 52, 52, 128, s, c, c)
                r = Runner(cfg, dev, args, True, args.warm)
                _, relay_ms = r.time_steps("relay", steps, 10)
                _, naive_ms = r.time_steps("naive", 30 if s < 8192 else 10, 3)
                rows.append({"batch": b, "context": c, "sys_len": s, "relay_us": relay_ms * 1e3,
                             "naive_us": naive_ms * 1e3, "measured_speedup": naive_ms / relay_ms,
                             "eq10_speedup": io_model.paper_speedup(b, s, c),
                             "byte_ratio": r.naive_bytes / r.relay_bytes,
                             "relay_hbm_gbs": r.relay_bytes / (relay_ms * 1e-3) / 1e9})
                del r
                torch.cuda.empty_cache()
    return rows


def decode_loop(dev, args, sys_lens=(512, 1024, 2048), shapes=((64, 128), (128, 256), (256, 512))):
    """Attention layers only, no weights: for every generated token, write the new key/value into
    the paged cache (Alg. 1's cache write) and run one decode attention step, with contexts that
    grow from the user-prompt length to user + generation length.  Shapes of App. C: (user,
    generation) = (64,128), (128,256), (256,512); Llama2-7B attention (32 heads, head_dim 128),
    batch 32.  Three ways per shape: relay with the cache write fused into the attention launch,
    relay with the cache write as a launch of its own, and the per-request kernel."""
    import torch
    import workloads as W
    import paper_2402_14808_amd as ra
    B, H, d, bs = 32, 32, 128, 16
    g = torch.Generator(device=dev)
    g.manual_seed(5)

    def normal(*shape):
        return torch.randn(*shape, generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)

    rows = []
    for s in sys_lens:
        for user, gen in shapes:
            cmax = user + gen
            nb = (cmax + bs - 1) // bs
            nsb = s // bs
            pool = B * nb
            k_cache, v_cache = normal(pool + nsb, H, bs, d), normal(pool + nsb, H, bs, d)
            k_sys, v_sys = normal(s, H, d), normal(s, H, d)
            k_cache[pool:] = k_sys.reshape(nsb, bs, H, d).permute(0, 2, 1, 3)
            v_cache[pool:] = v_sys.reshape(nsb, bs, H, d).permute(0, 2, 1, 3)
            k_sys, v_sys = system_cache(k_sys), system_cache(v_sys)
            order = torch.randperm(pool, generator=g, device=dev).to(torch.int32).view(B, nb)
            naive_tables = torch.cat([(pool + torch.arange(nsb, dtype=torch.int32, device=dev))
                                      .expand(B, nsb), order], dim=1).contiguous()
            q, out = normal(B, H, d), torch.empty(B, H, d, device=dev, dtype=torch.bfloat16)
            new_kv = normal(8, B, 2 * H, d)            # a few steps' worth of projections, reused
            p = ra.make_params(q, out, k_sys, k_cache, order, batch=B, softmax_scale=d ** -0.5,
                               max_context_len=cmax)
            pn = ra.make_params(q, out, None, k_cache, naive_tables, batch=B, softmax_scale=d ** -0.5,
                                max_context_len=cmax + s)
            ws = torch.empty(max(ra.relay_attn_workspace_bytes(p, B),
                                 ra.relay_attn_workspace_bytes(pn, B)), dtype=torch.uint8, device=dev)

            def run(kind):
                lens = torch.full((B,), user, dtype=torch.int32, device=dev)
                lens_naive = lens + s
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                torch.cuda.synchronize()
                e0.record()
                for t in range(gen):
                    lens += 1                           # the new token joins the context
                    kv = new_kv[t % 8]
                    if kind == "fused":
                        ra.relay_attn_decode_append(p, q, kv[:, :H], kv[:, H:], k_sys, v_sys, k_cache,
                                                    v_cache, order, lens, out, None, ws)
                        continue
                    ra.relay_attn_cache_append(p, kv[:, :H], kv[:, H:], None, B, k_cache, v_cache,
                                               order, lens)
                    if kind == "relay":
                        ra.relay_attn_decode(p, q, k_sys, v_sys, k_cache, v_cache, order, lens, out,
                                             None, ws)
                    else:
                        lens_naive += 1
                        ra.paged_attn_decode_naive(pn, q, k_cache, v_cache, naive_tables, lens_naive,
                                                   out, None, ws)
                e1.record()
                torch.cuda.synchronize()
                return e0.elapsed_time(e1)

            run("fused")
            fused_ms, relay_ms, naive_ms = run("fused"), run("relay"), run("naive")
            rows.append({"sys_len": s, "user_len": user, "gen_len": gen,
                         "relay_fused_append_us_per_step": fused_ms * 1e3 / gen,
                         "relay_us_per_step": relay_ms * 1e3 / gen,
                         "naive_us_per_step": naive_ms * 1e3 / gen,
                         "speedup": naive_ms / fused_ms,
                         "relay_attn_tokens_s": B * gen / (fused_ms * 1e-3)})
            del k_cache, v_cache, ws
            torch.cuda.empty_cache()
    return rows


def multi_prefix(dev, args):
    """Batch 32 of the Llama-30B attention shape split evenly over 1, 2, 4 or 8 applications with
    a system prompt each (App. D): one relay_attn_decode_multi call against one relay_attn_decode
    call per application, and against the bytes both have to move."""
    import torch
    import workloads as W
    import paper_2402_14808_amd as ra
    from paper_2402_14808_amd import io_model
    rows = []
    for s in (1024, 2048, 4096):
        for n_apps in (1, 2, 4, 8):
            cfg = W.llama30b(s)
            B, per = cfg.batch, cfg.batch // n_apps
            n_sets = max(2, int(math.ceil(COLD_FOOTPRINT_BYTES / (n_apps * s * 52 * 128 * 4 + 110e6))))
            grouped, separate, keep = [], [], []
            for i in range(n_sets):
                st = DeviceInputs(cfg, 3000 + i, dev, False)
                g = torch.Generator(device=dev)
                g.manual_seed(4000 + i)
                apps = [(st.k_sys, st.v_sys)]
                for _ in range(n_apps - 1):
                    apps.append(tuple(system_cache(torch.randn(s, 52, 128, generator=g, device=dev,
                                                               dtype=torch.float32).to(torch.bfloat16))
                                      for _ in range(2)))
                p = ra.make_params(st.q, st.out, st.k_sys, st.k_cache, st.block_tables, batch=B,
                                   softmax_scale=cfg.scale, max_context_len=st.max_ctx,
                                   sys_chunk_tokens=args.sys_chunk, ctx_part_tokens=args.ctx_part)
                ws = torch.empty(ra.relay_attn_workspace_bytes(p, B), dtype=torch.uint8, device=dev)
                groups = ra.make_prefixes([(k, v, a * per, per) for a, (k, v) in enumerate(apps)])
                grouped.append((p, groups, st, ws))
                subs = []
                for a, (k, v) in enumerate(apps):
                    sl = slice(a * per, (a + 1) * per)
                    q, o = st.q[sl], st.out[sl]
                    bt, cl = st.block_tables[sl], st.context_lens[sl]
                    ps = ra.make_params(q, o, k, st.k_cache, bt, batch=per, softmax_scale=cfg.scale,
                                        max_context_len=st.max_ctx)
                    subs.append((ps, (q, k, v, st.k_cache, st.v_cache, bt, cl, o, None, ws)))
                separate.append(subs)
                keep.append(apps)

            def run_grouped(i):
                p, groups, st, ws = grouped[i % n_sets]
                ra.relay_attn_decode_multi(p, groups, st.q, st.k_cache, st.v_cache, st.block_tables,
                                           st.context_lens, st.out, None, ws)

            def run_separate(i):
                for ps, a in separate[i % n_sets]:
                    ra.relay_attn_decode(ps, *a)

            def timed(fn, steps=300, warm=10):
                for i in range(warm):
                    fn(i)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                torch.cuda.synchronize()
                e0.record()
                for i in range(steps):
                    fn(warm + i)
                e1.record()
                torch.cuda.synchronize()
                return e0.elapsed_time(e1) / steps

            g_ms, s_ms = timed(run_grouped), timed(run_separate)
            total_ctx = sum(x[2].total_ctx for x in grouped) / n_sets
            nbytes = io_model.relay_decode_bytes(B, 52, 52, 128, s, total_ctx) + \
                (n_apps - 1) * 2 * s * 52 * 128 * 2
            rows.append({"sys_len": s, "applications": n_apps, "requests_each": per,
                         "grouped_us": g_ms * 1e3, "one_call_per_app_us": s_ms * 1e3,
                         "bytes": nbytes, "grouped_hbm_gbs": nbytes / (g_ms * 1e-3) / 1e9})
            del grouped, separate, keep
            torch.cuda.empty_cache()
    return rows


def timeline(dev, args, cfg):
    """When the wavefronts of the partial-attention launch begin and end (the device's 100 MHz
    counter, through relay_attn_debug_timeline), after the usual warm-up over cold input sets:
    percentiles per kind of workgroup and the means per XCD (workgroup i runs on XCD i mod 8)."""
    import numpy as np
    import torch
    import paper_2402_14808_amd as ra

    def pct(x):
        return [round(float(v), 2) for v in np.percentile(x, [0, 10, 50, 90, 100])]

    run = Runner(cfg, dev, args, False, False)
    run._loop(ra.relay_attn_decode, run.calls, 300)               # steady state, cold inputs
    p, fn_args = run.calls[300 % len(run.calls)]
    plan = ra.relay_attn_decode_plan(p)
    n_sys, n_ctx = 4 * plan.num_sys_workgroups, plan.num_ctx_wavefronts
    tl = torch.zeros(2 * (n_sys + n_ctx), dtype=torch.int64, device=dev)
    q, k_sys, v_sys, k_cache, v_cache, tables, lens, out, _, ws = fn_args
    ra.relay_attn_debug_timeline(p, q, None, cfg.batch, 1, k_sys, v_sys, k_cache, v_cache, tables, lens, out,
                                 None, ws, tl)
    torch.cuda.synchronize()
    t = tl.cpu().numpy().reshape(-1, 2).astype(np.float64)
    t0 = t[:, 0].min()
    b, e = (t[:, 0] - t0) / 100.0, (t[:, 1] - t0) / 100.0          # us
    wg_end = e.reshape(-1, 4).max(axis=1)
    n_wg = len(wg_end)
    res = {"workload": cfg.name, "system_workgroups": plan.num_sys_workgroups,
           "context_wavefronts": n_ctx, "launch_span_us": round(float(e.max()), 2),
           "percentiles": "min, 10 %, median, 90 %, max (us after the first wavefront began)",
           "context_begin_us": pct(b[n_sys:]), "context_end_us": pct(e[n_sys:])}
    if n_sys:
        res["system_begin_us"], res["system_end_us"] = pct(b[:n_sys]), pct(e[:n_sys])
        res["system_end_mean_by_xcd_us"] = [
            round(float(wg_end[:plan.num_sys_workgroups][np.arange(plan.num_sys_workgroups) % 8 == x].mean()), 2)
            for x in range(8) if (np.arange(plan.num_sys_workgroups) % 8 == x).any()]
    res["context_end_mean_by_xcd_us"] = [
        round(float(wg_end[plan.num_sys_workgroups:][np.arange(plan.num_sys_workgroups, n_wg) % 8 == x].mean()), 2)
        for x in range(8)]
    return res


def stream_probe(dev):
    """What the memory system delivers to a kernel that only reads (coalesced 16-byte loads,
    512 MiB per launch rotating over 2 GiB, far outside the last-level cache), and what an empty
    launch costs in a stream: the yardsticks for how much of a step is streaming and how much is
    launches."""
    import torch
    import paper_2402_14808_amd as ra
    per, total = 512 << 20, 2 << 30
    buf = torch.empty(total, dtype=torch.uint8, device=dev).fill_(1)
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    n = total // per

    def timed(fn, reps):
        for i in range(3):
            fn(i)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for i in range(reps):
            fn(i)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    out = {"bytes_per_launch": per}
    for name, nt in (("ordinary_loads_gbs", 0), ("nontemporal_loads_gbs", 1)):
        ms = timed(lambda i: ra.relay_attn_debug_stream_probe(buf[(i % n) * per:], per, nt, sink), 40)
        out[name] = per / (ms * 1e-3) / 1e9
    out["empty_launch_us"] = timed(lambda i: ra.relay_attn_debug_launch_probe(sink, 500), 8) * 1e3 / 500
    del buf
    torch.cuda.empty_cache()
    return out


def other_shape(name, dev, args):
    """A BASELINE shape other than the headline one, same protocol: whole step, the dominant
    kernel alone, the per-request kernel beside it."""
    import torch
    from paper_2402_14808_amd import io_model
    cfg = workload_config(name)
    with_naive = not args.no_naive and cfg.sys_len % cfg.block_size == 0
    r = Runner(cfg, dev, args, with_naive, args.warm)
    _, e_ms = r.time_steps("relay", 400, 300)     # (the first few hundred steps after idle run slower)
    _, k_ms = r.time_steps("partial", 200, 50)
    row = {"workload": "%s: batch %d, %d q heads / %d kv heads, head_dim %d, system prompt %d, context "
                       "%d..%d" % (cfg.name, cfg.batch, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim,
                                   cfg.sys_len, cfg.ctx_lo, cfg.ctx_hi),
           "gpu_us": e_ms * 1e3, "kernel_us": k_ms * 1e3, "attn_tokens_s": cfg.batch / (e_ms * 1e-3),
           "algorithmic_bytes": r.relay_bytes,
           "hbm_gbs": r.relay_bytes / (e_ms * 1e-3) / 1e9,
           "hbm_frac": r.relay_bytes / (e_ms * 1e-3) / 1e9 / io_model.HBM_PEAK_GBS,
           "kernel_hbm_frac": r.relay_bytes / (k_ms * 1e-3) / 1e9 / io_model.HBM_PEAK_GBS}
    if with_naive:
        _, n_ms = r.time_steps("naive", 20, 3)
        row.update({"naive_us": n_ms * 1e3, "speedup": n_ms / e_ms})
    del r
    torch.cuda.empty_cache()
    return row


def cpu_baseline(cfg, seed=1000):
    """The CPU oracle, as it stands, on the headline batch: attention tokens/s on the host."""
    import numpy as np
    import oracle
    import workloads as W
    case = W.make_case(cfg, seed, poison_tails=False)
    reps, spent, used = 0, 0.0, 1
    while spent < 10.0 and reps < 500:
        t0 = time.perf_counter()
        _, _, used = oracle.decode_attention(case.q, case.k_sys, case.v_sys, case.k_cache,
                                             case.v_cache, case.block_tables, case.context_lens,
                                             case.scale)
        spent += time.perf_counter() - t0
        reps += 1
    return {"value": cfg.batch * reps / spent, "unit": "attn tokens/s", "cores": int(used),
            "kind": "oracle",
            "sample": "whole batch of %s (%d requests x %d heads, fp64), %d repetitions, %.1f s"
                      % (cfg.name, cfg.batch, cfg.num_q_heads, reps, spent)}


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (--gpus 1); the path is a single-GPU "
              "kernel library and nothing in it uses a second GPU", file=sys.stderr)
        return 2
    import torch
    import workloads as W
    import paper_2402_14808_amd as ra
    from paper_2402_14808_amd import io_model
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")
    cfg = workload_config(args.workload)
    with_naive = not args.no_naive and cfg.sys_len % cfg.block_size == 0

    if args.speedup_grid:
        print(json.dumps({"metric": "relay vs per-request decode attention, measured and Eq. 10",
                          "data": "synthetic", "dtype": "bf16", "n_gpus": 1,
                          "grid": speedup_grid(dev, args)}))
        return 0
    if args.decode_loop:
        print(json.dumps({"metric": "generation loop, attention layers only: cache append + decode "
                                    "attention per step, relay vs per-request",
                          "data": "synthetic", "dtype": "bf16", "n_gpus": 1,
                          "config": {"workload": "batch 32, 32 heads, head_dim 128 (Llama2-7B attention), "
                                                 "block 16, contexts growing user -> user + gen"},
                          "loops": decode_loop(dev, args)}))
        return 0
    if args.prefill:
        print(json.dumps({"metric": "relay prefill attention, query tokens/s", "data": "synthetic",
                          "dtype": "bf16", "n_gpus": 1, "prefill_llama13b": time_prefill(dev, max(args.steps // 50, 20))}))
        return 0
    if args.multi_prefix:
        print(json.dumps({"metric": "decode attention with several system prompts per batch",
                          "data": "synthetic", "dtype": "bf16", "n_gpus": 1,
                          "config": {"workload": "batch 32, 52 heads, head_dim 128, context 128, "
                                                 "block 16, 1/2/4/8 applications"},
                          "rows": multi_prefix(dev, args)}))
        return 0
    if args.timeline:
        print(json.dumps({"metric": "per-wavefront timeline of the partial-attention launch",
                          "n_gpus": 1, "timeline": timeline(dev, args, cfg),
                          "prefill_llama13b": time_prefill(dev, 20, with_timeline=True)}))
        return 0
    if args.stream_probe:
        print(json.dumps({"metric": "read-only streaming kernels and empty launches (yardsticks)",
                          "n_gpus": 1, "stream_probe": stream_probe(dev)}))
        return 0
    if args.calibrate_copy:
        # a copy kernel of known size: read 512 MiB, write 512 MiB (scale for FETCH_SIZE/WRITE_SIZE)
        src = torch.empty(512 << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    run = Runner(cfg, dev, args, with_naive, args.warm)
    wall_ms, ev_ms = run.time_steps("relay", args.steps, args.warmup)
    _, part_ms = run.time_steps("partial", max(args.steps // 4, 200), 10)
    tokens_s = cfg.batch / (wall_ms * 1e-3)
    achieved = run.relay_bytes / (part_ms * 1e-3) / 1e9
    result = {
        "metric": "decode attn tokens/s + achieved HBM GB/s (% peak) vs system-prompt length",
        "value": tokens_s, "unit": "attn tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": wall_ms, "gpu_ms_per_step": ev_ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "%s: relay decode attention, batch %d, %d q heads / %d kv heads, "
                               "head_dim %d, system prompt %d, context %d..%d, block %d"
                               % (cfg.name, cfg.batch, cfg.num_q_heads, cfg.num_kv_heads,
                                  cfg.head_dim, cfg.sys_len, cfg.ctx_lo, cfg.ctx_hi, cfg.block_size),
                   "system_cache_layout": {"padded": "[s][Hkv][d], token rows padded to %d bytes "
                                                     "(relay_attn_system_cache_layout); the padding is "
                                                     "never read and not counted"
                                                     % (2 * ra.relay_attn_system_cache_layout(
                                                         cfg.sys_len, cfg.num_kv_heads, cfg.head_dim)[0]),
                                           "token": "[s][Hkv][d] dense",
                                           "head": "[Hkv][s][d]"}[args.sys_layout],
                   "cache_state": "warm (one input set)" if args.warm else
                                  "cold (rotating %d input sets, %.0f MiB)" %
                                  (len(run.sets), sum(s.nbytes() for s in run.sets) / 2**20)},
        "step_us_spread": time_spread(run),
        "hbm_gbs_whole_step": run.relay_bytes / (ev_ms * 1e-3) / 1e9,
        "hbm_frac_whole_step": run.relay_bytes / (ev_ms * 1e-3) / 1e9 / io_model.HBM_PEAK_GBS,
        "roofline": {"bound": "hbm", "kernel": "relay_tile_kernel (system + context partial attention)",
                     "achieved": achieved, "peak": io_model.HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / io_model.HBM_PEAK_GBS,
                     "traffic": MEASURED_TRAFFIC_BYTES.get(args.workload)
                     if not (args.sys_chunk or args.ctx_part or args.warm) else None,
                     "traffic_source": TRAFFIC_PROFILE + " (a constant from that counter run, not "
                                       "measured by this one)",
                     "algorithmic_bytes": run.relay_bytes, "kernel_ms": part_ms,
                     "kernel_launches_timed": max(args.steps // 4, 200)},
    }
    if not args.no_graph:
        g_ms = time_graph(run, min(args.steps, 600))
        result["graph_replay"] = {"gpu_ms_per_step": g_ms,
                                  "hbm_frac_whole_step": run.relay_bytes / (g_ms * 1e-3) / 1e9 / io_model.HBM_PEAK_GBS,
                                  "note": "same steps replayed from a captured HIP graph; not used for `value`"}
    if with_naive:
        _, nv_ms = run.time_steps("naive", max(args.steps // 10, 10), 5)
        result["naive"] = {"gpu_ms_per_step": nv_ms, "attn_tokens_s": cfg.batch / (nv_ms * 1e-3),
                           "bytes": run.naive_bytes,
                           "hbm_gbs": run.naive_bytes / (nv_ms * 1e-3) / 1e9,
                           "measured_speedup_of_relay": nv_ms / ev_ms,
                           "eq10_speedup": io_model.paper_speedup(cfg.batch, cfg.sys_len,
                                                                  (cfg.ctx_lo + cfg.ctx_hi) / 2),
                           "byte_model_speedup": run.naive_bytes / run.relay_bytes}
    del run
    torch.cuda.empty_cache()

    probe = None
    if not args.no_sweep:
        probe = stream_probe(dev)
        result["stream_probe"] = probe
        sweep = []
        for s in W.LLAMA30B_SWEEP:
            c = W.llama30b(s)
            r = Runner(c, dev, args, not args.no_naive, args.warm)
            steps = max(200, min(args.steps, 1000))
            w_ms, e_ms = r.time_steps("relay", steps, 200)
            _, k_ms = r.time_steps("partial", 200, 50)
            # where the step goes: the two launches as such, the bytes at the rate a pure
            # streaming kernel reaches on this machine, and the rest (ramp, uneven finish, the fusion
            # kernel's own work)
            launches_us = 2 * probe["empty_launch_us"]
            stream_us = r.relay_bytes / (probe["nontemporal_loads_gbs"] * 1e9) * 1e6
            row = {"sys_len": s, "gpu_us": e_ms * 1e3, "wall_us": w_ms * 1e3,
                   "kernel_us": k_ms * 1e3,
                   "attn_tokens_s": c.batch / (e_ms * 1e-3),
                   "hbm_gbs": r.relay_bytes / (e_ms * 1e-3) / 1e9,
                   "hbm_frac": r.relay_bytes / (e_ms * 1e-3) / 1e9 / io_model.HBM_PEAK_GBS,
                   "kernel_hbm_frac": r.relay_bytes / (k_ms * 1e-3) / 1e9 / io_model.HBM_PEAK_GBS,
                   "target_us_at_70pct": r.relay_bytes / (0.7 * io_model.HBM_PEAK_GBS * 1e9) * 1e6,
                   "decomposition_us": {"two_launches": launches_us, "streaming_at_probe_rate": stream_us,
                                        "second_launch_beyond_first": (e_ms - k_ms) * 1e3,
                                        "rest": e_ms * 1e3 - launches_us - stream_us}}
            if not args.no_graph:
                row["graph_us"] = time_graph(r, 300) * 1e3
            if not args.no_naive:
                _, n_ms = r.time_steps("naive", max(steps // 20, 10), 3)
                row.update({"naive_us": n_ms * 1e3, "speedup": n_ms / e_ms,
                            "eq10": io_model.paper_speedup(c.batch, s, 128),
                            "naive_hbm_gbs": r.naive_bytes / (n_ms * 1e-3) / 1e9})
            sweep.append(row)
            del r
            torch.cuda.empty_cache()
        result["sweep_llama30b"] = sweep

    if not args.no_sweep:
        result["prefill_llama13b"] = time_prefill(dev)
    if not args.no_sweep and not args.no_extras:
        result["other_shapes"] = [other_shape(n, dev, args) for n in ("llama7b", "llama3_8b_gqa")]
        result["speedup_grid_reduced"] = speedup_grid(dev, args, batches=(4, 32), contexts=(128, 256),
                                                      sys_lens=(512, 2048, 16384), steps=100)
        result["decode_loop"] = decode_loop(dev, args, sys_lens=(2048,), shapes=((64, 128),))
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg)
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
