#!/usr/bin/env python3
"""Benchmark of the quantized, paged KV decode step on one MI355X.

A step is one pass of the whole hot path over one synthetic serving batch that is
already resident in HBM: alise_kv_quant_write of the step's new tokens, then
alise_paged_decode_attn over every request's cached context, then
alise_kv_dequant_page of one page.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload int4|llama7b|gqa70b|opt13b|tiny]
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published peak HBM3E bandwidth

PROFILES = os.path.join(ROOT, "profiles")
# sources whose change makes a stored traffic figure stale: everything an attention call runs
ATTENTION_SOURCES = ("alise_api.hip", "alise_kernels.h", "attn_common.h", "decode_attn.hip", "decode_attn_gqa.hip", "mfma_stream.h")


def attention_sources_sha256() -> str:
    import hashlib
    h = hashlib.sha256()
    for name in ATTENTION_SOURCES:
        with open(os.path.join(ROOT, "paper_2410_23537_amd", "csrc", name), "rb") as f:
            h.update(name.encode() + b"\0" + f.read())
    return h.hexdigest()[:16]


def measured_traffic(workload: str):
    """HBM bytes per launch of the attention kernel from the rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE, scaled by a
    copy kernel of known size) whose summary is profiles/attention_step_<workload>.md.  The summary names the hash of
    the attention sources it was taken with; if they have changed since, the figure is stale and not reported.
    Returns (bytes or None, note)."""
    import re
    path = os.path.join(PROFILES, f"attention_step_{workload}.md")
    try:
        text = open(path).read()
    except OSError:
        return None, f"no {os.path.relpath(path, ROOT)}"
    m_bytes = re.search(r"^traffic_bytes_per_launch:\s*(\d+)", text, re.M)
    m_sha = re.search(r"^attention_sources_sha256:\s*([0-9a-f]+)", text, re.M)
    if not m_bytes or not m_sha:
        return None, f"{os.path.relpath(path, ROOT)} carries no traffic figure"
    now = attention_sources_sha256()
    if m_sha.group(1) != now:
        return None, (f"the counters in {os.path.relpath(path, ROOT)} were taken with attention sources {m_sha.group(1)}, "
                      f"they are {now} now: profile again")
    return int(m_bytes.group(1)), f"from {os.path.relpath(path, ROOT)} (same attention sources, {now})"


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="int4")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle baseline")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--only-steps", action="store_true",
                    help="skip the legs outside the timed steps (swap, prefill, fused operators, scheduler): for profiler runs")
    ap.add_argument("--only-prefill", action="store_true",
                    help="after the timed steps run only the prefill leg with a chunk from every request: for profiler runs")
    ap.add_argument("--only-scheduler", nargs="?", const="small", choices=("small", "large"), default=None,
                    help="after the timed steps run only the scheduled run through the C++ loop, the small trace or the large one: "
                         "for profiler runs")
    ap.add_argument("--traffic-calibration", action="store_true",
                    help="also launch an elementwise kernel that reads and writes exactly 1 GiB, so that a "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE run of this command can be scaled")
    return ap.parse_args()


def cpu_baseline(w, step, target_seconds):
    """The CPU oracle timed on a bounded sample of the same workload: whole requests taken in
    batch order until a token budget is reached.  Reported, never a target."""
    import numpy as np
    import oracle
    from paper_2410_23537_amd import workloads as wl

    oracle.build()
    threads = max(1, min(16, os.cpu_count() or 1))
    lens = step.lens
    # calibrate the oracle's two rates on one short request
    cal = wl.replace(w, B=1, name="cal")
    probe_len = int(min(256, lens.max()))
    pg1 = wl.paging(cal, np.array([probe_len], np.int32))
    c1 = oracle.Cache.empty(pg1.num_pages, w.P, w.Hkv, w.D, w.bits, w.G)
    k, v = wl.request_kv(w, step.pool_host, step.offs, 0, 0, probe_len, step.gain)
    t0 = time.perf_counter()
    oracle.kv_quant_write(c1, k, v, wl.slots_of(cal, pg1, 0, 0, probe_len))
    fill_per_token = (time.perf_counter() - t0) / probe_len / threads      # filled by `threads` workers
    qrep = np.repeat(step.q_host[:1], threads, axis=0)
    t0 = time.perf_counter()
    oracle.paged_decode_attn(c1, qrep, np.repeat(pg1.block_tables, threads, axis=0),
                             np.repeat(pg1.lens, threads), step.scale, num_threads=threads)
    attn_per_token = (time.perf_counter() - t0) / (probe_len * threads)
    # token budget: timed work near the target, untimed cache filling at most ~3x that
    budget = int(min(target_seconds / max(attn_per_token, 1e-9), 3 * target_seconds / max(fill_per_token, 1e-9)))
    budget = max(budget, int(lens.min()))
    # sample: every n-th request in batch order so the length mix is kept, within the budget
    stride = max(1, int(math.ceil(lens.astype(np.int64).sum() / budget)))
    chosen, tot = [], 0
    for i in range(0, w.B, stride):
        if tot + int(lens[i]) > budget and chosen:
            continue
        chosen.append(int(i))
        tot += int(lens[i])
    sub_lens = lens[chosen]
    ws = wl.replace(w, B=len(chosen), name="sample")
    pgs = wl.paging(ws, sub_lens)
    cache = oracle.Cache.empty(pgs.num_pages, w.P, w.Hkv, w.D, w.bits, w.G)
    from concurrent.futures import ThreadPoolExecutor

    def fill(j):
        # untimed set-up: the context of one sampled request (requests own disjoint pages)
        i = chosen[j]
        L = int(lens[i])
        k, v = wl.request_kv(w, step.pool_host, step.offs, i, 0, L, step.gain)
        slots = wl.slots_of(ws, pgs, j, 0, L)
        for a in range(0, L - 1, 512):
            b = min(L - 1, a + 512)
            oracle.kv_quant_write(cache, k[a:b], v[a:b], slots[a:b])
        return k[-1:].copy(), v[-1:].copy(), slots[-1:]

    with ThreadPoolExecutor(threads) as ex:
        parts = list(ex.map(fill, range(len(chosen))))
    step_k = np.concatenate([p[0] for p in parts])
    step_v = np.concatenate([p[1] for p in parts])
    step_slots = [p[2] for p in parts]
    step_slots = np.concatenate(step_slots)
    q = step.q_host[chosen]
    t0 = time.perf_counter()
    oracle.kv_quant_write(cache, step_k, step_v, step_slots)
    oracle.paged_decode_attn(cache, q, pgs.block_tables, pgs.lens, step.scale, num_threads=threads)
    oracle.kv_dequant_page(cache, int(pgs.block_tables[0, 0]))
    dt = time.perf_counter() - t0
    nbytes = (wl.algorithmic_bytes_attn(ws, sub_lens) + wl.algorithmic_bytes_write(ws, len(chosen))
              + wl.algorithmic_bytes_dequant(ws, 1))
    # the same attention on one thread, over the first sampled requests that fit about two seconds
    n1, tok1 = 0, 0
    while n1 < len(chosen) and (n1 == 0 or (tok1 + int(sub_lens[n1])) * attn_per_token * threads <= 2.0):
        tok1 += int(sub_lens[n1])
        n1 += 1
    t0 = time.perf_counter()
    oracle.paged_decode_attn(cache, q[:n1], pgs.block_tables[:n1], pgs.lens[:n1], step.scale, num_threads=1)
    dt1 = time.perf_counter() - t0
    one_thread = {"value": wl.algorithmic_bytes_attn(wl.replace(ws, B=n1), sub_lens[:n1]) / dt1 / 1e9, "unit": "GB/s", "cores": 1,
                  "sample": f"attention only, the first {n1} sampled requests ({tok1} KV tokens)", "seconds": dt1,
                  "kv_tokens_per_s": tok1 / dt1}
    return {"value": nbytes / dt / 1e9, "unit": "GB/s", "cores": threads, "kind": "oracle", "one_thread": one_thread,
            "sample": f"{len(chosen)} of {w.B} requests (every {stride}-th in batch order, {tot} of "
                      f"{int(lens.astype(np.int64).sum())} KV tokens), one decode token each, "
                      f"attention split over {threads} threads",
            "seconds": dt, "kv_tokens_per_s": tot / dt}


def swap_leg(step):
    """Offload + upload of the longest request (Sec. 3.2 "Dynamic Swapping", the data movement),
    outside the timed steps: into a device staging buffer (bound: HBM copy) and into pinned host
    memory written by the kernel itself (bound: the host link)."""
    import numpy as np
    import torch
    from paper_2410_23537_amd import binding as B
    cache = step.caches[0]
    i = int(np.argmax(step.lens))
    L = int(step.lens[i])
    bt = torch.from_numpy(np.ascontiguousarray(step.pg.block_tables[i])).cuda()
    n = B.alise_kv_swap_bytes(cache, L)
    out = {"request_tokens": L, "bytes": n}
    for where, buf in (("device_staging", torch.empty(n, dtype=torch.uint8, device="cuda")),
                       ("pinned_host", torch.empty(n, dtype=torch.uint8, pin_memory=True))):
        for name, fn in (("offload", B.alise_kv_swap_out), ("upload", B.alise_kv_swap_in)):
            reps = 10
            for _ in range(2):
                fn(cache, bt, L, buf)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                fn(cache, bt, L, buf)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / reps
            moved = 2 * n if where == "device_staging" else n      # HBM read + HBM write, or bytes over the link
            out[f"{where}_{name}_GBs"] = moved / (ms * 1e-3) / 1e9
    out["note"] = ("device_staging counts bytes read + written in HBM (plain copy on this box: about 5200 GB/s); "
                   "pinned_host counts bytes over the host link (hipMemcpyAsync of the same buffer: about 56 GB/s)")
    # Alg. 2 overlaps the movement with computation: the step's attention call alone, and with the offload of this
    # request running beside it on a second stream (the offload outlasts the call) -- once by the kernel writing pinned
    # host memory itself, once by the kernel gathering into device memory and the copy engine moving that to the host
    side = torch.cuda.Stream()
    host, stage = buf, torch.empty(n, dtype=torch.uint8, device="cuda")

    def attention_ms(beside):
        ts = []
        for _ in range(12):
            torch.cuda.synchronize()
            with torch.cuda.stream(side):
                if beside == "kernel":
                    B.alise_kv_swap_out(cache, bt, L, host)
                elif beside == "copy_engine":
                    B.alise_kv_swap_out(cache, bt, L, stage)
                    host.copy_(stage, non_blocking=True)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            step.attend(0)
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1))
        return float(np.mean(ts[2:]))
    out["attention_call_ms_alone"] = attention_ms(None)
    out["attention_call_ms_beside_offload_by_kernel_to_pinned_host"] = attention_ms("kernel")
    out["attention_call_ms_beside_offload_by_kernel_and_copy_engine"] = attention_ms("copy_engine")
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        B.alise_kv_swap_out(cache, bt, L, stage)
        host.copy_(stage, non_blocking=True)
    e1.record()
    torch.cuda.synchronize()
    out["copy_engine_offload_GBs"] = n / (e0.elapsed_time(e1) / 5 * 1e-3) / 1e9
    return out


MFMA_F16_PEAK_TFLOPS = 2500.0


def prefill_leg(w, step, every=8):
    """Chunked-prefill attention over the same cache (Sec. 2 "LLM Inference"), outside the timed
    steps: every `every`-th request brings its last min(512, L) tokens as a chunk of query tokens
    that attend causally over the request's quantized cache.  Bound: the fp16 matrix cores."""
    import numpy as np
    import torch
    from paper_2410_23537_amd import binding as B
    cache = step.caches[0]
    if w.D != 128 or w.P < 16 or w.H // w.Hkv > 16 or (w.bits == 8 and w.G < 64):
        return None                     # a layout without a matrix-core prefill kernel: its fallback on the single-query kernels is not benchmarked
    lens = step.lens.astype(np.int64)
    n = np.array([min(512, int(L)) if i % every == 0 else 0 for i, L in enumerate(lens)], np.int64)
    q_start = np.concatenate([[0], np.cumsum(n)]).astype(np.int32)
    total = int(q_start[-1])
    gen = torch.Generator(device="cuda").manual_seed(w.seed)
    q = torch.randn((total, w.H, w.D), dtype=torch.float16, device="cuda", generator=gen)
    out = torch.empty_like(q)
    bt = torch.from_numpy(step.pg.block_tables).cuda()
    lens_d = torch.from_numpy(step.lens.astype(np.int32)).cuda()
    qs = torch.from_numpy(q_start).cuda()
    ws = torch.empty(B.alise_paged_prefill_attn_workspace_bytes(cache, w.B, total, w.H, int(step.lens.max())), dtype=torch.uint8, device="cuda")
    pairs = sum(int((lens[i] - n[i] + np.arange(n[i]) + 1).sum()) for i in range(w.B) if n[i])
    flops = 4.0 * w.D * w.H * pairs     # q.k and p.v, a multiply and an add each, per (query, visible key, head)

    def run():
        B.alise_paged_prefill_attn(cache, q, out, qs, bt, lens_d, int(step.lens.max()), step.scale, ws)

    for _ in range(2):
        run()
    torch.cuda.synchronize()
    reps = 10
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        run()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    tflops = flops / (ms * 1e-3) / 1e12
    which = "every request" if every == 1 else f"every {every}th request"
    return {"workload": f"{which} of {w.name} brings its last min(512, L) tokens: {total} query tokens, "
                        f"{pairs} (query, visible key) pairs per head",
            "ms": ms, "flop": flops,
            "roofline": {"bound": "mfma", "achieved": tflops, "peak": MFMA_F16_PEAK_TFLOPS, "unit": "TFLOP/s",
                         "frac": tflops / MFMA_F16_PEAK_TFLOPS, "traffic": None}}


def graph_leg(step, total_bytes, steps):
    """The same step (quantize-and-write + attention + page dequantize) captured once in a HIP graph
    and replayed `steps` times: what a serving loop does to get rid of the launch gaps between the
    five kernels of a step.  The calls allocate nothing and read lengths, block tables and slots
    from device memory, so the captured graph stays valid when those change."""
    import torch
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step.step(0)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step.step(0)
    for _ in range(3):
        g.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        g.replay()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / steps * 1e3
    return {"ms_per_step": ms, "value": total_bytes / (ms * 1e-3) / 1e9, "unit": "GB/s",
            "pct_of_hbm_peak": 100.0 * total_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "note": "one captured step replayed; the headline figures above are the eager calls"}


def planned_leg(step, copies, b_attn, steps):
    """The attention call of one layer when the plan is made once per decode iteration
    (alise_paged_decode_attn_plan) and every layer runs alise_paged_decode_attn_planned on it."""
    import numpy as np
    import torch
    from paper_2410_23537_amd import binding as B
    B.alise_paged_decode_attn_plan(step.caches[0], step.context_lens, step.w.H, step.max_len, step.workspace)

    def run(c):
        B.alise_paged_decode_attn_planned(step.caches[c], step.q, step.out, step.block_tables, step.context_lens,
                                          step.max_len, step.scale, step.workspace)
    for s in range(3):
        run(s % copies)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for s, (e0, e1) in enumerate(ev):
        e0.record()
        run(s % copies)
        e1.record()
    torch.cuda.synchronize()
    ms = float(np.mean([e0.elapsed_time(e1) for e0, e1 in ev]))
    return {"ms": ms, "GBs": b_attn / (ms * 1e-3) / 1e9, "frac": b_attn / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "note": "alise_paged_decode_attn_planned: the layers of one decode iteration share the plan (their lengths are the same); "
                    "the headline figures above make the plan in every call"}


def iteration_graph_leg(step, copies, bytes_per_layer, n_layers=32, replays=5):
    """A decode iteration of n_layers attention layers as a serving loop runs it: one plan, then per layer the
    write of the new tokens and the planned attention call (the layers take the cache copies in turn), captured
    in a HIP graph and replayed."""
    import torch
    from paper_2410_23537_amd import binding as B

    def iteration():
        B.alise_paged_decode_attn_plan(step.caches[0], step.context_lens, step.w.H, step.max_len, step.workspace)
        for layer in range(n_layers):
            c = step.caches[layer % copies]
            B.alise_kv_quant_write(c, step.step_k, step.step_v, step.step_slots)
            B.alise_paged_decode_attn_planned(c, step.q, step.out, step.block_tables, step.context_lens, step.max_len,
                                              step.scale, step.workspace)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        iteration()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        iteration()
    g.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(replays):
        g.replay()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / replays / n_layers * 1e3
    return {"layers": n_layers, "ms_per_layer": ms, "value": bytes_per_layer / (ms * 1e-3) / 1e9, "unit": "GB/s",
            "pct_of_hbm_peak": 100.0 * bytes_per_layer / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "note": "write + attention per layer, one plan per iteration, one graph per iteration; no page dequantize"}


def read_ceiling_leg():
    """The second denominator: what a kernel that only reads sustains on this device (the library's
    streaming-read probe over 4 GiB, sixteen times the last-level cache), beside the published peak.
    Runs before the other legs, 3 warm-up + 10 timed calls."""
    import numpy as np
    import torch
    from paper_2410_23537_amd import binding as B
    src = torch.empty(1 << 32, dtype=torch.uint8, device="cuda")
    src.view(torch.int32).random_()
    out = torch.zeros(1, dtype=torch.int32, device="cuda")
    for _ in range(3):
        B.alise_hbm_read_probe(src, out)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(10)]
    for e0, e1 in ev:                       # back to back like the timed steps: no host wait in between
        e0.record()
        B.alise_hbm_read_probe(src, out)
        e1.record()
    torch.cuda.synchronize()
    ms = float(np.median([e0.elapsed_time(e1) for e0, e1 in ev]))
    return {"GBs": src.numel() / (ms * 1e-3) / 1e9, "bytes": src.numel(), "ms": ms,
            "note": "alise_hbm_read_probe over 4 GiB: 16-byte non-temporal loads from a persistent grid, two 8 KiB blocks in flight per wave, "
                    "nothing else; median of 10 calls, the call's two launches included"}


def issue_overlap_leg():
    """What bounds the matrix-core kernels: the library's issue probe (alise_issue_overlap_probe) with matrix instructions
    alone, vector instructions alone, and both in the same waves, two waves per SIMD.  If the two kinds ran side by side
    `both` would be the longer of the two; on this chip it is close to their sum, so a step of those kernels costs
    about the sum of its instruction times."""
    import torch
    from paper_2410_23537_amd import binding as B
    sink = torch.zeros(1, dtype=torch.float32, device="cuda")
    iters, out = 20000, {}
    for name, mode in (("mfma_only_ms", 1), ("valu_only_ms", 2), ("both_ms", 3)):
        B.alise_issue_overlap_probe(mode, 100, sink)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        B.alise_issue_overlap_probe(mode, iters, sink)
        e1.record()
        torch.cuda.synchronize()
        out[name] = e0.elapsed_time(e1)
    hidden = out["mfma_only_ms"] + out["valu_only_ms"] - out["both_ms"]
    out["overlap_fraction_of_the_shorter"] = hidden / min(out["mfma_only_ms"], out["valu_only_ms"])
    out["note"] = ("per wave and round: 16 v_mfma_f32_16x16x32_f16 and / or 64 v_fma_f32, independent chains, two waves per SIMD, "
                   f"{iters} rounds; 1.0 would mean the shorter kind is hidden behind the longer one, 0.0 that their times add up")
    return out


def quant_write_leg(w, tokens=65536):
    """Quantize-and-write of a prompt-sized batch (Sec. 3.2 "KV Compression"), outside the timed steps: `tokens` new tokens
    of this workload's shape written into pages of their own, whole prompts side by side in their pages.  The inputs
    (1-2 GB) do not fit the last-level cache, so every launch reads them from HBM.  Bound: HBM (read fp16, write codes
    and meta)."""
    import numpy as np
    import torch
    from paper_2410_23537_amd import binding as B
    from paper_2410_23537_amd import workloads as wl
    pages = tokens // w.P
    cache = B.KVCache.allocate(pages, w.P, w.Hkv, w.D, w.bits, w.G, fill=0)
    gen = torch.Generator(device="cuda").manual_seed(w.seed + 5)
    k = torch.randn((tokens, w.Hkv, w.D), dtype=torch.float16, device="cuda", generator=gen)
    v = torch.randn((tokens, w.Hkv, w.D), dtype=torch.float16, device="cuda", generator=gen)
    perm = torch.randperm(pages, device="cuda", generator=gen)
    t = torch.arange(tokens, device="cuda")
    slots = (perm[t // w.P] * w.P + t % w.P).to(torch.int64)
    for _ in range(2):
        B.alise_kv_quant_write(cache, k, v, slots)
    torch.cuda.synchronize()
    reps = 10
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for a, b in ev:
        a.record()
        B.alise_kv_quant_write(cache, k, v, slots)
        b.record()
    torch.cuda.synchronize()
    ms = float(np.mean([a.elapsed_time(b) for a, b in ev]))
    nbytes = wl.algorithmic_bytes_write(w, tokens)
    gbs = nbytes / (ms * 1e-3) / 1e9
    return {"workload": f"{tokens} tokens of {w.name}'s shape into {pages} pages in random order", "ms": ms, "bytes": nbytes,
            "roofline": {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
                         "traffic": None}}


def fused_ops_leg(w):
    """The two other fused operators of the layer (Sec. 3.3 "Implementation"), outside the timed
    steps, on a token batch of this workload's model: 16384 tokens (prefill chunks of an iteration;
    large enough that the matrices, 0.5 to 2.7 GB, cannot sit in the 256 MB last-level cache between
    repetitions), hidden = H * D, FFN width 4 * hidden.  Bound: HBM -- 8 bytes per element for the
    residual add + LayerNorm (x, residual in; sum, normalized row out), 4 for bias + ReLU in place."""
    import torch
    from paper_2410_23537_amd import binding as B
    rows, hidden = 16384, w.H * w.D
    gen = torch.Generator(device="cuda").manual_seed(w.seed + 1)
    mk = lambda *shape: torch.randn(shape, dtype=torch.float16, device="cuda", generator=gen)
    x, res, gamma, beta = mk(rows, hidden), mk(rows, hidden), mk(hidden), mk(hidden)
    h, y = torch.empty_like(x), torch.empty_like(x)
    f, fb = mk(rows, 4 * hidden), mk(4 * hidden)
    out = {}
    for name, fn, nbytes in (("add_layernorm", lambda: B.alise_add_layernorm(x, res, gamma, beta, 1e-5, h, y), 8 * rows * hidden),
                             ("bias_relu", lambda: B.alise_bias_relu(f, fb, f), 4 * rows * 4 * hidden)):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        reps = 20
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        gbs = nbytes / (ms * 1e-3) / 1e9
        out[name] = {"shape": [rows, hidden if name == "add_layernorm" else 4 * hidden], "ms": ms, "bytes": nbytes,
                     "roofline": {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                  "frac": gbs / HBM_PEAK_GBS, "traffic": None}}
    out["note"] = "a plain device-to-device copy (read + write) reaches about 5200 GB/s on this box"
    return out


def large_scheduled_run(w):
    """The scheduled run at a size where the kernels, not the launches, set the pace: 384 jobs with prompts of
    hundreds to thousands of tokens, batches of 128, 320 caches resident (74 offloads and uploads), through the C++ loop.  Reports the wall
    clock and what the decode batches streamed from the compressed cache while it ran."""
    import numpy as np
    import torch
    from paper_2410_23537_amd import binding as B
    from paper_2410_23537_amd import workloads as wl
    n_jobs, M, batch = 384, 320, 128
    arrival, s, n_true, n_pred = (a.tolist() for a in wl.job_trace(n_jobs, 29, mean_gap=400.0, max_prompt=4096, max_output=128,
                                                                    prompt_median=800.0, output_median=48.0))
    cfg = dict(num_queues=4, limit0=200000, age_threshold=5000000, max_batch=batch, gpu_job_limit=M, t0=2, alpha=1, beta=20)
    max_ctx = max(a + b for a, b in zip(s, n_true)) + 1
    pages_per_job = (max_ctx + w.P - 1) // w.P
    max_iter_tokens = sum(sorted(s)[-batch:])                     # no batch can bring more prompt tokens than its longest prompts
    pool_n = 1 << 16
    gen = torch.Generator(device="cuda").manual_seed(w.seed + 3)
    pk = torch.randn((pool_n + max_ctx, w.Hkv, w.D), dtype=torch.float16, device="cuda", generator=gen)
    pv = torch.randn((pool_n + max_ctx, w.Hkv, w.D), dtype=torch.float16, device="cuda", generator=gen)
    pq = torch.randn((pool_n + max_ctx, w.H, w.D), dtype=torch.float16, device="cuda", generator=gen)

    def run_once():
        cache = B.KVCache.allocate((M + batch + 1) * pages_per_job, w.P, w.Hkv, w.D, w.bits, w.G, fill=0)
        rp = B.NativeReplay(cache, w.H, cfg, max_ctx, max_iter_tokens, pk, pv, pq, 1.0 / math.sqrt(w.D))
        order = sorted(range(n_jobs), key=lambda i: (arrival[i], i))
        k, now, produced, attended = 0, 0, [0] * n_jobs, 0
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        while True:
            while k < n_jobs and arrival[order[k]] <= now:
                i = order[k]
                rp.add_job(i, arrival[i], s[i], n_pred[i], (i * 7919) % pool_n)
                k += 1
            if rp.num_jobs() == 0:
                if k == n_jobs:
                    break
                now = arrival[order[k]]
                continue
            d = rp.iterate()
            fin = []
            for id, ph in zip(d["batch"], d["phase"]):
                produced[id] += 1
                if ph == 1:
                    attended += s[id] + produced[id] - 1          # the tokens this decode step read from the cache
                if produced[id] >= n_true[id]:
                    fin.append(id)
            rp.commit(d["model_time"], fin)
            now += d["model_time"]
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        st = rp.stats()
        rp.close()
        return st, dt, attended

    run_once()
    st, dt, attended = run_once()
    streamed = attended * w.Hkv * w.row_bytes
    return {"workload": f"{n_jobs} jobs (log-normal prompts, median 800, <= 4096; outputs, median 48, <= 128; 15 % underpredicted 4x), "
                        f"batch {batch}, GPU job limit {M}, 4 queues; one attention layer of {w.name}'s shape, the C++ loop",
            "seconds": dt, "iterations": st["iterations"], "iterations_per_s": st["iterations"] / dt,
            "prefill_tokens": st["prefill_tokens"], "decode_tokens": st["decode_tokens"],
            "tokens_per_s": (st["prefill_tokens"] + st["decode_tokens"]) / dt,
            "offloads": st["offloads"], "uploads": st["uploads"], "swapped_bytes": st["offload_bytes"] + st["upload_bytes"],
            "decode_kv_tokens_attended": attended, "decode_cache_GB_streamed": streamed / 1e9,
            "decode_cache_GBs_over_the_whole_run": streamed / dt / 1e9,
            "note": "wall clock of the whole run (prefill, writes, swaps and the host included), second run of the trace; "
                    "the last figure divides the cache bytes the decode batches read by that wall clock"}


def scheduled_run_leg(w, python_loop=True, which=None):
    """The host-side scheduler (Sec. 3.1 "Preemptive Scheduling", Sec. 3.2 Alg. 2) outside the timed
    steps: (1) decisions per second of the C++ scheduler alone on 1024 live jobs; (2) a scheduled
    run of 192 synthetic jobs through one attention layer of this workload's shape on the GPU --
    prompts through quantize-and-write + chunked prefill, every later token through
    quantize-and-write + decode attention, preempted jobs offloaded to pinned host memory and
    uploaded again as Alg. 2 decides -- with the wall clock around it, once through the C++ loop of
    alise_replay.h and once through the Python loop of replay.py."""
    import numpy as np
    import torch
    from paper_2410_23537_amd import binding as B
    from paper_2410_23537_amd import workloads as wl
    from paper_2410_23537_amd.replay import Replay
    out = {}
    # ---- (1) the scheduler alone
    cfg = dict(num_queues=4, limit0=4000, age_threshold=400000, max_batch=64, gpu_job_limit=256, t0=2, alpha=1, beta=20)
    arrival, s, n_true, n_pred = (a.tolist() for a in wl.job_trace(1024, 3, mean_gap=0.0, max_prompt=2048, max_output=100000))
    sched = B.Scheduler(**cfg, want_order=False)
    for i in range(1024):
        sched.add_job(i, 0, s[i], max(n_pred[i], 4096))           # nobody finishes or is demoted during the timing
    for _ in range(20):
        sched.commit(sched.step()["model_time"], [])
    reps = 300
    t0 = time.perf_counter()
    for _ in range(reps):
        sched.commit(sched.step()["model_time"], [])
    dt = time.perf_counter() - t0
    out["scheduler_alone"] = {"live_jobs": 1024, "us_per_iteration": dt / reps * 1e6,
                              "note": "alise_sched_step + alise_sched_commit through ctypes, 1024 live jobs, batch 64, M 256"}
    # ---- (2) a scheduled run on the GPU
    if w.D != 128 or w.P < 16 or w.H // w.Hkv > 16 or (w.bits == 8 and w.G < 64):
        out["scheduled_run"] = None             # no matrix-core prefill kernel for this layout: not benchmarked
        return out
    n_jobs, M, batch = 192, 48, 32
    arrival, s, n_true, n_pred = (a.tolist() for a in wl.job_trace(n_jobs, 17, mean_gap=120.0, max_prompt=1024, max_output=96))
    cfg = dict(num_queues=4, limit0=8000, age_threshold=200000, max_batch=batch, gpu_job_limit=M, t0=2, alpha=1, beta=20)
    max_ctx = max(a + b for a, b in zip(s, n_true)) + 1
    pages_per_job = (max_ctx + w.P - 1) // w.P
    pool_n = 1 << 16
    gen = torch.Generator(device="cuda").manual_seed(w.seed + 2)
    pk = torch.randn((pool_n + max_ctx, w.Hkv, w.D), dtype=torch.float16, device="cuda", generator=gen)
    pv = torch.randn((pool_n + max_ctx, w.Hkv, w.D), dtype=torch.float16, device="cuda", generator=gen)
    pq = torch.randn((pool_n + max_ctx, w.H, w.D), dtype=torch.float16, device="cuda", generator=gen)

    def source(spans):
        # rows of the pools, gathered with one index per iteration
        idx = torch.from_numpy(np.concatenate([np.arange((id * 7919) % pool_n + a, (id * 7919) % pool_n + b) for id, a, b in spans])).cuda()
        return pk.index_select(0, idx), pv.index_select(0, idx), pq.index_select(0, idx)

    def drive(add_job, num_jobs, iterate, commit):
        order = sorted(range(n_jobs), key=lambda i: (arrival[i], i))
        k, now, produced = 0, 0, [0] * n_jobs
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        while True:
            while k < n_jobs and arrival[order[k]] <= now:
                i = order[k]
                add_job(i)
                k += 1
            if num_jobs() == 0:
                if k == n_jobs:
                    break
                now = arrival[order[k]]
                continue
            d = iterate()
            fin = []
            for id in d["batch"]:
                produced[id] += 1
                if produced[id] >= n_true[id]:
                    fin.append(id)
            commit(d["model_time"], fin)
            now += d["model_time"]
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    def run_python():
        rp = Replay(w, B.Scheduler(**cfg, want_order=False), num_pages=2 * (M + 1) * pages_per_job, max_context=max_ctx, kv_source=source)
        dt = drive(lambda i: rp.add_job(i, arrival[i], s[i], n_pred[i]), rp.sched.num_jobs, rp.iterate, rp.commit)
        return rp.stats, dt

    def run_native():
        cache = B.KVCache.allocate(2 * (M + 1) * pages_per_job, w.P, w.Hkv, w.D, w.bits, w.G, fill=0)
        rp = B.NativeReplay(cache, w.H, cfg, max_ctx, batch * max(s), pk, pv, pq, 1.0 / math.sqrt(w.D))
        dt = drive(lambda i: rp.add_job(i, arrival[i], s[i], n_pred[i], (i * 7919) % pool_n), rp.num_jobs, rp.iterate, rp.commit)
        st = rp.stats()
        rp.close()
        return st, dt

    def report(st, dt, note):
        return {"seconds": dt, "iterations": st["iterations"], "iterations_per_s": st["iterations"] / dt,
                "prefill_tokens": st["prefill_tokens"], "decode_tokens": st["decode_tokens"],
                "tokens_per_s": (st["prefill_tokens"] + st["decode_tokens"]) / dt,
                "offloads": st["offloads"], "uploads": st["uploads"], "swapped_bytes": st["offload_bytes"] + st["upload_bytes"],
                "note": note}

    what = (f"{n_jobs} jobs (Poisson arrivals, log-normal prompts <= 1024 and outputs <= 96, 15 % underpredicted 4x), "
            f"batch {batch}, GPU job limit {M}, 4 queues; one attention layer of {w.name}'s shape")
    if which != "large":
        run_native()                # the first run pays for pinned allocations and one-time queries
        st, dt = run_native()
        out["scheduled_run"] = dict(workload=what, **report(
            st, dt, "the C++ loop of alise_replay.h (one call per iteration from the driver, no host synchronisation inside), "
                    "second run of the same trace; the clock the scheduler sees is its own model time"))
    if which != "small":
        out["scheduled_run_large"] = large_scheduled_run(w)
    if not python_loop:
        return out
    run_python()
    st, dt = run_python()
    out["scheduled_run_python_loop"] = report(st, dt, "the same trace through replay.py, the Python loop around the same entry points")
    return out


def cache_copies(w):
    """Copies of the cache the steps rotate over: enough distinct addresses that a step's working set (at least 1 GiB
    in total) cannot be served from the 256 MB last-level cache by the step before it."""
    import numpy as np
    from paper_2410_23537_amd import workloads as wl
    working_set = int(wl.context_lens(w).astype(np.int64).sum()) * w.Hkv * w.row_bytes
    copies = 1 if working_set >= (1 << 30) else int(math.ceil((1 << 30) / max(working_set, 1))) + 1
    return min(copies, 64)


def time_steps(step, copies, steps, warmup):
    """`warmup` untimed steps, then exactly `steps` timed ones between two synchronisations; HIP events on the stream
    of the calls (torch's current stream) around every write and every attention call."""
    import numpy as np
    import torch
    for s in range(warmup):
        step.step(s % copies)
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    evw = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(steps):
        c = s % copies
        evw[s][0].record()
        step.quant_write(c)
        evw[s][1].record()
        ev[s][0].record()
        step.attend(c)
        ev[s][1].record()
        step.dequant_page(c)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    attn_all = [a.elapsed_time(b) for a, b in ev]
    return {"ms_per_step": elapsed / steps * 1e3, "attn_all": attn_all, "attn_ms": float(np.mean(attn_all)),
            "write_ms": float(np.mean([a.elapsed_time(b) for a, b in evw]))}


def other_config_leg(name, steps, warmup):
    """The same eager step on one of the other benchmark configurations, built, timed and freed: the step time,
    the attention call's time and roofline, KV tokens per second."""
    import torch
    from paper_2410_23537_amd import workloads as wl
    from paper_2410_23537_amd.decode_step import DecodeStep
    w = wl.CONFIGS[name]
    copies = cache_copies(w)
    step = DecodeStep(w, n_cache_copies=copies)
    step.populate()
    t = time_steps(step, copies, steps, warmup)
    b_attn, b_write, b_dq = step.bytes_attn(), step.bytes_write(), step.bytes_dequant()
    total = b_attn + b_write + b_dq
    achieved = b_attn / (t["attn_ms"] * 1e-3) / 1e9
    traffic, note = measured_traffic(name)
    out = {"workload": f"{w.name}: B={w.B} H={w.H} Hkv={w.Hkv} D={w.D} page={w.P} INT{w.bits} G={w.G} "
                       f"lengths={w.length_law} sum(L)={step.kv_tokens()}",
           "step_tokens_written": int(step.step_slots.numel()), "cache_copies_rotated": copies,
           "ms_per_step": t["ms_per_step"], "value": total / (t["ms_per_step"] * 1e-3) / 1e9, "unit": "GB/s",
           "pct_of_hbm_peak": 100.0 * total / (t["ms_per_step"] * 1e-3) / 1e9 / HBM_PEAK_GBS,
           "kv_tokens_per_s": step.kv_tokens() / (t["ms_per_step"] * 1e-3),
           "attention_call_ms": t["attn_ms"], "attention_call_ms_min": float(min(t["attn_all"])), "quant_write_ms": t["write_ms"],
           "bytes_per_step": {"attn": b_attn, "quant_write": b_write, "dequant_page": b_dq},
           "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                        "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_note": note}}
    del step
    torch.cuda.empty_cache()
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus above 1 is not supported "
              "(the path would shard by request or by KV head, without any exchange between the GPUs)", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2410_23537_amd import workloads as wl
    from paper_2410_23537_amd.decode_step import DecodeStep

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    torch.cuda.set_device(0)
    w = wl.CONFIGS[args.workload]
    copies = cache_copies(w)
    t_setup = time.perf_counter()
    step = DecodeStep(w, n_cache_copies=copies)
    step.populate()
    torch.cuda.synchronize()
    print(f"[bench] workload {w.name}: B={w.B} H={w.H} Hkv={w.Hkv} D={w.D} P={w.P} bits={w.bits} G={w.G} "
          f"sum(L)={step.kv_tokens()} step tokens={int(step.step_slots.numel())} cache copies={copies} "
          f"setup {time.perf_counter() - t_setup:.1f}s", file=sys.stderr, flush=True)

    timed = time_steps(step, copies, args.steps, args.warmup)
    ms_per_step, attn_all, attn_ms, write_ms = timed["ms_per_step"], timed["attn_all"], timed["attn_ms"], timed["write_ms"]

    if args.traffic_calibration:
        src = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(2):
            torch.add(src, 1.0, out=dst)
        torch.cuda.synchronize()

    b_attn, b_write, b_dq = step.bytes_attn(), step.bytes_write(), step.bytes_dequant()
    total_bytes = b_attn + b_write + b_dq
    value = total_bytes / (ms_per_step * 1e-3) / 1e9
    achieved = b_attn / (attn_ms * 1e-3) / 1e9
    traffic, traffic_note = measured_traffic(w.name)
    result = {
        "metric": "quantized-KV decode attention HBM GB/s (% of peak) + KV-tokens/s attended",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: B={w.B} H={w.H} Hkv={w.Hkv} D={w.D} page={w.P} INT{w.bits} G={w.G} "
                               f"lengths={w.length_law} sum(L)={step.kv_tokens()}",
                   "step": "quant_write(step tokens) + paged_decode_attn + dequant_page(1)",
                   "step_tokens_written": int(step.step_slots.numel()), "cache_copies_rotated": copies},
        "pct_of_hbm_peak": 100.0 * value / HBM_PEAK_GBS,
        "kv_tokens_per_s": step.kv_tokens() / (ms_per_step * 1e-3),
        "bytes_per_step": {"attn": b_attn, "quant_write": b_write, "dequant_page": b_dq},
        "kernel_ms": {"paged_decode_attn": attn_ms, "quant_write": write_ms,
                      "paged_decode_attn_min": float(np.min(attn_all)), "paged_decode_attn_median": float(np.median(attn_all))},
        "roofline": {"bound": "hbm",
                     "kernel": "alise_paged_decode_attn = plan_kernel + decode_attn(_gqa)_kernel + merge_kernel, "
                               "timed as one call; the attention kernel is >97 % of it",
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_note": traffic_note,
                     "attention_sources_sha256": attention_sources_sha256()},
    }
    if args.only_prefill:
        result["prefill_full_batch"] = prefill_leg(w, step, every=1)
    elif args.only_scheduler:
        result["scheduler"] = scheduled_run_leg(w, python_loop=False, which=args.only_scheduler)
    elif not args.only_steps:
        ceiling = read_ceiling_leg()
        result["hbm_read_ceiling"] = ceiling
        result["roofline"]["frac_of_read_ceiling"] = achieved / ceiling["GBs"]
        result["planned_attention"] = planned_leg(step, copies, b_attn, args.steps)
        result["graph_replay"] = graph_leg(step, total_bytes, args.steps)
        result["iteration_graph"] = iteration_graph_leg(step, copies, b_attn + b_write)
        result["swap"] = swap_leg(step)
        prefill = prefill_leg(w, step)
        if prefill is not None:
            result["prefill"] = prefill
            result["prefill_full_batch"] = prefill_leg(w, step, every=1)      # the same with a grid that fills the chip
            from paper_2410_23537_amd import binding as _B
            os.environ["ALISE_PREFILL_WEIGHTS"] = "single"                    # the library reads its environment on request
            _B.alise_reload_environment()
            fast = prefill_leg(w, step, every=1)
            del os.environ["ALISE_PREFILL_WEIGHTS"]
            _B.alise_reload_environment()
            fast["note"] = ("ALISE_PREFILL_WEIGHTS=single: one rounded fp16 number per softmax weight instead of a high and "
                            "a low part; adds up to 2^-12 max|v| to the error, not the default")
            result["prefill_full_batch_single_weight"] = fast
        if args.workload == "int4":
            # the other three benchmark configurations, one after another (each built, timed and freed)
            result["all_configs"] = {n: other_config_leg(n, args.steps, args.warmup) for n in ("opt13b", "llama7b", "gqa70b")}
        result["quant_write_large"] = quant_write_leg(w)
        result["issue_overlap"] = issue_overlap_leg()
        result["fused_ops"] = fused_ops_leg(w)
        result["scheduler"] = scheduled_run_leg(w)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w, step, args.cpu_seconds)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
