"""Runs the scheduler's decisions through the GPU path: one attention layer's worth of every
iteration that the speculative scheduler of ALISE plans (Sec. 3.1 "Preemptive Scheduling"), with
the KV caches of preempted jobs moved by the swap calls as Alg. 2 decides (Sec. 3.2 "Dynamic
Swapping"), overlapped with the iteration's compute on a second stream.

Per iteration: offload the jobs that lost their place (their pages are free again one iteration
later), upload the ones that got one, quantize-and-write the new K/V of the batch (whole prompts
for jobs in their first iteration, one token for the others), then chunked-prefill attention for
the former and single-query attention for the latter.  This module is plumbing: a page free
list, block tables, pinned host buffers, streams and events.  Every decision comes from the
scheduler object of the library, every byte is touched by the library's kernels.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np
import torch

from . import binding as B


@dataclass
class _Job:
    s: int                              # prompt length
    L: int = 0                          # tokens in the cache
    pages: list = field(default_factory=list)
    host: torch.Tensor | None = None    # the offloaded form, pinned host memory
    host_bytes: int = 0


class Replay:
    """kv_source(spans) -> (k, v, q): spans is a list of (job_id, t0, t1); the answer holds, span after
    span, the device fp16 tensors [tokens, Hkv, D], same, and [tokens, H, D] of the jobs' tokens
    t0 .. t1 - 1 (prompt tokens first, then generated ones).  One call per iteration."""

    def __init__(self, shape, sched: B.Scheduler, num_pages: int, max_context: int, kv_source, overlap_swaps: bool = True):
        self.w = shape
        self.sched = sched
        self.kv_source = kv_source
        self.cache = B.KVCache.allocate(num_pages, shape.P, shape.Hkv, shape.D, shape.bits, shape.G, fill=0)
        if B.alise_paged_prefill_attn_workspace_bytes(self.cache, 1, 1, shape.H, max_context) == 0:
            raise ValueError("unsupported cache layout")
        self.free = list(range(num_pages - 1, -1, -1))
        self.pending_free: list[int] = []
        self.max_context = max_context
        self.max_blocks = (max_context + shape.P - 1) // shape.P
        self.jobs: dict[int, _Job] = {}
        self.scale = 1.0 / math.sqrt(shape.D)
        self.main = torch.cuda.current_stream()
        self.side = torch.cuda.Stream() if overlap_swaps else self.main
        self.iter_done = torch.cuda.Event()
        self.swap_done = torch.cuda.Event()
        self.iter_done.record(self.main)
        self.swap_done.record(self.side)
        # offloads and uploads go through device memory: the kernels gather and scatter there, the copy engine moves the
        # bytes over the host link (a kernel that touches host memory itself slows the attention call beside it)
        self._swap_stage = torch.empty(B.alise_kv_swap_bytes(self.cache, max_context), dtype=torch.uint8, device="cuda")
        self._ws_dec = torch.empty(0, dtype=torch.uint8, device="cuda")
        self._ws_pre = torch.empty(0, dtype=torch.uint8, device="cuda")
        self._host_pool: dict[int, list] = {}
        self.stats = {"iterations": 0, "prefill_tokens": 0, "decode_tokens": 0, "offloads": 0, "uploads": 0,
                      "offload_bytes": 0, "upload_bytes": 0}

    # ---- bookkeeping
    def add_job(self, id: int, arrival: int, prompt_len: int, predicted_len: int) -> None:
        assert prompt_len + 1 <= self.max_context
        self.sched.add_job(id, arrival, prompt_len, predicted_len)
        self.jobs[id] = _Job(s=prompt_len)

    def _alloc(self, n: int) -> list:
        if n > len(self.free):
            raise RuntimeError(f"out of KV pages: {n} wanted, {len(self.free)} free (size the pool for the GPU job limit)")
        return [self.free.pop() for _ in range(n)]

    def _host_buffer(self, nbytes: int) -> torch.Tensor:
        cls = 1 << max(12, (nbytes - 1).bit_length())            # pinned buffers are recycled by power-of-two size
        pool = self._host_pool.setdefault(cls, [])
        return pool.pop() if pool else torch.empty(cls, dtype=torch.uint8, pin_memory=True)

    def _release_host(self, t: torch.Tensor) -> None:
        self._host_pool.setdefault(t.numel(), []).append(t)

    def _bt(self, ids) -> torch.Tensor:
        m = np.zeros((len(ids), self.max_blocks), np.int32)
        for r, id in enumerate(ids):
            p = self.jobs[id].pages
            m[r, :len(p)] = p
        return torch.from_numpy(m).cuda()

    def _workspace(self, which: str, nbytes: int) -> torch.Tensor:
        cur = getattr(self, which)
        if cur.numel() < nbytes:
            cur = torch.empty(int(nbytes * 1.5) + 256, dtype=torch.uint8, device="cuda")
            setattr(self, which, cur)
        return cur

    # ---- one iteration
    def iterate(self) -> dict:
        """Plans and runs one iteration.  Returns the decision plus 'prefill_ids', 'prefill_out'
        (fp16 [sum of prompt lengths, H, D]), 'decode_ids', 'decode_out' (fp16 [n, H, D]) and
        'offloaded' (id -> (pinned tensor, bytes)).  Call commit() next."""
        w, cache = self.w, self.cache
        d = self.sched.step()
        # pages given up by the offloads of the last iteration: every later writer is ordered behind those copies
        self.main.wait_event(self.swap_done)
        self.free.extend(self.pending_free)
        self.pending_free = []
        self.side.wait_event(self.iter_done)                     # the swaps see what the last iteration wrote

        offloaded = {}
        with torch.cuda.stream(self.side):
            for id in d["offload"]:
                j = self.jobs[id]
                n = B.alise_kv_swap_bytes(cache, j.L)
                buf = self._host_buffer(n)
                B.alise_kv_swap_out(cache, torch.tensor(j.pages, dtype=torch.int32, device="cuda"), j.L, self._swap_stage[:n])
                buf[:n].copy_(self._swap_stage[:n], non_blocking=True)
                self.pending_free.extend(j.pages)
                j.pages, j.host, j.host_bytes = [], buf, n
                offloaded[id] = (buf, n)
                self.stats["offloads"] += 1
                self.stats["offload_bytes"] += n
            for id in d["upload"]:
                j = self.jobs[id]
                j.pages = self._alloc((j.L + w.P - 1) // w.P)
                self._swap_stage[:j.host_bytes].copy_(j.host[:j.host_bytes], non_blocking=True)
                B.alise_kv_swap_in(cache, torch.tensor(j.pages, dtype=torch.int32, device="cuda"), j.L, self._swap_stage[:j.host_bytes])
                self.stats["uploads"] += 1
                self.stats["upload_bytes"] += j.host_bytes
            self.swap_done.record(self.side)
        in_batch = set(d["batch"])
        if any(id in in_batch for id in d["upload"]):
            self.main.wait_event(self.swap_done)                 # a job that runs now needs its cache back first
        # the uploaded jobs' host buffers are free once the copies are done; recycled at commit()
        self._uploaded = [self.jobs[id] for id in d["upload"]]

        # ---- new K/V of the batch: whole prompts (phase 0), one token (phase 1)
        pre = [id for id, ph in zip(d["batch"], d["phase"]) if ph == 0]
        dec = [id for id, ph in zip(d["batch"], d["phase"]) if ph == 1]
        spans, slots = [], []
        for id in pre + dec:
            j = self.jobs[id]
            t0, t1 = (0, j.s) if j.L == 0 else (j.L, j.L + 1)
            need = (t1 + w.P - 1) // w.P - len(j.pages)
            if need > 0:
                j.pages.extend(self._alloc(need))
            spans.append((id, t0, t1))
            t = np.arange(t0, t1)
            slots.append(np.asarray(j.pages, np.int64)[t // w.P] * w.P + t % w.P)
            j.L = t1
        out = dict(d)
        out.update(prefill_ids=pre, decode_ids=dec, prefill_out=None, decode_out=None, offloaded=offloaded)
        n_pre = sum(self.jobs[id].s for id in pre)
        if spans:
            k_all, v_all, q_all = self.kv_source(spans)
            B.alise_kv_quant_write(cache, k_all, v_all, torch.from_numpy(np.concatenate(slots)).cuda())
        if pre:
            lens = np.array([self.jobs[id].L for id in pre], np.int32)
            q_start = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
            q = q_all[:n_pre]
            o = torch.empty_like(q)
            ws = self._workspace("_ws_pre", B.alise_paged_prefill_attn_workspace_bytes(cache, len(pre), int(q_start[-1]), w.H, int(lens.max())))
            B.alise_paged_prefill_attn(cache, q, o, torch.from_numpy(q_start).cuda(), self._bt(pre), torch.from_numpy(lens).cuda(),
                                       int(lens.max()), self.scale, ws)
            out["prefill_out"] = o
            self.stats["prefill_tokens"] += int(q_start[-1])
        if dec:
            lens = np.array([self.jobs[id].L for id in dec], np.int32)
            q = q_all[n_pre:]
            o = torch.empty_like(q)
            ws = self._workspace("_ws_dec", B.alise_paged_decode_attn_workspace_bytes(cache, len(dec), w.H, int(lens.max())))
            B.alise_paged_decode_attn(cache, q, o, self._bt(dec), torch.from_numpy(lens).cuda(), int(lens.max()), self.scale, ws)
            out["decode_out"] = o
            self.stats["decode_tokens"] += len(dec)
        self.iter_done.record(self.main)
        self.stats["iterations"] += 1
        return out

    def commit(self, elapsed: int, finished) -> None:
        self.sched.commit(elapsed, list(finished))
        if self._uploaded:
            self.swap_done.synchronize()                         # the host buffers are read by the upload copies until here
            for j in self._uploaded:
                self._release_host(j.host)
                j.host, j.host_bytes = None, 0
            self._uploaded = []
        for id in finished:
            j = self.jobs.pop(id)
            self.pending_free.extend(j.pages)                    # the iteration that read them is ordered before any reuse
