"""One decode step of a synthetic serving batch on the device, driven through the C ABI.

This is glue for ``bench.py`` and the full-size GPU tests: it places a seeded
workload (``workloads.py``) in device memory, fills the compressed cache through
``alise_kv_quant_write`` and replays the step the paper's decode iteration performs
(Sec. 2, "LLM Inference": append the new token's K/V, then attend over the cache;
Sec. 3.2: the cache holds b-bit codes).  torch is used for device memory, slicing
of the input pool and events only; every operation of the method runs in the HIP
library.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B
from . import workloads as wl


class DecodeStep:
    def __init__(self, w: wl.Workload, n_cache_copies: int = 1, device: str = "cuda", layout: str = "interleaved"):
        self.w = w
        self.device = device
        self.pg = wl.paging(w)
        self.lens = self.pg.lens
        self.offs = wl.request_offsets(w)
        self.gain = wl.k_channel_gain(w)
        self.pool_host = wl.value_pool(w, n_min=int(self.lens.max()) * w.Hkv * w.D)
        self.pool = torch.from_numpy(self.pool_host).to(device)
        self.gain_dev = torch.from_numpy(self.gain).to(device) if w.outlier_frac > 0 else None
        self.q_host = wl.queries(w)
        self.q = torch.from_numpy(self.q_host).to(device)
        self.out = torch.zeros_like(self.q)
        self.block_tables = torch.from_numpy(self.pg.block_tables).to(device)
        self.context_lens = torch.from_numpy(self.lens.astype(np.int32)).to(device)
        self.max_len = int(self.lens.max())
        self.scale = 1.0 / float(np.sqrt(w.D))
        self.caches = [B.KVCache.allocate(self.pg.num_pages, w.P, w.Hkv, w.D, w.bits, w.G, device=device, layout=layout)
                       for _ in range(n_cache_copies)]
        nbytes = B.alise_paged_decode_attn_workspace_bytes(self.caches[0], w.B, w.H, self.max_len)
        if nbytes == 0:
            raise RuntimeError("unsupported workload shape")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=device)
        # the tokens the timed quantize-and-write call stores
        req, pos = wl.step_tokens(w, self.lens)
        self.step_req, self.step_pos = req, pos
        self.step_k, self.step_v = self._gather_tokens(req, pos)
        slots = self.pg.block_tables[req, pos // w.P].astype(np.int64) * w.P + (pos % w.P)
        self.step_slots = torch.from_numpy(slots).to(device)
        self.dq_page = int(self.pg.block_tables[int(np.argmax(self.lens)), 0])
        self.dq_k = torch.empty((w.P, w.Hkv, w.D), dtype=torch.float16, device=device)
        self.dq_v = torch.empty_like(self.dq_k)

    # -- inputs ---------------------------------------------------------------
    def _kv_range(self, i: int, t0: int, t1: int):
        """Device views (no copy unless K carries channel gains) of tokens t0..t1-1 of request i."""
        w = self.w
        row = w.Hkv * w.D
        ko = int(self.offs[0][i]) + t0 * row
        vo = int(self.offs[1][i]) + t0 * row
        n = (t1 - t0) * row
        k = self.pool[ko:ko + n].view(t1 - t0, w.Hkv, w.D)
        v = self.pool[vo:vo + n].view(t1 - t0, w.Hkv, w.D)
        if self.gain_dev is not None:
            k = (k.float() * self.gain_dev[None]).half()
        return k, v

    def _gather_tokens(self, req: np.ndarray, pos: np.ndarray):
        w = self.w
        row = w.Hkv * w.D
        ar = torch.arange(row, device=self.device, dtype=torch.int64)[None]
        ko = torch.from_numpy(self.offs[0][req] + pos.astype(np.int64) * row).to(self.device)[:, None] + ar
        vo = torch.from_numpy(self.offs[1][req] + pos.astype(np.int64) * row).to(self.device)[:, None] + ar
        k = self.pool[ko].view(-1, w.Hkv, w.D)
        v = self.pool[vo].view(-1, w.Hkv, w.D)
        if self.gain_dev is not None:
            k = (k.float() * self.gain_dev[None]).half()
        return k.contiguous(), v.contiguous()

    def populate(self, include_step_tokens: bool = False, max_tokens_per_call: int = 1 << 15) -> None:
        """Fill every cache copy with the context of every request through alise_kv_quant_write
        (untimed set-up).  The tokens of the timed step are left to ``step()`` unless asked for."""
        w = self.w
        for i, L in enumerate(self.lens):
            L = int(L)
            first_step_pos = L
            if not include_step_tokens:
                mine = self.step_pos[self.step_req == i]
                first_step_pos = int(mine.min()) if mine.size else L
            for t0 in range(0, first_step_pos, max_tokens_per_call):
                t1 = min(first_step_pos, t0 + max_tokens_per_call)
                k, v = self._kv_range(i, t0, t1)
                slots = torch.from_numpy(wl.slots_of(w, self.pg, i, t0, t1)).to(self.device)
                for c in self.caches:
                    B.alise_kv_quant_write(c, k.contiguous(), v.contiguous(), slots)
        torch.cuda.synchronize()

    # -- the step -------------------------------------------------------------
    def quant_write(self, copy: int = 0) -> None:
        B.alise_kv_quant_write(self.caches[copy], self.step_k, self.step_v, self.step_slots)

    def attend(self, copy: int = 0) -> None:
        B.alise_paged_decode_attn(self.caches[copy], self.q, self.out, self.block_tables, self.context_lens,
                                  self.max_len, self.scale, self.workspace)

    def dequant_page(self, copy: int = 0) -> None:
        B.alise_kv_dequant_page(self.caches[copy], self.dq_page, self.dq_k, self.dq_v)

    def step(self, copy: int = 0) -> None:
        self.quant_write(copy)
        self.attend(copy)
        self.dequant_page(copy)

    # -- accounting -----------------------------------------------------------
    def bytes_attn(self) -> int:
        return wl.algorithmic_bytes_attn(self.w, self.lens)

    def bytes_write(self) -> int:
        return wl.algorithmic_bytes_write(self.w, int(self.step_slots.numel()))

    def bytes_dequant(self) -> int:
        return wl.algorithmic_bytes_dequant(self.w, 1)

    def kv_tokens(self) -> int:
        return int(self.lens.astype(np.int64).sum())
