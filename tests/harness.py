"""Shared set-up for the GPU parity tests: builds the same seeded problem on the
host (oracle cache) and on the device (HIP cache), each filled by its own writer."""
from __future__ import annotations

import numpy as np

from paper_2410_23537_amd import workloads as wl


def fill_oracle_cache(oracle_mod, w, pg, pool, offs, gain):
    cache = oracle_mod.Cache.empty(pg.num_pages, w.P, w.Hkv, w.D, w.bits, w.G, fill=0xFF)
    cache.k_meta.view(np.uint16)[:] = 0x7E00      # NaN
    cache.v_meta.view(np.uint16)[:] = 0x7E00
    for i, L in enumerate(pg.lens):
        if L <= 0:
            continue
        k, v = wl.request_kv(w, pool, offs, i, 0, int(L), gain)
        oracle_mod.kv_quant_write(cache, k, v, wl.slots_of(w, pg, i, 0, int(L)))
    return cache


def fill_device_cache(B, torch, w, pg, pool, offs, gain, max_tokens_per_call=1 << 16, layout="interleaved"):
    """Poisoned device cache (0xFF codes, NaN meta) filled through alise_kv_quant_write."""
    cache = B.KVCache.allocate(pg.num_pages, w.P, w.Hkv, w.D, w.bits, w.G, fill=0xFF, layout=layout)
    cache.k_meta.view(torch.int16).fill_(0x7E00)  # NaN, same bit pattern as on the host
    cache.v_meta.view(torch.int16).fill_(0x7E00)
    ks, vs, ss, n = [], [], [], 0

    def flush():
        nonlocal ks, vs, ss, n
        if n == 0:
            return
        k = torch.from_numpy(np.concatenate(ks)).cuda()
        v = torch.from_numpy(np.concatenate(vs)).cuda()
        s = torch.from_numpy(np.concatenate(ss)).cuda()
        B.alise_kv_quant_write(cache, k, v, s)
        torch.cuda.synchronize()
        ks, vs, ss, n = [], [], [], 0

    for i, L in enumerate(pg.lens):
        L = int(L)
        for t0 in range(0, L, max_tokens_per_call):
            t1 = min(L, t0 + max_tokens_per_call)
            k, v = wl.request_kv(w, pool, offs, i, t0, t1, gain)
            ks.append(k)
            vs.append(v)
            ss.append(wl.slots_of(w, pg, i, t0, t1))
            n += t1 - t0
            if n >= max_tokens_per_call:
                flush()
    flush()
    return cache


def written_mask(w, pg):
    """bool [num_pages, P]: slots that hold a token of some request."""
    m = np.zeros((pg.num_pages, w.P), bool)
    for i, L in enumerate(pg.lens):
        if L > 0:
            s = wl.slots_of(w, pg, i, 0, int(L))
            m[s // w.P, s % w.P] = True
    return m


def run_device_attn(B, torch, w, cache, q_np, pg, max_len=None):
    q = torch.from_numpy(q_np).cuda()
    out = torch.full(q.shape, float("nan"), dtype=torch.float16, device="cuda")
    bt = torch.from_numpy(pg.block_tables).cuda()
    lens = torch.from_numpy(pg.lens.astype(np.int32)).cuda()
    max_len = int(max(1, pg.lens.max(initial=0))) if max_len is None else max_len
    nbytes = B.alise_paged_decode_attn_workspace_bytes(cache, q.shape[0], q.shape[1], max_len)
    assert nbytes > 0
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    B.alise_paged_decode_attn(cache, q, out, bt, lens, max_len, 1.0 / np.sqrt(w.D), ws)
    torch.cuda.synchronize()
    return out.cpu().numpy()
