"""Run-to-run determinism on the device: every kernel gives the work out in a fixed order (static item
lists, no counters; partial results merged in tile order), so a call repeated on the same inputs must
return the same bytes -- codes and meta of a write, every attention row of the vector, the matrix-core
and the prefill kernels, an offloaded request.  A difference would mean an order that depends on timing
(or a read of something another wave has not finished writing)."""
import numpy as np
import pytest

from paper_2410_23537_amd import workloads as wl
from tests import harness

pytestmark = pytest.mark.gpu

LAYOUTS = [
    wl.replace(wl.scaled(wl.CONFIGS["llama7b"], B=24, max_len=3000, name="mha_int8"), Hkv=4, H=4),
    wl.replace(wl.scaled(wl.CONFIGS["int4"], B=40, max_len=5000, name="mha_int4"), Hkv=4, H=4),
    wl.replace(wl.scaled(wl.CONFIGS["gqa70b"], B=12, max_len=4000, name="gqa_int8"), Hkv=2, H=16),
    wl.replace(wl.scaled(wl.CONFIGS["gqa70b"], B=12, max_len=4000, name="gqa_int4"), bits=4, G=32, Hkv=2, H=16),
]


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2410_23537_amd import binding
    return binding, torch


@pytest.mark.parametrize("w", LAYOUTS, ids=lambda w: w.name)
def test_repeated_calls_return_the_same_bytes(env, w):
    B, torch = env
    print(f"case determinism {w.name}", flush=True)
    pg = wl.paging(w)
    pool = wl.value_pool(w, n_min=int(pg.lens.max()) * w.Hkv * w.D)
    offs, gain = wl.request_offsets(w), wl.k_channel_gain(w)
    caches = [harness.fill_device_cache(B, torch, w, pg, pool, offs, gain) for _ in range(2)]
    for name in ("k_codes", "v_codes", "k_meta", "v_meta"):
        a, b = getattr(caches[0], name), getattr(caches[1], name)
        assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), f"{name} differs between two writes"
    dev = caches[0]
    q_np = wl.queries(w)
    runs = [harness.run_device_attn(B, torch, w, dev, q_np, pg) for _ in range(3)]
    for r in runs[1:]:
        assert np.array_equal(runs[0].view(np.uint16), r.view(np.uint16)), "decode attention differs between two calls"

    # prefill: every third request brings its last min(300, L) tokens
    lens = pg.lens.astype(np.int64)
    n = np.array([min(300, int(L)) if i % 3 == 0 else 0 for i, L in enumerate(lens)], np.int64)
    q_start = np.concatenate([[0], np.cumsum(n)]).astype(np.int32)
    total = int(q_start[-1])
    rng = np.random.default_rng([w.seed, 17])
    qp = torch.from_numpy(rng.standard_normal((total, w.H, w.D)).astype(np.float16)).cuda()
    ws = torch.empty(B.alise_paged_prefill_attn_workspace_bytes(dev, w.B, total, w.H, int(lens.max())), dtype=torch.uint8, device="cuda")
    bt, lens_d, qs = torch.from_numpy(pg.block_tables).cuda(), torch.from_numpy(pg.lens.astype(np.int32)).cuda(), torch.from_numpy(q_start).cuda()
    outs = []
    for _ in range(3):
        o = torch.full(qp.shape, float("nan"), dtype=torch.float16, device="cuda")
        B.alise_paged_prefill_attn(dev, qp, o, qs, bt, lens_d, int(lens.max()), 1.0 / np.sqrt(w.D), ws)
        outs.append(o)
    torch.cuda.synchronize()
    for o in outs[1:]:
        assert torch.equal(outs[0].view(torch.int16), o.view(torch.int16)), "prefill attention differs between two calls"

    # offload of the longest request
    i = int(np.argmax(lens))
    nbytes = B.alise_kv_swap_bytes(dev, int(lens[i]))
    bufs = [torch.zeros(nbytes, dtype=torch.uint8, device="cuda") for _ in range(2)]
    row = torch.from_numpy(pg.block_tables[i]).cuda()
    for b in bufs:
        B.alise_kv_swap_out(dev, row, int(lens[i]), b)
    torch.cuda.synchronize()
    assert torch.equal(bufs[0], bufs[1])
