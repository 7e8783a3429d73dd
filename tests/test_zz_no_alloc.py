"""alise_paged_decode_attn_static -- the attention call for callers that cannot allocate: its workspace is a
static device array inside the library.  Through the C ABI, two calls in a row on the same GPU (the second on a
smaller batch, so that whatever the first left in the array is there when it runs) must give bit for bit what
alise_paged_decode_attn gives with a caller's workspace, and the oracle's answer within 2e-3; torch's allocator
must not have been asked for anything in between."""
import numpy as np
import pytest

from paper_2410_23537_amd import workloads as wl
from tests import harness

pytestmark = pytest.mark.gpu

CASES = [
    # (first batch, second, smaller batch): vector path with split requests, matrix-core path
    (wl.replace(wl.scaled(wl.CONFIGS["int4"], B=24, max_len=5000, name="mha_int4"), Hkv=4, H=4),
     wl.replace(wl.scaled(wl.CONFIGS["int4"], B=5, max_len=700, name="mha_int4_small"), Hkv=4, H=4)),
    (wl.replace(wl.scaled(wl.CONFIGS["gqa70b"], B=12, max_len=4000, name="gqa_int8"), Hkv=2, H=16),
     wl.replace(wl.scaled(wl.CONFIGS["gqa70b"], B=3, max_len=900, name="gqa_int8_small"), Hkv=2, H=16)),
]


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2410_23537_amd import binding
    import oracle
    oracle.build()
    return binding, torch, oracle


def _problem(B, torch, oracle, w):
    lens = wl.context_lens(w).astype(np.int32)
    lens[1] = 0                               # an empty request: a zero row
    pg = wl.paging(w, lens)
    pool = wl.value_pool(w, n_min=int(lens.max()) * w.Hkv * w.D)
    offs, gain = wl.request_offsets(w), wl.k_channel_gain(w)
    dev = harness.fill_device_cache(B, torch, w, pg, pool, offs, gain)
    orc = harness.fill_oracle_cache(oracle, w, pg, pool, offs, gain)
    q_np = wl.queries(w)
    want = oracle.paged_decode_attn(orc, q_np, pg.block_tables, pg.lens, 1.0 / np.sqrt(w.D), num_threads=8)
    return dict(w=w, pg=pg, dev=dev, q=torch.from_numpy(q_np).cuda(), bt=torch.from_numpy(pg.block_tables).cuda(),
                lens=torch.from_numpy(lens).cuda(), max_len=int(max(1, lens.max())), want=want)


@pytest.mark.parametrize("first,second", CASES, ids=lambda w: w.name)
def test_static_workspace_matches_the_callers_workspace(env, first, second):
    B, torch, oracle = env
    print(f"case no_alloc {first.name} then {second.name}", flush=True)
    probs = [_problem(B, torch, oracle, w) for w in (first, second)]
    # the reference: the existing entry point, each problem with a workspace of its own
    refs = []
    for p in probs:
        w = p["w"]
        nbytes = B.alise_paged_decode_attn_workspace_bytes(p["dev"], w.B, w.H, p["max_len"])
        assert 0 < nbytes <= B.ALISE_STATIC_SCRATCH_BYTES
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        o = torch.full(p["q"].shape, float("nan"), dtype=torch.float16, device="cuda")
        B.alise_paged_decode_attn(p["dev"], p["q"], o, p["bt"], p["lens"], p["max_len"], 1.0 / np.sqrt(w.D), ws)
        refs.append(o)
    outs = [torch.full(p["q"].shape, float("nan"), dtype=torch.float16, device="cuda") for p in probs]
    torch.cuda.synchronize()
    before = torch.cuda.memory_stats()["allocation.all.allocated"]
    for p, o in zip(probs, outs):               # back to back on one stream, the smaller batch second
        B.alise_paged_decode_attn_static(p["dev"], p["q"], o, p["bt"], p["lens"], p["max_len"], 1.0 / np.sqrt(p["w"].D))
    torch.cuda.synchronize()
    assert torch.cuda.memory_stats()["allocation.all.allocated"] == before
    for p, o, ref in zip(probs, outs, refs):
        assert torch.equal(o.view(torch.int16), ref.view(torch.int16)), p["w"].name
        assert not o[1].any()
        err = np.abs(o.cpu().numpy().astype(np.float64) - p["want"]).max()
        assert err <= 2e-3, (p["w"].name, err)


def test_static_workspace_refuses_what_does_not_fit(env):
    """A batch whose workspace is larger than the static array: a clear status, nothing launched, output untouched."""
    B, torch, _ = env
    print("case no_alloc oversize", flush=True)
    w = wl.replace(wl.scaled(wl.CONFIGS["gqa70b"], B=4096, max_len=16384, name="big"))
    cache = B.KVCache.allocate(4, w.P, w.Hkv, w.D, w.bits, w.G, fill=0)
    assert B.alise_paged_decode_attn_workspace_bytes(cache, w.B, w.H, 16384) > B.ALISE_STATIC_SCRATCH_BYTES
    q = torch.zeros((w.B, w.H, w.D), dtype=torch.float16, device="cuda")
    out = torch.full(q.shape, 7.0, dtype=torch.float16, device="cuda")
    bt = torch.zeros((w.B, 16384 // w.P), dtype=torch.int32, device="cuda")
    lens = torch.zeros(w.B, dtype=torch.int32, device="cuda")
    with pytest.raises(B.AliseError) as e:
        B.alise_paged_decode_attn_static(cache, q, out, bt, lens, 16384, 1.0 / np.sqrt(w.D))
    assert e.value.status == B.ALISE_WORKSPACE_TOO_SMALL
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())
