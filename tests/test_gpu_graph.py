"""The decode step under HIP graph capture (ALISE Sec. 2 "LLM Inference": every iteration appends
the new token's K/V and attends over the cache; a serving loop replays that iteration thousands
of times).  The library calls allocate nothing, synchronise nothing and read lengths, block
tables and slots from device memory, so one captured graph serves iterations with different
lengths.  The graph is replayed several times with the program's own eager work and
synchronisations in between; every replay must equal the same step done eagerly on a second,
identical cache bit for bit, and the oracle within the usual tolerance."""
import numpy as np
import pytest

from paper_2410_23537_amd import workloads as wl
from tests import harness

pytestmark = pytest.mark.gpu

ATTN_TOL = 2e-3


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2410_23537_amd import binding
    import oracle
    oracle.build()
    return binding, torch, oracle


CASES = [
    wl.scaled(wl.CONFIGS["llama7b"], B=12, max_len=900),
    wl.replace(wl.scaled(wl.CONFIGS["gqa70b"], B=6, max_len=1500), length_law="uniform:200,1500"),
    wl.scaled(wl.CONFIGS["int4"], B=16, max_len=1200),
]


@pytest.mark.parametrize("w", CASES, ids=lambda w: w.name)
def test_captured_decode_step_replays_like_eager(env, w):
    B, torch, oracle = env
    print(f"case graph {w.name}: B={w.B} H={w.H} Hkv={w.Hkv} bits={w.bits}", flush=True)
    pg = wl.paging(w)
    pool = wl.value_pool(w, n_min=int(pg.lens.max()) * w.Hkv * w.D)
    offs, gain = wl.request_offsets(w), wl.k_channel_gain(w)
    orc = harness.fill_oracle_cache(oracle, w, pg, pool, offs, gain)
    dev_g = harness.fill_device_cache(B, torch, w, pg, pool, offs, gain)        # the graph works on this one
    dev_e = harness.fill_device_cache(B, torch, w, pg, pool, offs, gain)        # the eager twin
    scale = 1.0 / np.sqrt(w.D)
    max_len = int(pg.lens.max())
    bt = torch.from_numpy(pg.block_tables).cuda()
    page0 = int(pg.block_tables[0, 0])

    # static buffers of the graph
    q = torch.zeros((w.B, w.H, w.D), dtype=torch.float16, device="cuda")
    k_new = torch.zeros((w.B, w.Hkv, w.D), dtype=torch.float16, device="cuda")
    v_new = torch.zeros_like(k_new)
    slots = torch.zeros(w.B, dtype=torch.int64, device="cuda")
    lens = torch.ones(w.B, dtype=torch.int32, device="cuda")
    out = torch.zeros_like(q)
    k_pg = torch.zeros((w.P, w.Hkv, w.D), dtype=torch.float16, device="cuda")
    v_pg = torch.zeros_like(k_pg)
    ws = torch.empty(B.alise_paged_decode_attn_workspace_bytes(dev_g, w.B, w.H, max_len), dtype=torch.uint8, device="cuda")

    def step(cache, q, k_new, v_new, slots, lens, out, k_pg, v_pg, ws):
        B.alise_kv_quant_write(cache, k_new, v_new, slots)
        B.alise_paged_decode_attn(cache, q, out, bt, lens, max_len, scale, ws)
        B.alise_kv_dequant_page(cache, page0, k_pg, v_pg)

    def inputs(r):
        """Replay r: every request is cut back to a random length, its next token is written and attended to."""
        rng = np.random.default_rng([w.seed, r, 17])
        L = np.array([rng.integers(0, int(x)) for x in pg.lens], np.int64)      # tokens kept; the new one lands at position L
        s = pg.block_tables[np.arange(w.B), L // w.P].astype(np.int64) * w.P + L % w.P
        return (rng.standard_normal((w.B, w.H, w.D)).astype(np.float16), rng.standard_normal((w.B, w.Hkv, w.D)).astype(np.float16),
                rng.standard_normal((w.B, w.Hkv, w.D)).astype(np.float16), s, (L + 1).astype(np.int32))

    def load(r):
        qn, kn, vn, sn, ln = inputs(r)
        q.copy_(torch.from_numpy(qn)); k_new.copy_(torch.from_numpy(kn)); v_new.copy_(torch.from_numpy(vn))
        slots.copy_(torch.from_numpy(sn)); lens.copy_(torch.from_numpy(ln))
        return qn, kn, vn, sn, ln

    # warm-up on a side stream (occupancy queries and the like happen here, not under capture), then capture
    load(0)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(dev_g, q, k_new, v_new, slots, lens, out, k_pg, v_pg, ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(dev_g, q, k_new, v_new, slots, lens, out, k_pg, v_pg, ws)
    # the warm-up wrote replay 0's tokens into dev_g: give the eager twin the same history
    e_out, e_k, e_v = torch.zeros_like(out), torch.zeros_like(k_pg), torch.zeros_like(v_pg)
    e_ws = torch.empty_like(ws)
    step(dev_e, q, k_new, v_new, slots, lens, e_out, e_k, e_v, e_ws)
    qn, kn, vn, sn, ln = inputs(0)
    oracle.kv_quant_write(orc, kn, vn, sn)

    for r in range(1, 5):
        qn, kn, vn, sn, ln = load(r)
        out.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        # the same step eagerly, on the twin cache, with buffers of its own
        step(dev_e, q, k_new, v_new, slots, lens, e_out, e_k, e_v, e_ws)
        torch.cuda.synchronize()
        assert np.array_equal(got.view(np.uint16), e_out.cpu().numpy().view(np.uint16)), f"replay {r}: attention differs from eager"
        assert torch.equal(k_pg, e_k) and torch.equal(v_pg, e_v), f"replay {r}: dequantized page differs from eager"
        for name in ("k_codes", "v_codes", "k_meta", "v_meta"):
            a, b = getattr(dev_g, name), getattr(dev_e, name)
            assert torch.equal(a.view(torch.uint8) if a.dtype == torch.uint8 else a.view(torch.int16),
                               b.view(torch.uint8) if b.dtype == torch.uint8 else b.view(torch.int16)), f"replay {r}: {name} differs"
        # and against the oracle
        oracle.kv_quant_write(orc, kn, vn, sn)
        want = oracle.paged_decode_attn(orc, qn, pg.block_tables, ln, scale)
        err = float(np.abs(got.astype(np.float64) - want).max())
        print(f"  replay {r}: max-abs error against the oracle {err:.2e}", flush=True)
        assert np.isfinite(got).all() and err <= ATTN_TOL
        # eager work of the program's own between replays
        (q.float() * 2.0).sum().item()


@pytest.mark.parametrize("w", CASES[:2], ids=lambda w: w.name)
def test_captured_iteration_of_three_layers_with_one_plan(env, w):
    """What a serving loop captures: the plan once, then per layer the write of the new token and the planned
    attention call, each layer with a cache of its own.  Replayed with other lengths and tokens, every layer's
    output must equal the single (plan + run) call done eagerly on a twin cache, bit for bit."""
    B, torch, oracle = env
    print(f"case graph planned {w.name}", flush=True)
    n_layers = 3
    pg = wl.paging(w)
    scale = 1.0 / np.sqrt(w.D)
    max_len = int(pg.lens.max())
    bt = torch.from_numpy(pg.block_tables).cuda()
    caches_g, caches_e = [], []
    for layer in range(n_layers):
        wl_layer = wl.replace(w, seed=w.seed + 100 * layer)
        pool = wl.value_pool(wl_layer, n_min=max_len * w.Hkv * w.D)
        offs, gain = wl.request_offsets(wl_layer), wl.k_channel_gain(wl_layer)
        caches_g.append(harness.fill_device_cache(B, torch, wl_layer, pg, pool, offs, gain))
        caches_e.append(harness.fill_device_cache(B, torch, wl_layer, pg, pool, offs, gain))
    q = torch.zeros((n_layers, w.B, w.H, w.D), dtype=torch.float16, device="cuda")
    k_new = torch.zeros((n_layers, w.B, w.Hkv, w.D), dtype=torch.float16, device="cuda")
    v_new = torch.zeros_like(k_new)
    slots = torch.zeros(w.B, dtype=torch.int64, device="cuda")
    lens = torch.ones(w.B, dtype=torch.int32, device="cuda")
    out = torch.zeros_like(q)
    ws = torch.empty(B.alise_paged_decode_attn_workspace_bytes(caches_g[0], w.B, w.H, max_len), dtype=torch.uint8, device="cuda")

    def iteration():
        B.alise_paged_decode_attn_plan(caches_g[0], lens, w.H, max_len, ws)
        for layer in range(n_layers):
            B.alise_kv_quant_write(caches_g[layer], k_new[layer], v_new[layer], slots)
            B.alise_paged_decode_attn_planned(caches_g[layer], q[layer], out[layer], bt, lens, max_len, scale, ws)

    def load(r):
        rng = np.random.default_rng([w.seed, r, 23])
        L = np.array([rng.integers(0, int(x)) for x in pg.lens], np.int64)
        if r == 2:
            L[0] = 0                                    # a one-token request
        s = pg.block_tables[np.arange(w.B), L // w.P].astype(np.int64) * w.P + L % w.P
        q.copy_(torch.from_numpy(rng.standard_normal(tuple(q.shape)).astype(np.float16)))
        k_new.copy_(torch.from_numpy(rng.standard_normal(tuple(k_new.shape)).astype(np.float16)))
        v_new.copy_(torch.from_numpy(rng.standard_normal(tuple(v_new.shape)).astype(np.float16)))
        slots.copy_(torch.from_numpy(s))
        lens.copy_(torch.from_numpy((L + 1).astype(np.int32)))

    def eager():
        e_out = torch.zeros_like(out)
        e_ws = torch.empty_like(ws)
        for layer in range(n_layers):
            B.alise_kv_quant_write(caches_e[layer], k_new[layer], v_new[layer], slots)
            B.alise_paged_decode_attn(caches_e[layer], q[layer], e_out[layer], bt, lens, max_len, scale, e_ws)
        torch.cuda.synchronize()
        return e_out

    load(0)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        iteration()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        iteration()
    eager()                                             # the twin caches get replay 0's tokens too
    for r in range(1, 5):
        load(r)
        out.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        want = eager()
        assert torch.equal(out.view(torch.int16), want.view(torch.int16)), f"replay {r} differs from the eager single calls"
        _ = (q.float() @ q.float().transpose(-1, -2)).sum().item()          # eager work of the program's own between replays


@pytest.mark.parametrize("w", [CASES[0], CASES[2]], ids=lambda w: w.name)
def test_captured_prefill_call_replays_like_eager(env, w):
    """The chunked-prefill call under graph capture: chunk boundaries and lengths are read from device memory, so
    one captured call serves other chunk mixes of at most as many query tokens; every replay equals the eager call."""
    B, torch, oracle = env
    print(f"case graph prefill {w.name}", flush=True)
    pg = wl.paging(w)
    pool = wl.value_pool(w, n_min=int(pg.lens.max()) * w.Hkv * w.D)
    offs, gain = wl.request_offsets(w), wl.k_channel_gain(w)
    dev = harness.fill_device_cache(B, torch, w, pg, pool, offs, gain)
    scale = 1.0 / np.sqrt(w.D)
    max_len = int(pg.lens.max())
    bt = torch.from_numpy(pg.block_tables).cuda()
    total_cap = 64 * w.B
    q = torch.zeros((total_cap, w.H, w.D), dtype=torch.float16, device="cuda")
    out = torch.zeros_like(q)
    q_start = torch.zeros(w.B + 1, dtype=torch.int32, device="cuda")
    lens = torch.ones(w.B, dtype=torch.int32, device="cuda")
    ws = torch.empty(B.alise_paged_prefill_attn_workspace_bytes(dev, w.B, total_cap, w.H, max_len), dtype=torch.uint8, device="cuda")
    e_ws = torch.empty_like(ws)

    def call(o, wsp):
        B.alise_paged_prefill_attn(dev, q, o, q_start, bt, lens, max_len, scale, wsp)

    def load(r):
        rng = np.random.default_rng([w.seed, r, 29])
        L = np.array([rng.integers(1, int(x) + 1) for x in pg.lens], np.int64)
        n = np.minimum(L, rng.integers(0, 65, w.B))
        qs = np.concatenate([[0], np.cumsum(n)]).astype(np.int32)
        q.copy_(torch.from_numpy(rng.standard_normal(tuple(q.shape)).astype(np.float16)))
        q_start.copy_(torch.from_numpy(qs))
        lens.copy_(torch.from_numpy(L.astype(np.int32)))
        return int(qs[-1])

    load(0)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        call(out, ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call(out, ws)
    for r in range(1, 5):
        total = load(r)
        out.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        e_out = torch.full_like(out, float("nan"))
        call(e_out, e_ws)
        torch.cuda.synchronize()
        assert torch.equal(out[:total].view(torch.int16), e_out[:total].view(torch.int16)), f"replay {r} differs from the eager call"
        assert torch.isfinite(out[:total].float()).all()
