"""One plan for all layers of a decode iteration: alise_paged_decode_attn_plan once, then
alise_paged_decode_attn_planned per layer (each layer its own cache and queries, one workspace) must give
bit for bit what the single call gives per layer -- on the vector and the matrix-core path, with empty
requests (zero rows written by the run, not by the plan), unsplit and split requests."""
import numpy as np
import pytest

from paper_2410_23537_amd import workloads as wl
from tests import harness

pytestmark = pytest.mark.gpu

LAYOUTS = [
    wl.replace(wl.scaled(wl.CONFIGS["llama7b"], B=9, max_len=2600, name="mha_int8"), Hkv=4, H=4),
    wl.replace(wl.scaled(wl.CONFIGS["int4"], B=9, max_len=2600, name="mha_int4"), Hkv=4, H=4),
    wl.replace(wl.scaled(wl.CONFIGS["gqa70b"], B=7, max_len=2600, name="gqa_int8"), Hkv=2, H=16),
]


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2410_23537_amd import binding
    import oracle
    oracle.build()
    return binding, torch, oracle


@pytest.mark.parametrize("w", LAYOUTS, ids=lambda w: w.name)
def test_one_plan_serves_every_layer(env, w):
    B, torch, oracle = env
    print(f"case planned {w.name}", flush=True)
    lens = wl.context_lens(w).astype(np.int32)
    lens[1] = 0                                   # an empty request
    lens[2] = 1
    pg = wl.paging(w, lens)
    n_layers = 3
    scale = 1.0 / np.sqrt(w.D)
    layers = []
    for layer in range(n_layers):
        wl_layer = wl.replace(w, seed=w.seed + 100 * layer)
        pool = wl.value_pool(wl_layer, n_min=int(lens.max()) * w.Hkv * w.D)
        offs, gain = wl.request_offsets(wl_layer), wl.k_channel_gain(wl_layer)
        dev = harness.fill_device_cache(B, torch, wl_layer, pg, pool, offs, gain)
        q = torch.from_numpy(wl.queries(wl_layer)).cuda()
        layers.append((wl_layer, pool, offs, gain, dev, q))
    bt = torch.from_numpy(pg.block_tables).cuda()
    lens_d = torch.from_numpy(lens).cuda()
    max_len = int(lens.max())
    ws = torch.empty(B.alise_paged_decode_attn_workspace_bytes(layers[0][4], w.B, w.H, max_len), dtype=torch.uint8, device="cuda")

    single = []
    for _, _, _, _, dev, q in layers:
        o = torch.full(q.shape, float("nan"), dtype=torch.float16, device="cuda")
        B.alise_paged_decode_attn(dev, q, o, bt, lens_d, max_len, scale, ws)
        single.append(o)
    torch.cuda.synchronize()

    ws.fill_(0xA5)                                # nothing of the single calls may be needed
    B.alise_paged_decode_attn_plan(layers[0][4], lens_d, w.H, max_len, ws)
    for (_, _, _, _, dev, q), ref in zip(layers, single):
        o = torch.full(q.shape, float("nan"), dtype=torch.float16, device="cuda")
        B.alise_paged_decode_attn_planned(dev, q, o, bt, lens_d, max_len, scale, ws)
        torch.cuda.synchronize()
        assert torch.equal(o.view(torch.int16), ref.view(torch.int16))
        assert not o[1].any() and not o[lens_d == 0].any()

    # and the single call is the oracle's answer (first layer)
    wl0, pool, offs, gain, dev, q = layers[0]
    orc = harness.fill_oracle_cache(oracle, wl0, pg, pool, offs, gain)
    want = oracle.paged_decode_attn(orc, q.cpu().numpy(), pg.block_tables, pg.lens, scale, num_threads=8)
    assert np.abs(single[0].cpu().numpy().astype(np.float64) - want).max() <= 2e-3
