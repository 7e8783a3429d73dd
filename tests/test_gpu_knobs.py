"""Every kernel variant that a tuning knob can select (environment variables, read again on request) must
compute the same attention (ALISE Sec. 2, Eq. 1-2 over the cache of Sec. 3.2): stage counts and
wave-loads per block, waves per compute unit, split lengths, the floor of items per wave, and
the one-row-tile and the single-weight prefill kernels.  Each setting is run on small batches of the four layouts
(MHA INT8, MHA INT4, GQA INT8, GQA INT4 with groups of 32 and of 128) and compared with the oracle."""
import os

import numpy as np
import pytest

from paper_2410_23537_amd import workloads as wl
from tests import harness

pytestmark = pytest.mark.gpu

ATTN_TOL = 2e-3
KNOBS = ("ALISE_SPLIT_TOKENS", "ALISE_SPLIT_TOKENS_GQA", "ALISE_WAVES_PER_CU", "ALISE_LOADS_PER_BLOCK",
         "ALISE_MIN_ITEMS_PER_WAVE", "ALISE_PREFILL_ROW_TILES", "ALISE_PREFILL_WEIGHTS", "ALISE_XCD_SKEW")

LAYOUTS = [
    wl.replace(wl.scaled(wl.CONFIGS["llama7b"], B=6, max_len=2600, name="mha_int8"), Hkv=4, H=4, length_law="uniform:1,2600"),
    wl.replace(wl.scaled(wl.CONFIGS["int4"], B=6, max_len=2600, name="mha_int4"), Hkv=4, H=4, length_law="uniform:1,2600"),
    wl.replace(wl.scaled(wl.CONFIGS["gqa70b"], B=5, max_len=2600, name="gqa_int8"), Hkv=2, H=16, length_law="uniform:1,2600"),
    wl.replace(wl.scaled(wl.CONFIGS["gqa70b"], B=5, max_len=2600, name="gqa_int4"), bits=4, G=32, Hkv=2, H=16,
               length_law="uniform:1,2600"),
    wl.replace(wl.scaled(wl.CONFIGS["gqa70b"], B=5, max_len=2600, name="gqa_int4_g128"), bits=4, G=128, Hkv=2, H=8,
               length_law="uniform:1,2600"),
]

SETTINGS = [
    {"ALISE_LOADS_PER_BLOCK": "3"}, {"ALISE_LOADS_PER_BLOCK": "4"}, {"ALISE_LOADS_PER_BLOCK": "2"},
    {"ALISE_WAVES_PER_CU": "4"}, {"ALISE_WAVES_PER_CU": "8"},
    {"ALISE_SPLIT_TOKENS": "256", "ALISE_SPLIT_TOKENS_GQA": "256"}, {"ALISE_SPLIT_TOKENS": "512", "ALISE_SPLIT_TOKENS_GQA": "512"},
    {"ALISE_SPLIT_TOKENS": "1024", "ALISE_SPLIT_TOKENS_GQA": "1024"},
    {"ALISE_MIN_ITEMS_PER_WAVE": "1"}, {"ALISE_MIN_ITEMS_PER_WAVE": "16"},
    {"ALISE_LOADS_PER_BLOCK": "4", "ALISE_WAVES_PER_CU": "4", "ALISE_SPLIT_TOKENS": "512", "ALISE_SPLIT_TOKENS_GQA": "512"},
]


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2410_23537_amd import binding
    import oracle
    oracle.build()
    return binding, torch, oracle


@pytest.fixture(scope="module")
def problems(env):
    B, torch, oracle = env
    out = {}
    for w in LAYOUTS:
        pg = wl.paging(w)
        pool = wl.value_pool(w, n_min=int(pg.lens.max()) * w.Hkv * w.D)
        offs, gain = wl.request_offsets(w), wl.k_channel_gain(w)
        orc = harness.fill_oracle_cache(oracle, w, pg, pool, offs, gain)
        dev = harness.fill_device_cache(B, torch, w, pg, pool, offs, gain)
        q = wl.queries(w)
        want = oracle.paged_decode_attn(orc, q, pg.block_tables, pg.lens, 1.0 / np.sqrt(w.D))
        out[w.name] = (w, pg, orc, dev, q, want)
    return out


@pytest.fixture(autouse=True)
def clean_environment(env):
    saved = {k: os.environ.pop(k, None) for k in KNOBS}
    env[0].alise_reload_environment()
    yield
    for k in KNOBS:
        os.environ.pop(k, None)
        if saved[k] is not None:
            os.environ[k] = saved[k]
    env[0].alise_reload_environment()


def _set(B, setting):
    """The library reads its environment once per process: change it, then have it read again."""
    os.environ.update(setting)
    B.alise_reload_environment()


@pytest.mark.parametrize("setting", SETTINGS, ids=lambda s: ",".join(f"{k[6:].lower()}={v}" for k, v in s.items()))
def test_decode_under_every_knob(env, problems, setting):
    B, torch, oracle = env
    _set(B, setting)
    for name, (w, pg, orc, dev, q, want) in problems.items():
        print(f"case knobs {setting} {name}", flush=True)
        got = harness.run_device_attn(B, torch, w, dev, q, pg).astype(np.float64)
        err = float(np.abs(got - want).max())
        assert np.isfinite(got).all() and err <= ATTN_TOL, f"{name} under {setting}: {err:.3e}"


@pytest.mark.parametrize("weights", ["split", "single"])
@pytest.mark.parametrize("tiles", ["1", "2"])
def test_prefill_with_one_and_two_row_tiles(env, problems, tiles, weights):
    B, torch, oracle = env
    _set(B, {"ALISE_PREFILL_ROW_TILES": tiles, "ALISE_PREFILL_WEIGHTS": weights})
    for name, (w, pg, orc, dev, q, _) in problems.items():
        print(f"case knobs prefill row tiles {tiles} {name}", flush=True)
        lens = pg.lens.astype(np.int64)
        n = np.minimum(lens, [150, 1, 97, 33, 64, 200][:w.B])
        q_start = np.concatenate([[0], np.cumsum(n)]).astype(np.int32)
        total = int(q_start[-1])
        rng = np.random.default_rng([w.seed, 3])
        q_np = rng.standard_normal((total, w.H, w.D)).astype(np.float16)
        scale = 1.0 / np.sqrt(w.D)
        want = oracle.paged_prefill_attn(orc, q_np, q_start, pg.block_tables, pg.lens, scale)
        qd = torch.from_numpy(q_np).cuda()
        out = torch.full(qd.shape, float("nan"), dtype=torch.float16, device="cuda")
        ws = torch.empty(B.alise_paged_prefill_attn_workspace_bytes(dev, w.B, total, w.H, int(lens.max())), dtype=torch.uint8, device="cuda")
        B.alise_paged_prefill_attn(dev, qd, out, torch.from_numpy(q_start).cuda(), torch.from_numpy(pg.block_tables).cuda(),
                                   torch.from_numpy(pg.lens.astype(np.int32)).cuda(), int(lens.max()), scale, ws)
        torch.cuda.synchronize()
        got = out.cpu().numpy().astype(np.float64)
        err = float(np.abs(got - want).max())
        assert np.isfinite(got).all() and err <= ATTN_TOL, f"{name} with {tiles} row tiles, {weights} weights: {err:.3e}"


@pytest.mark.parametrize("bits,G,Hkv,H", [(8, 64, 2, 2), (8, 128, 1, 8), (4, 32, 1, 4)])
def test_more_than_64_splits_of_one_request(env, bits, G, Hkv, H):
    """A request of 20 000 tokens in splits of 256: 79 partial results, more than the 64 that the merge
    kernel combines in one pass of a wave, beside short requests that need no merge at all."""
    B, torch, oracle = env
    _set(B, {"ALISE_SPLIT_TOKENS": "256", "ALISE_SPLIT_TOKENS_GQA": "256"})
    if True:
        lens = np.array([20000, 3, 700, 0, 257], np.int32)
        w = wl.Workload("many_splits", B=len(lens), H=H, Hkv=Hkv, D=128, P=16, bits=bits, G=G, length_law="fixed:1", seed=9,
                        max_len=int(lens.max()))
        print(f"case knobs many splits bits={bits} H={H}", flush=True)
        pg = wl.paging(w, lens)
        pool = wl.value_pool(w, n_min=int(lens.max()) * Hkv * 128)
        offs, gain = wl.request_offsets(w), wl.k_channel_gain(w)
        orc = harness.fill_oracle_cache(oracle, w, pg, pool, offs, gain)
        dev = harness.fill_device_cache(B, torch, w, pg, pool, offs, gain)
        q = wl.queries(w)
        want = oracle.paged_decode_attn(orc, q, pg.block_tables, pg.lens, 1.0 / np.sqrt(w.D), num_threads=8)
        got = harness.run_device_attn(B, torch, w, dev, q, pg).astype(np.float64)
        err = float(np.abs(got - want).max())
        assert np.isfinite(got).all() and err <= ATTN_TOL, f"{err:.3e}"


@pytest.mark.parametrize("skew", ["0", "50", "200"])
def test_short_items_dealt_to_half_of_the_waves(env, skew):
    """ALISE_XCD_SKEW: the shortest items of a large batch go to the waves of even workgroups only.  The plan
    applies it when a wave gets many items, so: 420 requests, 8 heads, splits of 256 tokens and an item floor of
    one (6 700 items and more against a threshold of 6 144).  Every (request, head) must still be attended to
    exactly once: compared with the oracle."""
    B, torch, oracle = env
    _set(B, {"ALISE_XCD_SKEW": skew, "ALISE_MIN_ITEMS_PER_WAVE": "1", "ALISE_SPLIT_TOKENS": "256"})
    if True:
        rng = np.random.default_rng(31)
        lens = rng.integers(0, 600, 420).astype(np.int32)
        lens[:5] = [0, 1, 256, 257, 3000]
        w = wl.Workload("skew", B=len(lens), H=8, Hkv=8, D=128, P=16, bits=8, G=128, length_law="fixed:1", seed=19, max_len=int(lens.max()))
        print(f"case knobs skew {skew}", flush=True)
        pg = wl.paging(w, lens)
        pool = wl.value_pool(w, n_min=int(lens.max()) * w.Hkv * w.D)
        offs, gain = wl.request_offsets(w), wl.k_channel_gain(w)
        orc = harness.fill_oracle_cache(oracle, w, pg, pool, offs, gain)
        dev = harness.fill_device_cache(B, torch, w, pg, pool, offs, gain)
        q = wl.queries(w)
        want = oracle.paged_decode_attn(orc, q, pg.block_tables, pg.lens, 1.0 / np.sqrt(w.D), num_threads=8)
        got = harness.run_device_attn(B, torch, w, dev, q, pg).astype(np.float64)
        err = float(np.abs(got - want).max())
        assert np.isfinite(got).all() and not got[lens == 0].any() and err <= ATTN_TOL, f"{err:.3e}"


@pytest.mark.parametrize("Hkv,H,split", [(2, 2, "320"), (2, 2, "32704"), (1, 8, "320"), (1, 8, "16320")])
def test_fixed_split_that_is_no_multiple_of_the_page(env, Hkv, H, split):
    """Pages of 256 tokens and a fixed split that is a multiple of 64 but not of the page: the splits of a request
    start at multiples of the split, so such a split would begin inside a page and reach one page more than the
    kernels' page window holds.  The library rounds it down to whole pages; requests of several splits must come
    out right on the vector path and on the matrix-core path."""
    B, torch, oracle = env
    _set(B, {"ALISE_SPLIT_TOKENS": split, "ALISE_SPLIT_TOKENS_GQA": split})
    lens = np.array([70000 if int(split) > 4096 else 1000, 3, 700, 257, 256], np.int32)
    w = wl.Workload("page256", B=len(lens), H=H, Hkv=Hkv, D=128, P=256, bits=8, G=128, length_law="fixed:1", seed=23,
                    max_len=int(lens.max()))
    print(f"case knobs page 256 split {split} H={H}", flush=True)
    pg = wl.paging(w, lens)
    pool = wl.value_pool(w, n_min=int(lens.max()) * Hkv * 128)
    offs, gain = wl.request_offsets(w), wl.k_channel_gain(w)
    orc = harness.fill_oracle_cache(oracle, w, pg, pool, offs, gain)
    dev = harness.fill_device_cache(B, torch, w, pg, pool, offs, gain)
    q = wl.queries(w)
    want = oracle.paged_decode_attn(orc, q, pg.block_tables, pg.lens, 1.0 / np.sqrt(w.D), num_threads=8)
    got = harness.run_device_attn(B, torch, w, dev, q, pg).astype(np.float64)
    err = float(np.abs(got - want).max())
    assert np.isfinite(got).all() and err <= ATTN_TOL, f"{err:.3e}"
