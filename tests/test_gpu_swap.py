"""GPU parity of the offload / upload calls (ALISE Sec. 3.2 "Dynamic Swapping", Alg. 2: the
data movement) against the CPU oracle, through the C ABI.  Everything is bytes, so
everything is compared bit for bit: the offloaded form of every request, the pages after
an upload into another cache under another paging (and another memory layout), the pages
nobody named.  Attention after the round trip is checked against the oracle as well."""
import numpy as np
import pytest

from paper_2410_23537_amd import workloads as wl
from tests import harness

pytestmark = pytest.mark.gpu

ATTN_TOL = 2e-3

CASES = [
    wl.CONFIGS["tiny"],
    wl.scaled(wl.CONFIGS["opt13b"], B=6, max_len=700),
    wl.scaled(wl.CONFIGS["llama7b"], B=6, max_len=1300),
    wl.replace(wl.scaled(wl.CONFIGS["gqa70b"], B=4, max_len=900), length_law="uniform:100,900"),
    wl.scaled(wl.CONFIGS["int4"], B=12, max_len=1700),
    wl.replace(wl.scaled(wl.CONFIGS["int4"], B=4, max_len=600, name="int4_d64"), D=64, G=32, P=32),
    wl.replace(wl.scaled(wl.CONFIGS["opt13b"], B=4, max_len=300, name="int8_g16_p8"), G=16, P=8, Hkv=3, H=3),
    wl.replace(wl.scaled(wl.CONFIGS["llama7b"], B=3, max_len=64, name="lengths_1_16_17"), length_law="fixed:1,16,17"),
]


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2410_23537_amd import binding
    import oracle
    oracle.build()
    return binding, torch, oracle


def _problem(w):
    pg = wl.paging(w)
    pool = wl.value_pool(w, n_min=int(max(1, pg.lens.max(initial=1))) * w.Hkv * w.D)
    return pg, pool, wl.request_offsets(w), wl.k_channel_gain(w)


def _arrays_equal(dev, orc, pages=None):
    for name in ("k_codes", "v_codes", "k_meta", "v_meta"):
        d = getattr(dev, name).cpu().numpy()
        o = getattr(orc, name)
        if name.endswith("meta"):
            d, o = d.view(np.uint16), o.view(np.uint16)
        if pages is not None:
            d, o = d[pages], o[pages]
        assert np.array_equal(d, o), f"{name} differ"


@pytest.mark.parametrize("layouts", [("interleaved", "dense"), ("dense", "interleaved")], ids=lambda l: f"{l[0]}->{l[1]}")
@pytest.mark.parametrize("w", CASES, ids=lambda w: w.name)
def test_offload_then_upload_elsewhere(env, w, layouts):
    B, torch, oracle = env
    print(f"case swap {w.name} {layouts}: B={w.B} Hkv={w.Hkv} D={w.D} P={w.P} bits={w.bits} G={w.G}", flush=True)
    pg, pool, offs, gain = _problem(w)
    orc = harness.fill_oracle_cache(oracle, w, pg, pool, offs, gain)
    dev = harness.fill_device_cache(B, torch, w, pg, pool, offs, gain, layout=layouts[0])
    _arrays_equal(dev, orc)          # both writers agree on every byte, named or not (same poison)

    # ---- offload: every request into its own device buffer, 64 guard bytes behind it
    bt_dev = torch.from_numpy(pg.block_tables).cuda()
    packed_dev = []
    for i, L in enumerate(pg.lens):
        L = int(L)
        n = B.alise_kv_swap_bytes(dev, L)
        assert n == oracle.kv_swap_bytes(orc, L)
        buf = torch.full((n + 64,), 0xA5, dtype=torch.uint8, device="cuda")
        B.alise_kv_swap_out(dev, bt_dev[i], L, buf[:n])
        packed_dev.append(buf)
    torch.cuda.synchronize()
    for i, L in enumerate(pg.lens):
        want = oracle.kv_swap_out(orc, pg.block_tables[i], int(L))
        got = packed_dev[i].cpu().numpy()
        assert np.array_equal(got[:want.size], want), f"offloaded form of request {i} differs"
        assert (got[want.size:] == 0xA5).all(), "wrote past the end of the buffer"

    # ---- upload into another cache: other pages, the other memory layout, sentinel everywhere else
    pg2 = wl.paging(wl.replace(w, seed=w.seed + 99), lens=pg.lens)
    orc2 = oracle.Cache.empty(pg2.num_pages, w.P, w.Hkv, w.D, w.bits, w.G, fill=0x3C)
    orc2.k_meta.view(np.uint16)[:] = 0x1234
    orc2.v_meta.view(np.uint16)[:] = 0x4321
    dev2 = B.KVCache.allocate(pg2.num_pages, w.P, w.Hkv, w.D, w.bits, w.G, fill=0x3C, layout=layouts[1])
    dev2.k_meta.view(torch.int16).fill_(0x1234)
    dev2.v_meta.view(torch.int16).fill_(0x4321)
    bt2_dev = torch.from_numpy(pg2.block_tables).cuda()
    for i, L in enumerate(pg.lens):
        L = int(L)
        n = B.alise_kv_swap_bytes(dev2, L)
        B.alise_kv_swap_in(dev2, bt2_dev[i], L, packed_dev[i][:n])
        oracle.kv_swap_in(orc2, pg2.block_tables[i], L, oracle.kv_swap_out(orc, pg.block_tables[i], L))
    torch.cuda.synchronize()
    _arrays_equal(dev2, orc2)        # named pages hold the request, every other byte is the sentinel

    # ---- and the uploaded cache attends like the oracle's
    q = wl.queries(w)
    want = oracle.paged_decode_attn(orc2, q, pg2.block_tables, pg.lens, 1.0 / np.sqrt(w.D))
    got = harness.run_device_attn(B, torch, w, dev2, q, pg2).astype(np.float64)
    assert np.abs(got - want).max() <= ATTN_TOL


def test_pinned_host_buffer_on_a_side_stream_while_attention_runs(env):
    """The buffer in pinned host memory, the copy on its own stream, attention on the main one."""
    B, torch, oracle = env
    w = wl.scaled(wl.CONFIGS["llama7b"], B=8, max_len=1500)
    pg, pool, offs, gain = _problem(w)
    orc = harness.fill_oracle_cache(oracle, w, pg, pool, offs, gain)
    dev = harness.fill_device_cache(B, torch, w, pg, pool, offs, gain)
    i = int(np.argmax(pg.lens))
    L = int(pg.lens[i])
    n = B.alise_kv_swap_bytes(dev, L)
    host = torch.empty(n, dtype=torch.uint8, pin_memory=True)
    host.fill_(0x77)
    bt_dev = torch.from_numpy(pg.block_tables).cuda()
    q_np = wl.queries(w)
    q = torch.from_numpy(q_np).cuda()
    out = torch.full(q.shape, float("nan"), dtype=torch.float16, device="cuda")
    lens = torch.from_numpy(pg.lens.astype(np.int32)).cuda()
    max_len = int(pg.lens.max())
    ws = torch.empty(B.alise_paged_decode_attn_workspace_bytes(dev, w.B, w.H, max_len), dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        B.alise_kv_swap_out(dev, bt_dev[i], L, host)             # reads the cache only: may overlap with attention
    B.alise_paged_decode_attn(dev, q, out, bt_dev, lens, max_len, 1.0 / np.sqrt(w.D), ws)
    torch.cuda.synchronize()
    assert np.array_equal(host.numpy(), oracle.kv_swap_out(orc, pg.block_tables[i], L))
    want = oracle.paged_decode_attn(orc, q_np, pg.block_tables, pg.lens, 1.0 / np.sqrt(w.D))
    assert np.abs(out.cpu().numpy().astype(np.float64) - want).max() <= ATTN_TOL

    # upload from the pinned buffer into fresh pages of the same cache: the spare pages of a bigger cache
    nblk = (L + w.P - 1) // w.P
    big = B.KVCache.allocate(nblk + 3, w.P, w.Hkv, w.D, w.bits, w.G, fill=0)
    bt_new = torch.arange(nblk - 1, -1, -1, dtype=torch.int32, device="cuda") + 2
    with torch.cuda.stream(side):
        B.alise_kv_swap_in(big, bt_new, L, host)
    side.synchronize()
    ref = oracle.Cache.empty(nblk + 3, w.P, w.Hkv, w.D, w.bits, w.G, fill=0)
    oracle.kv_swap_in(ref, bt_new.cpu().numpy(), L, host.numpy())
    _arrays_equal(big, ref)


def test_zero_tokens_is_a_no_op(env):
    B, torch, oracle = env
    c = B.KVCache.allocate(4, 16, 2, 64, 8, 64, fill=9)
    assert B.alise_kv_swap_bytes(c, 0) == 0
    buf = torch.full((64,), 1, dtype=torch.uint8, device="cuda")
    bt = torch.zeros(1, dtype=torch.int32, device="cuda")
    B.alise_kv_swap_out(c, bt, 0, buf)
    B.alise_kv_swap_in(c, bt, 0, buf)
    torch.cuda.synchronize()
    assert (buf == 1).all() and (c.k_codes == 9).all()
