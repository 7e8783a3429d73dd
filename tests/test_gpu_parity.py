"""GPU parity: the HIP path through the C ABI against the CPU oracle on the same
seeded inputs.  Codes and meta bit for bit; attention within 2e-3 max-abs of the
fp64 oracle (fp16 output); page dequantizer bit for bit."""
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


def _problem(w, lens=None):
    pg = wl.paging(w, lens)
    pool = wl.value_pool(w, n_min=int(max(1, pg.lens.max(initial=1))) * w.Hkv * w.D)
    offs = wl.request_offsets(w)
    gain = wl.k_channel_gain(w)
    return pg, pool, offs, gain


def _compare_caches(w, pg, dev, orc):
    mask = harness.written_mask(w, pg)
    for name in ("k_codes", "v_codes", "k_meta", "v_meta"):
        d = getattr(dev, name).cpu().numpy()
        o = getattr(orc, name)
        if name.endswith("meta"):
            d, o = d.view(np.uint16), o.view(np.uint16)
        d = np.moveaxis(d, 1, 2)      # [page, off, head, ...]
        o = np.moveaxis(o, 1, 2)
        assert np.array_equal(d[mask], o[mask]), f"{name}: written slots differ"
        assert np.array_equal(d[~mask], o[~mask]), f"{name}: untouched slots were modified"


SMALL = [
    wl.CONFIGS["tiny"],
    wl.scaled(wl.CONFIGS["opt13b"], B=9, max_len=700),
    wl.scaled(wl.CONFIGS["llama7b"], B=10, max_len=1300),
    wl.replace(wl.scaled(wl.CONFIGS["gqa70b"], B=4, max_len=900), length_law="uniform:100,900"),
    wl.scaled(wl.CONFIGS["int4"], B=24, max_len=1700),
    wl.replace(wl.scaled(wl.CONFIGS["int4"], B=6, max_len=600, name="int4_d64"), D=64, G=32, P=32),
    wl.replace(wl.scaled(wl.CONFIGS["opt13b"], B=5, max_len=300, name="int8_g16_p8"), G=16, P=8, Hkv=3, H=3),
    wl.replace(wl.scaled(wl.CONFIGS["int4"], B=5, max_len=400, name="int4_g128_gqa"), G=128, Hkv=2, H=6, P=64),
    # grouped-query layouts on the matrix-core path: two groups per row, 16 and 3 query heads per KV head
    wl.replace(wl.scaled(wl.CONFIGS["gqa70b"], B=5, max_len=700, name="gqa_g64_p16"), G=64, P=16, Hkv=2, H=8,
               length_law="uniform:1,700"),
    wl.replace(wl.scaled(wl.CONFIGS["gqa70b"], B=4, max_len=600, name="gqa_q16_p64"), G=128, P=64, Hkv=1, H=16,
               length_law="uniform:30,600"),
    wl.replace(wl.scaled(wl.CONFIGS["gqa70b"], B=6, max_len=300, name="gqa_q3"), G=128, P=32, Hkv=2, H=6,
               length_law="uniform:1,300"),
    # INT4 with groups of 32 on the matrix-core path: 8, 16 and 3 query heads per KV head, long splits
    wl.replace(wl.scaled(wl.CONFIGS["gqa70b"], B=5, max_len=2600, name="gqa_int4_q8"), bits=4, G=32, P=32, Hkv=2, H=16,
               length_law="uniform:1,2600"),
    wl.replace(wl.scaled(wl.CONFIGS["gqa70b"], B=4, max_len=600, name="gqa_int4_q16_p16"), bits=4, G=32, P=16, Hkv=1, H=16,
               length_law="uniform:30,600"),
    # grouped-query layouts that stay on the vector kernel: head_dim 64, and 32 query heads per KV head
    wl.replace(wl.scaled(wl.CONFIGS["gqa70b"], B=6, max_len=900, name="gqa_d64_vector"), D=64, G=64, P=16, Hkv=2, H=8,
               length_law="uniform:1,900"),
    wl.replace(wl.scaled(wl.CONFIGS["gqa70b"], B=4, max_len=700, name="gqa_q32_vector"), G=128, P=32, Hkv=1, H=32,
               length_law="uniform:1,700"),
    # the largest pages: 128 and 256 tokens, vector and matrix-core path
    wl.replace(wl.scaled(wl.CONFIGS["llama7b"], B=7, max_len=2300, name="mha_p256"), P=256, Hkv=2, H=2, length_law="uniform:1,2300"),
    wl.replace(wl.scaled(wl.CONFIGS["int4"], B=7, max_len=2300, name="mha_int4_p128"), P=128, Hkv=2, H=2, length_law="uniform:1,2300"),
    wl.replace(wl.scaled(wl.CONFIGS["gqa70b"], B=6, max_len=3000, name="gqa_p256"), P=256, Hkv=2, H=16, length_law="uniform:1,3000"),
    wl.replace(wl.scaled(wl.CONFIGS["gqa70b"], B=6, max_len=3000, name="gqa_int4_p128"), bits=4, G=32, P=128, Hkv=2, H=8,
               length_law="uniform:1,3000"),
    # INT4 with one and two scale groups per head on the matrix-core path
    wl.replace(wl.scaled(wl.CONFIGS["gqa70b"], B=5, max_len=2600, name="gqa_int4_g64_q8"), bits=4, G=64, P=16, Hkv=2, H=16,
               length_law="uniform:1,2600"),
    wl.replace(wl.scaled(wl.CONFIGS["gqa70b"], B=5, max_len=1500, name="gqa_int4_g128_q4"), bits=4, G=128, P=32, Hkv=2, H=8,
               length_law="uniform:1,1500"),
    wl.replace(wl.scaled(wl.CONFIGS["gqa70b"], B=6, max_len=300, name="gqa_int4_q3"), bits=4, G=32, P=64, Hkv=2, H=6,
               length_law="uniform:1,300"),
]


@pytest.mark.parametrize("layout", ["interleaved", "dense"])
@pytest.mark.parametrize("w", SMALL, ids=lambda w: w.name)
def test_write_attend_dequant(env, w, layout):
    B, torch, oracle = env
    print(f"case {w.name} ({layout}): B={w.B} H={w.H} Hkv={w.Hkv} D={w.D} P={w.P} bits={w.bits} G={w.G}", flush=True)
    pg, pool, offs, gain = _problem(w)
    orc = harness.fill_oracle_cache(oracle, w, pg, pool, offs, gain)
    dev = harness.fill_device_cache(B, torch, w, pg, pool, offs, gain, max_tokens_per_call=777, layout=layout)
    _compare_caches(w, pg, dev, orc)

    q = wl.queries(w)
    want = oracle.paged_decode_attn(orc, q, pg.block_tables, pg.lens, 1.0 / np.sqrt(w.D), num_threads=8)
    got = harness.run_device_attn(B, torch, w, dev, q, pg).astype(np.float64)
    assert np.isfinite(got).all()
    err = np.abs(got - want).max()
    print(f"  max-abs attention error {err:.3e}", flush=True)
    assert err <= ATTN_TOL

    # page dequantizer on a fully written page, a partly written one and the untouched one
    last = int(np.argmax(pg.lens % w.P != 0)) if np.any(pg.lens % w.P != 0) else 0
    pages = {int(pg.block_tables[0, 0]), int(pg.block_tables[last, (int(pg.lens[last]) - 1) // w.P])}
    k_out = torch.empty((w.P, w.Hkv, w.D), dtype=torch.float16, device="cuda")
    v_out = torch.empty_like(k_out)
    written = harness.written_mask(w, pg)
    for page in pages:
        B.alise_kv_dequant_page(dev, page, k_out, v_out)
        torch.cuda.synchronize()
        ko, vo = oracle.kv_dequant_page(orc, page)
        rows = written[page]
        assert np.array_equal(k_out.cpu().numpy().view(np.uint16)[rows], ko.view(np.uint16)[rows])
        assert np.array_equal(v_out.cpu().numpy().view(np.uint16)[rows], vo.view(np.uint16)[rows])


@pytest.mark.parametrize("bits,G,H", [(8, 64, 4), (4, 32, 4), (8, 128, 16)])
def test_edge_lengths_and_splits(env, bits, G, H):
    """Empty and one-token requests, lengths around page and split boundaries, several splits;
    H = 16 over 4 KV heads takes the grouped-query path (splits of 256 tokens)."""
    B, torch, oracle = env
    lens = np.array([0, 1, 15, 16, 17, 31, 32, 33, 63, 64, 65, 255, 256, 257, 511, 512, 513, 1024, 1025, 2, 2100, 0, 3],
                    np.int32)
    w = wl.Workload("edges", B=len(lens), H=H, Hkv=4, D=128, P=16, bits=bits, G=G,
                    length_law="fixed:1", seed=77 + bits, max_len=int(lens.max()))
    print(f"case edges bits={bits} G={G} H={H}", flush=True)
    pg, pool, offs, gain = _problem(w, lens)
    orc = harness.fill_oracle_cache(oracle, w, pg, pool, offs, gain)
    dev = harness.fill_device_cache(B, torch, w, pg, pool, offs, gain)
    _compare_caches(w, pg, dev, orc)
    q = wl.queries(w)
    want = oracle.paged_decode_attn(orc, q, pg.block_tables, pg.lens, 1.0 / np.sqrt(w.D), num_threads=8)
    got = harness.run_device_attn(B, torch, w, dev, q, pg).astype(np.float64)
    assert np.isfinite(got).all()
    assert not got[lens == 0].any()
    assert np.abs(got - want).max() <= ATTN_TOL
    # a larger max_context_len than any request changes the plan, not the result
    wide = np.full((w.B, pg.max_blocks + 70), pg.poison_page, np.int32)
    wide[:, :pg.max_blocks] = pg.block_tables
    pg_wide = wl.Paging(pg.lens, wide, pg.num_pages, pg.poison_page, wide.shape[1])
    got2 = harness.run_device_attn(B, torch, w, dev, q, pg_wide, max_len=int(lens.max()) + 1000).astype(np.float64)
    assert np.array_equal(got, got2)


def test_dominant_and_large_values(env):
    """Scores with a wide spread (running maximum moves a lot) and |v| large enough that
    a single V row carries almost all the weight."""
    B, torch, oracle = env
    print("case dominant", flush=True)
    rng = np.random.default_rng(5)
    Hkv, D, P, L = 2, 128, 16, 700
    w = wl.Workload("dom", B=2, H=2, Hkv=Hkv, D=D, P=P, bits=8, G=32, length_law="fixed:700", seed=5, max_len=L)
    pg = wl.paging(w, np.array([L, L], np.int32))
    q = rng.standard_normal((2, Hkv, D)).astype(np.float16)
    k = (rng.standard_normal((2, L, Hkv, D)) * 0.2).astype(np.float16)
    v = (rng.standard_normal((2, L, Hkv, D)) * 0.8).astype(np.float16)
    # keys that grow towards the end: every block brings a new maximum
    ramp = np.linspace(0.0, 6.0, L, dtype=np.float32)[None, :, None, None]
    k = (k.astype(np.float32) + ramp * q[:, None].astype(np.float32) / np.sqrt(D)).astype(np.float16)
    k[1, 123] = (q[1].astype(np.float32) * 3).astype(np.float16)      # one dominant key
    orc = oracle.Cache.empty(pg.num_pages, P, Hkv, D, 8, 32)
    dev = B.KVCache.allocate(pg.num_pages, P, Hkv, D, 8, 32, fill=0)
    for i in range(2):
        slots = wl.slots_of(w, pg, i, 0, L)
        oracle.kv_quant_write(orc, k[i], v[i], slots)
        B.alise_kv_quant_write(dev, torch.from_numpy(k[i]).cuda(), torch.from_numpy(v[i]).cuda(),
                               torch.from_numpy(slots).cuda())
    torch.cuda.synchronize()
    _compare_caches(w, pg, dev, orc)
    want = oracle.paged_decode_attn(orc, q, pg.block_tables, pg.lens, 1.0 / np.sqrt(D))
    got = harness.run_device_attn(B, torch, w, dev, q, pg).astype(np.float64)
    assert np.abs(got - want).max() <= ATTN_TOL


def test_skipped_slots_and_empty_write(env):
    B, torch, oracle = env
    print("case skipped slots", flush=True)
    rng = np.random.default_rng(8)
    P, Hkv, D, T = 16, 5, 64, 33
    dev = B.KVCache.allocate(4, P, Hkv, D, 4, 32, fill=0x5A, layout="dense")
    orc = oracle.Cache.empty(4, P, Hkv, D, 4, 32, fill=0x5A)
    dev.k_meta.fill_(0.0)
    dev.v_meta.fill_(0.0)
    k = rng.standard_normal((T, Hkv, D)).astype(np.float16)
    v = rng.standard_normal((T, Hkv, D)).astype(np.float16)
    slots = rng.permutation(4 * P)[:T].astype(np.int64)
    slots[[0, 7, 32]] = -1
    oracle.kv_quant_write(orc, k, v, slots)
    B.alise_kv_quant_write(dev, torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda(), torch.from_numpy(slots).cuda())
    B.alise_kv_quant_write(dev, torch.empty((0, Hkv, D), dtype=torch.float16, device="cuda"),
                           torch.empty((0, Hkv, D), dtype=torch.float16, device="cuda"),
                           torch.empty(0, dtype=torch.int64, device="cuda"))
    torch.cuda.synchronize()
    for name in ("k_codes", "v_codes", "k_meta", "v_meta"):
        d = getattr(dev, name).cpu().numpy()
        o = getattr(orc, name)
        if name.endswith("meta"):
            d, o = d.view(np.uint16), o.view(np.uint16)
        assert np.array_equal(d, o), name


def test_quantizer_corner_values(env):
    """Groups built to sit on rounding ties, the scale floor, subnormals and the fp16 maximum."""
    B, torch, oracle = env
    print("case quantizer corners", flush=True)
    rng = np.random.default_rng(13)
    P, Hkv, D = 16, 2, 128
    for bits, G in ((8, 16), (8, 128), (4, 32)):
        T = 64
        x = rng.standard_normal((2, T, Hkv, D)).astype(np.float16)
        x[:, 0] = 0
        x[:, 1] = np.float16(6e-8)
        x[:, 2] = np.float16(-6e-8)
        x[:, 3] = np.float16(65504.0)
        x[:, 4, :, ::2] = np.float16(-65504.0)
        x[:, 5] = np.float16(0.3)
        x[:, 6] = (np.arange(D) % 16 * (1 / 64)).astype(np.float16)          # exact multiples of a power-of-two scale
        x[:, 7] = ((np.arange(D) % 32) * 0.5 / 64 + 0.25 / 64).astype(np.float16)   # half-way values
        x[:, 8] = (rng.integers(-255, 256, (Hkv, D)) * 2.0 ** -10).astype(np.float16)
        x[:, 9] = np.abs(x[:, 9])
        x[:, 10] = -np.abs(x[:, 10])
        x[:, 11] = (rng.standard_normal((Hkv, D)) * 1e-4).astype(np.float16)
        x[:, 12] = (rng.standard_normal((Hkv, D)) * 3e3).astype(np.float16)
        dev = B.KVCache.allocate(T // P, P, Hkv, D, bits, G, fill=0)
        orc = oracle.Cache.empty(T // P, P, Hkv, D, bits, G)
        slots = np.arange(T, dtype=np.int64)
        oracle.kv_quant_write(orc, x[0], x[1], slots)
        B.alise_kv_quant_write(dev, torch.from_numpy(x[0]).cuda(), torch.from_numpy(x[1]).cuda(),
                               torch.from_numpy(slots).cuda())
        torch.cuda.synchronize()
        for name in ("k_codes", "v_codes", "k_meta", "v_meta"):
            d = getattr(dev, name).cpu().numpy()
            o = getattr(orc, name)
            if name.endswith("meta"):
                d, o = d.view(np.uint16), o.view(np.uint16)
            assert np.array_equal(d, o), (bits, G, name)


def test_invariances_on_device(env):
    """Page permutation and batch order leave the device result unchanged (bit for bit:
    the arithmetic per request does not depend on where its pages live)."""
    B, torch, oracle = env
    print("case invariances", flush=True)
    w = wl.scaled(wl.CONFIGS["llama7b"], B=7, max_len=900)
    pg, pool, offs, gain = _problem(w)
    dev = harness.fill_device_cache(B, torch, w, pg, pool, offs, gain)
    q = wl.queries(w)
    base = harness.run_device_attn(B, torch, w, dev, q, pg)
    rng = np.random.default_rng(3)
    perm = rng.permutation(pg.num_pages)
    dev2 = B.KVCache.allocate(pg.num_pages, w.P, w.Hkv, w.D, w.bits, w.G)
    idx = torch.from_numpy(perm).cuda()
    for name in ("k_codes", "v_codes", "k_meta", "v_meta"):
        getattr(dev2, name)[idx] = getattr(dev, name)
    pg2 = wl.Paging(pg.lens, perm[pg.block_tables].astype(np.int32), pg.num_pages, int(perm[pg.poison_page]), pg.max_blocks)
    out2 = harness.run_device_attn(B, torch, w, dev2, q, pg2)
    assert np.array_equal(base.view(np.uint16), out2.view(np.uint16))
    order = rng.permutation(w.B)
    pg3 = wl.Paging(pg.lens[order], pg.block_tables[order], pg.num_pages, pg.poison_page, pg.max_blocks)
    out3 = harness.run_device_attn(B, torch, w, dev, q[order], pg3)
    assert np.array_equal(base[order].view(np.uint16), out3.view(np.uint16))


@pytest.mark.parametrize("bits,G,Hkv,H", [(8, 64, 4, 4), (4, 32, 4, 4), (8, 128, 2, 16), (4, 32, 2, 16), (8, 64, 2, 6)])
@pytest.mark.parametrize("qgain", [1.0, 3.0, 8.0])
def test_peaked_rows_with_values_up_to_the_fp16_limit_of_the_bar(env, bits, G, Hkv, H, qgain):
    """Dequantized V values just below 4 are the largest for which an fp16 output can meet 2e-3 at all (half an
    ulp is 9.8e-4 in [2, 4) and 1.95e-3 in [4, 8)).  Scaled queries make the rows peaked: a few tokens carry the
    sum and whatever error their weights have reaches the output unaveraged.  Vector kernel (MHA) and
    matrix-core kernel (GQA), INT8 and INT4, long requests split into tiles."""
    B, torch, oracle = env
    print(f"case peaked bits {bits} G {G} Hkv {Hkv} H {H} qgain {qgain}", flush=True)
    D, P = 128, 16
    lens = np.array([333, 1, 64, 2600, 17], np.int32)
    vmax = 3.9 if bits == 8 else 3.5              # INT4 steps are 0.5 wide: the dequantized values reach vmax + 0.25
    rng = np.random.default_rng([2025, bits, G, H, int(qgain)])
    w = wl.Workload("peaked", B=len(lens), H=H, Hkv=Hkv, D=D, P=P, bits=bits, G=G, length_law="fixed:1", seed=11, max_len=int(lens.max()))
    pg = wl.paging(w, lens)
    orc = oracle.Cache.empty(pg.num_pages, P, Hkv, D, bits, G)
    dev = B.KVCache.allocate(pg.num_pages, P, Hkv, D, bits, G, fill=0)
    for i, L in enumerate(lens):
        k = rng.standard_normal((int(L), Hkv, D)).astype(np.float16)
        v = rng.uniform(-vmax, vmax, (int(L), Hkv, D)).astype(np.float16)
        slots = wl.slots_of(w, pg, i, 0, int(L))
        oracle.kv_quant_write(orc, k, v, slots)
        B.alise_kv_quant_write(dev, torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda(), torch.from_numpy(slots).cuda())
    q = (rng.standard_normal((len(lens), H, D)) * qgain).astype(np.float16)
    want = oracle.paged_decode_attn(orc, q, pg.block_tables, pg.lens, 1.0 / np.sqrt(D))
    assert np.abs(want).max() < 4.0
    got = harness.run_device_attn(B, torch, w, dev, q, pg).astype(np.float64)
    err = np.abs(got - want).max()
    print(f"  max|want| {np.abs(want).max():.3f} max-abs error {err:.3e}", flush=True)
    assert np.isfinite(got).all() and err <= ATTN_TOL


@pytest.mark.parametrize("bits,G,Hkv,H", [(8, 64, 2, 2), (4, 32, 2, 2), (8, 128, 1, 8)])
def test_more_requests_than_a_plan_pass_holds(env, bits, G, Hkv, H):
    """2 300 requests: the plan kernels take the batch 1024 requests at a time (scans carried from pass to
    pass, merge list and tile bases across passes).  Mostly short requests, empty ones, and a few long
    enough to be split, scattered over the batch; decode on the vector and the matrix-core path, then
    prefill chunks of a few tokens for every third request."""
    B, torch, oracle = env
    rng = np.random.default_rng([31, bits, H])
    n = 2300
    lens = rng.integers(0, 40, n).astype(np.int32)
    lens[rng.choice(n, 12, replace=False)] = rng.integers(600, 2500, 12).astype(np.int32)
    w = wl.Workload("many", B=n, H=H, Hkv=Hkv, D=128, P=16, bits=bits, G=G, length_law="fixed:1", seed=123, max_len=int(lens.max()))
    print(f"case many requests bits={bits} G={G} H={H}", flush=True)
    pg, pool, offs, gain = _problem(w, lens)
    orc = harness.fill_oracle_cache(oracle, w, pg, pool, offs, gain)
    dev = harness.fill_device_cache(B, torch, w, pg, pool, offs, gain)
    q = wl.queries(w)
    want = oracle.paged_decode_attn(orc, q, pg.block_tables, pg.lens, 1.0 / np.sqrt(w.D), num_threads=8)
    got = harness.run_device_attn(B, torch, w, dev, q, pg).astype(np.float64)
    assert np.isfinite(got).all() and not got[lens == 0].any()
    assert np.abs(got - want).max() <= ATTN_TOL

    chunk = np.where(np.arange(n) % 3 == 0, np.minimum(lens, 5), 0).astype(np.int64)
    chunk[lens >= 600] = 70
    q_start = np.concatenate([[0], np.cumsum(chunk)]).astype(np.int32)
    total = int(q_start[-1])
    qp_np = rng.standard_normal((total, H, 128)).astype(np.float16)
    wantp = oracle.paged_prefill_attn(orc, qp_np, q_start, pg.block_tables, pg.lens, 1.0 / np.sqrt(w.D))
    qp = torch.from_numpy(qp_np).cuda()
    op = torch.full(qp.shape, float("nan"), dtype=torch.float16, device="cuda")
    ws = torch.empty(B.alise_paged_prefill_attn_workspace_bytes(dev, n, total, H, int(lens.max())), dtype=torch.uint8, device="cuda")
    B.alise_paged_prefill_attn(dev, qp, op, torch.from_numpy(q_start).cuda(), torch.from_numpy(pg.block_tables).cuda(),
                               torch.from_numpy(pg.lens.astype(np.int32)).cuda(), int(lens.max()), 1.0 / np.sqrt(w.D), ws)
    torch.cuda.synchronize()
    gotp = op.cpu().numpy().astype(np.float64)
    assert np.isfinite(gotp).all() and np.abs(gotp - wantp).max() <= ATTN_TOL


@pytest.mark.parametrize("bits,G", [(8, 64), (8, 16), (4, 32), (4, 128)])
def test_every_scale_with_values_on_rounding_ties(env, bits, G):
    """The quantizer's two divisions are not written as divisions in the kernel (a constant reciprocal with one
    fma correction for (max - min) / qmax, one Newton step on the hardware reciprocal for 1 / scale); both must
    still be the correctly rounded quotients.  One group for every fp16 scale the format can produce, built so
    that its range lands just inside the interval that rounds up to that scale, and filled with values
    (k + 1/2 - zero) * scale: products with 1 / scale that sit on or next to a rounding tie, where a reciprocal
    off by one ulp flips the code.  Codes, scales and zero-points bit for bit against the oracle, which divides."""
    B, torch, oracle = env
    D, P, qmax = 128, 16, (1 << bits) - 1
    print(f"case every scale bits={bits} G={G}", flush=True)
    hs = np.arange(0x0400, 0x7C00, dtype=np.uint16)
    lam = hs.view(np.float16).astype(np.float64)
    hs, lam = hs[lam * qmax <= 131008.0 * 0.999], lam[lam * qmax <= 131008.0 * 0.999]
    ulp = lam - (hs - 1).astype(np.uint16).view(np.float16).astype(np.float64)
    rng = np.random.default_rng(bits * 1000 + G)
    target = qmax * (lam - ulp * rng.uniform(0.02, 0.98, lam.shape))          # inside (qmax * prev, qmax * lam)
    share = rng.uniform(0.3, 0.9, lam.shape)                                   # how much of the range is above zero
    mx16 = np.minimum(target * share, 65504.0).astype(np.float16)
    mx16 = np.where(mx16.astype(np.float64) > target * share, np.nextafter(mx16, np.float16(0)), mx16)
    mn16 = (-(np.minimum(target - mx16.astype(np.float64), 65504.0))).astype(np.float16)
    mx, mn = mx16.astype(np.float64), mn16.astype(np.float64)
    z = np.clip(np.rint(-mn / lam), 0, qmax)
    k = rng.integers(0, qmax, size=(len(lam), G))                              # codes 0 .. qmax - 1, then + 1/2
    x = ((k + 0.5 - z[:, None]) * lam[:, None])
    x = np.clip(x, mn[:, None], mx[:, None]).astype(np.float16)
    x = np.clip(x, mn16[:, None], mx16[:, None])                               # rounding to fp16 must not widen the range
    x[:, 0], x[:, 1] = mx16, mn16
    n_groups = len(lam) // (D // G) * (D // G)
    T = n_groups * G // D
    T -= T % P
    n_groups = T * D // G
    rows = x[:n_groups].reshape(T, 1, D)
    other = rng.standard_normal((T, 1, D)).astype(np.float16)
    slots = np.arange(T, dtype=np.int64)
    orc = oracle.Cache.empty(T // P, P, 1, D, bits, G, fill=0)
    oracle.kv_quant_write(orc, rows, other, slots)
    got_scales = orc.k_meta.view(np.uint16).reshape(-1, 2)[:, 0]
    hit = np.isin(hs[:n_groups], got_scales)
    print(f"  {n_groups} groups, {len(np.unique(got_scales))} distinct scales, {hit.mean() * 100:.1f} % of the targets produced", flush=True)
    assert hit.mean() > 0.85
    for T_call in (T, 512):                    # the head-major numbering of large writes and the token-major one
        dev = B.KVCache.allocate(T // P, P, 1, D, bits, G, fill=0)
        for t0 in range(0, T, T_call):
            t1 = min(T, t0 + T_call)
            B.alise_kv_quant_write(dev, torch.from_numpy(rows[t0:t1]).cuda(), torch.from_numpy(other[t0:t1]).cuda(),
                                   torch.from_numpy(slots[t0:t1]).cuda())
        torch.cuda.synchronize()
        for name in ("k_codes", "v_codes", "k_meta", "v_meta"):
            d, o = getattr(dev, name).cpu().numpy(), getattr(orc, name)
            if name.endswith("meta"):
                d, o = d.view(np.uint16), o.view(np.uint16)
            bad = np.argwhere(d != o)
            assert len(bad) == 0, f"{name}, writes of {T_call} tokens: {len(bad)} differ, first at {bad[0]}"
