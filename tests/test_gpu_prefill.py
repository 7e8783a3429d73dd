"""GPU parity of chunked-prefill attention (ALISE Sec. 2 "LLM Inference", Eq. 1-2 in causal
order, over the quantized cache of Sec. 3.2) against the CPU oracle, through the C ABI.
The fp16 output must be within 2e-3 max-abs of the fp64 oracle, like the decode step."""
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


def _w(name, **kw):
    base = dict(B=4, H=8, Hkv=8, D=128, P=16, bits=8, G=64, length_law="fixed:1", seed=4100, max_len=4096)
    base.update(kw)
    return wl.Workload(name=name, **base)


# (workload, context lengths, chunk lengths): chunks of 0, 1, exactly one wave / one workgroup of
# rows, ragged ones, whole prompts, a context that crosses several 64-page windows
CASES = [
    (_w("mha_g64_p16"), [40, 200, 65, 1, 333, 64], [40, 7, 65, 1, 0, 64]),
    (_w("mha_g128_p32", G=128, P=32, Hkv=4, H=4), [500, 129, 96], [300, 129, 1]),
    (_w("mha_long_context", Hkv=2, H=2), [2500, 1100], [70, 33]),
    (_w("gqa8_g128_p32", G=128, P=32, Hkv=2, H=16), [300, 77, 150], [100, 77, 9]),
    (_w("gqa2_g64_p16", Hkv=4, H=8), [210, 18], [210, 5]),
    (_w("gqa16_p64", G=128, P=64, Hkv=1, H=16), [400, 50], [37, 50]),
    (_w("gqa3_g128_p16", G=128, Hkv=2, H=6), [90, 260], [90, 41]),
    (_w("gqa4", Hkv=2, H=8), [1, 17, 128], [1, 17, 128]),
    (_w("int4_g32_mha", bits=4, G=32, Hkv=4, H=4), [40, 200, 65, 1, 333, 64], [40, 7, 65, 1, 0, 64]),
    (_w("int4_g32_long", bits=4, G=32, Hkv=2, H=2), [2500, 1100], [70, 33]),
    (_w("int4_g32_gqa4_p32", bits=4, G=32, P=32, Hkv=2, H=8), [300, 77, 150], [100, 77, 9]),
    (_w("mha_p256", P=256, Hkv=2, H=2), [700, 256, 257, 40], [300, 256, 1, 40]),
    (_w("gqa8_int4_p128", bits=4, G=32, P=128, Hkv=1, H=8), [1500, 129, 128], [200, 129, 7]),
    (_w("int4_g64_mha", bits=4, G=64, Hkv=4, H=4), [40, 200, 65, 1, 333, 64], [40, 7, 65, 1, 0, 64]),
    (_w("int4_g64_gqa8_long", bits=4, G=64, P=32, Hkv=1, H=8), [2500, 1100], [70, 33]),
    (_w("int4_g128_mha_long", bits=4, G=128, Hkv=2, H=2), [2500, 300], [130, 300]),
    (_w("int4_g128_gqa4_p64", bits=4, G=128, P=64, Hkv=2, H=8), [300, 77, 150], [100, 77, 9]),
]


@pytest.mark.parametrize("layout", ["interleaved", "dense"])
@pytest.mark.parametrize("case", CASES, ids=lambda c: c[0].name)
def test_prefill_against_oracle(env, case, layout):
    B, torch, oracle = env
    w, lens, chunks = case
    w = wl.replace(w, B=len(lens))
    print(f"case prefill {w.name} ({layout}): H={w.H} Hkv={w.Hkv} P={w.P} G={w.G} lens={lens} chunks={chunks}", flush=True)
    pg = wl.paging(w, np.array(lens, np.int32))
    pool = wl.value_pool(w, n_min=max(lens) * w.Hkv * w.D)
    offs, gain = wl.request_offsets(w), wl.k_channel_gain(w)
    orc = harness.fill_oracle_cache(oracle, w, pg, pool, offs, gain)
    dev = harness.fill_device_cache(B, torch, w, pg, pool, offs, gain, layout=layout)

    q_start = np.concatenate([[0], np.cumsum(chunks)]).astype(np.int32)
    total = int(q_start[-1])
    rng = np.random.default_rng([w.seed, 7, len(lens)])
    q_np = rng.standard_normal((total, w.H, w.D)).astype(np.float16)
    scale = 1.0 / np.sqrt(w.D)
    want = oracle.paged_prefill_attn(orc, q_np, q_start, pg.block_tables, pg.lens, scale)

    q = torch.from_numpy(q_np).cuda()
    out = torch.full(q.shape, float("nan"), dtype=torch.float16, device="cuda")
    guard = torch.full((64, w.H, w.D), 7.0, dtype=torch.float16, device="cuda")      # rows nobody owns
    bt = torch.from_numpy(pg.block_tables).cuda()
    lens_d = torch.from_numpy(pg.lens.astype(np.int32)).cuda()
    qs_d = torch.from_numpy(q_start).cuda()
    max_len = int(max(lens))
    nbytes = B.alise_paged_prefill_attn_workspace_bytes(dev, len(lens), total, w.H, max_len)
    assert nbytes > 0
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    both = torch.cat([out, guard])              # the guard sits right behind the output
    B.alise_paged_prefill_attn(dev, q, both[:total], qs_d, bt, lens_d, max_len, scale, ws)
    torch.cuda.synchronize()
    got = both[:total].cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all(), "a row was not written"
    err = np.abs(got - want).max()
    print(f"  max-abs error {err:.3e}", flush=True)
    assert err <= ATTN_TOL
    assert (both[total:] == 7.0).all(), "wrote past the last row"


def test_one_token_chunks_equal_the_decode_call(env):
    B, torch, oracle = env
    w = wl.replace(wl.scaled(wl.CONFIGS["llama7b"], B=12, max_len=900), name="decode_as_prefill")
    pg = wl.paging(w)
    pool = wl.value_pool(w, n_min=int(pg.lens.max()) * w.Hkv * w.D)
    dev = harness.fill_device_cache(B, torch, w, pg, pool, wl.request_offsets(w), wl.k_channel_gain(w))
    q_np = wl.queries(w)
    dec = harness.run_device_attn(B, torch, w, dev, q_np, pg).astype(np.float64)
    q = torch.from_numpy(q_np).cuda()
    out = torch.full(q.shape, float("nan"), dtype=torch.float16, device="cuda")
    qs = torch.arange(w.B + 1, dtype=torch.int32, device="cuda")
    bt = torch.from_numpy(pg.block_tables).cuda()
    lens_d = torch.from_numpy(pg.lens.astype(np.int32)).cuda()
    ws = torch.empty(B.alise_paged_prefill_attn_workspace_bytes(dev, w.B, w.B, w.H, int(pg.lens.max())), dtype=torch.uint8, device="cuda")
    B.alise_paged_prefill_attn(dev, q, out, qs, bt, lens_d, int(pg.lens.max()), 1.0 / np.sqrt(w.D), ws)
    torch.cuda.synchronize()
    pre = out.cpu().numpy().astype(np.float64)
    # two kernels, two summation orders: both within the tolerance of the oracle, hence within twice of each other
    assert np.abs(pre - dec).max() <= 2 * ATTN_TOL


FALLBACK_LAYOUTS = [
    # layouts without a matrix-core prefill kernel: they run on the single-query kernel, one request per query token
    wl.Workload("tiny_d64", B=4, H=8, Hkv=8, D=64, P=16, bits=8, G=64, length_law="fixed:17,64,100,255", seed=1001, max_len=255),
    wl.Workload("page8", B=5, H=4, Hkv=2, D=128, P=8, bits=8, G=128, length_law="uniform:1,700", seed=41, max_len=700),
    wl.Workload("int8_g32", B=5, H=2, Hkv=2, D=128, P=16, bits=8, G=32, length_law="uniform:1,3000", seed=42, max_len=3000),
    wl.Workload("int8_g16_d64", B=4, H=4, Hkv=4, D=64, P=32, bits=8, G=16, length_law="uniform:1,500", seed=43, max_len=500),
    wl.Workload("int4_d64", B=4, H=4, Hkv=2, D=64, P=16, bits=4, G=32, length_law="uniform:1,900", seed=44, max_len=900),
    wl.Workload("gqa32", B=3, H=32, Hkv=1, D=128, P=16, bits=8, G=128, length_law="uniform:1,400", seed=45, max_len=400),
]


@pytest.mark.parametrize("w", FALLBACK_LAYOUTS, ids=lambda w: w.name)
def test_layouts_without_a_matrix_core_kernel(env, w):
    """Causal prefill over every layout the cache supports: chunks of mixed sizes (none, one token, the whole request,
    a longer one than the request), rows behind the last chunk that must stay untouched."""
    B, torch, oracle = env
    print(f"case prefill fallback {w.name}", flush=True)
    pg = wl.paging(w)
    lens = pg.lens.astype(np.int64)
    pool = wl.value_pool(w, n_min=int(lens.max()) * w.Hkv * w.D)
    offs, gain = wl.request_offsets(w), wl.k_channel_gain(w)
    orc = harness.fill_oracle_cache(oracle, w, pg, pool, offs, gain)
    dev = harness.fill_device_cache(B, torch, w, pg, pool, offs, gain)
    n = np.minimum(lens, [60, 0, 1, 10 ** 6, 33, 7][:w.B])
    q_start = np.concatenate([[0], np.cumsum(n)]).astype(np.int32)
    total = int(q_start[-1])
    rng = np.random.default_rng([w.seed, 3])
    q_np = rng.standard_normal((total + 5, w.H, w.D)).astype(np.float16)       # five rows that no chunk owns
    scale = 1.0 / np.sqrt(w.D)
    want = oracle.paged_prefill_attn(orc, q_np[:total], q_start, pg.block_tables, pg.lens, scale)
    q = torch.from_numpy(q_np).cuda()
    out = torch.full(q.shape, 7.0, dtype=torch.float16, device="cuda")
    max_len = int(lens.max())
    nbytes = B.alise_paged_prefill_attn_workspace_bytes(dev, w.B, total + 5, w.H, max_len)
    assert nbytes > 0
    ws = torch.full((nbytes,), 0xA5, dtype=torch.uint8, device="cuda")
    B.alise_paged_prefill_attn(dev, q, out, torch.from_numpy(q_start).cuda(), torch.from_numpy(pg.block_tables).cuda(),
                               torch.from_numpy(pg.lens.astype(np.int32)).cuda(), max_len, scale, ws)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    err = float(np.abs(got[:total] - want).max())
    print(f"  max-abs error {err:.3e}", flush=True)
    assert np.isfinite(got).all() and err <= ATTN_TOL
    assert (got[total:] == 7.0).all(), "rows behind the last chunk were written"
    with pytest.raises(B.AliseError) as e:
        B.alise_paged_prefill_attn(dev, q, out, torch.from_numpy(q_start).cuda(), torch.from_numpy(pg.block_tables).cuda(),
                                   torch.from_numpy(pg.lens.astype(np.int32)).cuda(), max_len, scale, ws[:nbytes - 256])
    assert e.value.status == B.ALISE_WORKSPACE_TOO_SMALL


@pytest.mark.parametrize("vgain", [1.0, 150.0, 20000.0])
def test_large_value_scales_decode_and_prefill(env, vgain):
    """V groups whose scale reaches 2 and more: the matrix-core kernels lower their weight bias for
    such steps (and only then).  The outputs are vgain times larger, so the bar is relative:
    the tolerance of the other tests scaled by the largest output magnitude."""
    B, torch, oracle = env
    Hkv, H, D, P, G = 2, 16, 128, 32, 128            # 8 query heads per KV head: matrix-core decode path too
    L, n_q = 700, 90
    rng = np.random.default_rng(99)
    k = rng.standard_normal((L, Hkv, D)).astype(np.float16)
    v = (rng.standard_normal((L, Hkv, D)) * vgain / 4.0).astype(np.float16)
    v[L // 2:] = (v[L // 2:].astype(np.float32) / vgain * 4.0).astype(np.float16)      # large scales first, ordinary ones after
    nblk = (L + P - 1) // P
    slots = np.arange(L, dtype=np.int64)
    orc = oracle.Cache.empty(nblk, P, Hkv, D, 8, G)
    oracle.kv_quant_write(orc, k, v, slots)
    dev = B.KVCache.allocate(nblk, P, Hkv, D, 8, G, fill=0)
    B.alise_kv_quant_write(dev, torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda(), torch.from_numpy(slots).cuda())
    scale = 1.0 / np.sqrt(D)
    bt_np = np.arange(nblk, dtype=np.int32)[None]
    bt = torch.from_numpy(bt_np).cuda()
    lens_np = np.array([L], np.int32)
    lens_d = torch.from_numpy(lens_np).cuda()

    q_np = rng.standard_normal((n_q, H, D)).astype(np.float16)
    q = torch.from_numpy(q_np).cuda()
    out = torch.full(q.shape, float("nan"), dtype=torch.float16, device="cuda")
    qs_np = np.array([0, n_q], np.int32)
    ws = torch.empty(B.alise_paged_prefill_attn_workspace_bytes(dev, 1, n_q, H, L), dtype=torch.uint8, device="cuda")
    B.alise_paged_prefill_attn(dev, q, out, torch.from_numpy(qs_np).cuda(), bt, lens_d, L, scale, ws)
    want = oracle.paged_prefill_attn(orc, q_np, qs_np, bt_np, lens_np, scale)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    bar = ATTN_TOL * max(1.0, np.abs(want).max() / 2.0)
    assert np.isfinite(got).all() and np.abs(got - want).max() <= bar, (np.abs(got - want).max(), bar)

    qd_np = q_np[-1:]                                   # decode: the last query token alone, over all L tokens
    qd = torch.from_numpy(qd_np).cuda()
    od = torch.full(qd.shape, float("nan"), dtype=torch.float16, device="cuda")
    wsd = torch.empty(B.alise_paged_decode_attn_workspace_bytes(dev, 1, H, L), dtype=torch.uint8, device="cuda")
    B.alise_paged_decode_attn(dev, qd, od, bt, lens_d, L, scale, wsd)
    torch.cuda.synchronize()
    wd = oracle.paged_decode_attn(orc, qd_np, bt_np, lens_np, scale)
    gd = od.cpu().numpy().astype(np.float64)
    bar = ATTN_TOL * max(1.0, np.abs(wd).max() / 2.0)
    assert np.isfinite(gd).all() and np.abs(gd - wd).max() <= bar, (np.abs(gd - wd).max(), bar)


def _peaked_problem(B, torch, oracle, bits, G, Hkv, H, qgain):
    """Three requests whose dequantized V values come close to 4 and whose queries are scaled by `qgain` (peaked
    rows for large gains), written by both sides; chunks of 80, 64 and 130 query tokens."""
    D, P = 128, 16
    lens = [333, 64, 1100]
    chunks = [80, 64, 130]
    vmax = 3.9 if bits == 8 else 3.5              # INT4 steps are 0.5 wide: the dequantized values reach vmax + 0.25
    rng = np.random.default_rng([2024, bits, G, H, int(qgain)])
    nblk_of = [(L + P - 1) // P for L in lens]
    num_pages = sum(nblk_of)
    orc = oracle.Cache.empty(num_pages, P, Hkv, D, bits, G)
    dev = B.KVCache.allocate(num_pages, P, Hkv, D, bits, G, fill=0)
    bt_np = np.zeros((len(lens), max(nblk_of)), np.int32)
    perm = rng.permutation(num_pages).astype(np.int32)
    at = 0
    for i, L in enumerate(lens):
        bt_np[i, :nblk_of[i]] = perm[at:at + nblk_of[i]]
        at += nblk_of[i]
        k = rng.standard_normal((L, Hkv, D)).astype(np.float16)
        v = rng.uniform(-vmax, vmax, (L, Hkv, D)).astype(np.float16)
        t = np.arange(L)
        slots = bt_np[i, t // P].astype(np.int64) * P + t % P
        oracle.kv_quant_write(orc, k, v, slots)
        B.alise_kv_quant_write(dev, torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda(), torch.from_numpy(slots).cuda())
    qs_np = np.concatenate([[0], np.cumsum(chunks)]).astype(np.int32)
    q_np = (rng.standard_normal((int(qs_np[-1]), H, D)) * qgain).astype(np.float16)
    return dev, orc, bt_np, np.array(lens, np.int32), qs_np, q_np


@pytest.fixture
def knobs(env):
    """Sets tuning variables for one test: the library reads its environment once and again on request."""
    import os
    B = env[0]
    touched = []

    def set_(**kw):
        for k, v in kw.items():
            touched.append((k, os.environ.get(k)))
            os.environ[k] = v
        B.alise_reload_environment()
    yield set_
    for k, old in reversed(touched):
        if old is None:
            os.environ.pop(k, None)
        else:
            os.environ[k] = old
    B.alise_reload_environment()


@pytest.mark.parametrize("weights", ["split", "single"])
@pytest.mark.parametrize("bits,G,Hkv,H", [(8, 64, 4, 4), (8, 128, 2, 16), (4, 32, 4, 4)])
@pytest.mark.parametrize("qgain", [1.0, 3.0, 8.0])
def test_peaked_rows_with_values_up_to_the_fp16_limit_of_the_bar(env, knobs, bits, G, Hkv, H, qgain, weights):
    """Dequantized V values just below 4 are the largest for which an fp16 output can meet 2e-3 at all (half an
    ulp is 9.8e-4 in [2, 4) and 1.95e-3 in [4, 8)); scaled queries make the rows peaked (a few tokens carry the
    sum, so errors of single weights do not average out), unscaled ones flat.  The default kernels (a weight
    as a high and a low fp16 part) must meet the bar there.  With ALISE_PREFILL_WEIGHTS=single a weight
    is one fp16 number rounded to nearest, which adds at most 2^-12 max|v| to the error: that bound is the bar."""
    B, torch, oracle = env
    knobs(ALISE_PREFILL_WEIGHTS=weights)
    dev, orc, bt_np, lens_np, qs_np, q_np = _peaked_problem(B, torch, oracle, bits, G, Hkv, H, qgain)
    lens, total = [int(x) for x in lens_np], int(qs_np[-1])
    scale = 1.0 / np.sqrt(128)
    want = oracle.paged_prefill_attn(orc, q_np, qs_np, bt_np, lens_np, scale)
    assert np.abs(want).max() < 4.0
    q = torch.from_numpy(q_np).cuda()
    out = torch.full(q.shape, float("nan"), dtype=torch.float16, device="cuda")
    ws = torch.empty(B.alise_paged_prefill_attn_workspace_bytes(dev, len(lens), total, H, max(lens)), dtype=torch.uint8, device="cuda")
    B.alise_paged_prefill_attn(dev, q, out, torch.from_numpy(qs_np).cuda(), torch.from_numpy(bt_np).cuda(),
                               torch.from_numpy(lens_np).cuda(), max(lens), scale, ws)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    err = np.abs(got - want)
    bar = ATTN_TOL if weights == "split" else ATTN_TOL + 2.0 ** -12 * 4.0
    print(f"  max|want| {np.abs(want).max():.3f} max-abs error {err.max():.3e} (bar {bar:.3e})", flush=True)
    assert np.isfinite(got).all() and err.max() <= bar


@pytest.mark.parametrize("bits,G,Hkv,H", [(8, 64, 4, 4), (8, 128, 2, 16), (4, 32, 2, 16), (4, 128, 4, 4)])
def test_hand_scheduled_instructions_on_peaked_rows(env, knobs, bits, G, Hkv, H):
    """The matrix-core kernels contain multiply-adds written in assembly that take softmax weights straight from the
    exponential instruction and bring their own wait states, and waits for loads placed by hand.  Nothing checks
    those at build time, so this does at run time: on peaked rows (the weights that matter come out of the
    exponential one instruction before they are used) every variant -- one and two row tiles per wave, split and
    single weights, and the grouped-query decode kernel -- runs twice with other work on the device in between, and
    must return the same bytes both times and the oracle's answer.  A missing wait state would show as a difference
    between the runs or as a row off the bar, not as noise inside it."""
    B, torch, oracle = env
    dev, orc, bt_np, lens_np, qs_np, q_np = _peaked_problem(B, torch, oracle, bits, G, Hkv, H, 8.0)
    lens, total = [int(x) for x in lens_np], int(qs_np[-1])
    scale = 1.0 / np.sqrt(128)
    want = oracle.paged_prefill_attn(orc, q_np, qs_np, bt_np, lens_np, scale)
    q = torch.from_numpy(q_np).cuda()
    bt, lens_d, qs = torch.from_numpy(bt_np).cuda(), torch.from_numpy(lens_np).cuda(), torch.from_numpy(qs_np).cuda()
    noise = torch.empty(1 << 26, dtype=torch.float16, device="cuda")
    for tiles in ("1", "2"):
        for weights in ("split", "single"):
            print(f"case hazards prefill bits={bits} G={G} H={H} row tiles {tiles} weights {weights}", flush=True)
            knobs(ALISE_PREFILL_ROW_TILES=tiles, ALISE_PREFILL_WEIGHTS=weights)
            ws = torch.empty(B.alise_paged_prefill_attn_workspace_bytes(dev, len(lens), total, H, max(lens)), dtype=torch.uint8, device="cuda")
            outs = []
            for rep in range(2):
                o = torch.full(q.shape, float("nan"), dtype=torch.float16, device="cuda")
                B.alise_paged_prefill_attn(dev, q, o, qs, bt, lens_d, max(lens), scale, ws)
                noise.normal_()                    # other kernels in between: the second run meets another machine state
                outs.append(o)
            torch.cuda.synchronize()
            assert torch.equal(outs[0].view(torch.int16), outs[1].view(torch.int16)), "two runs differ"
            err = np.abs(outs[0].cpu().numpy().astype(np.float64) - want).max()
            bar = ATTN_TOL if weights == "split" else ATTN_TOL + 2.0 ** -12 * 4.0
            assert err <= bar, (tiles, weights, err)
    if H > Hkv:
        # the grouped-query decode kernel on the same cache: the last token of every request as its query
        print(f"case hazards grouped-query decode bits={bits} G={G} H={H}", flush=True)
        qd_np = np.stack([q_np[qs_np[i + 1] - 1] for i in range(len(lens))])
        wd = oracle.paged_decode_attn(orc, qd_np, bt_np, lens_np, scale)
        qd = torch.from_numpy(qd_np).cuda()
        wsd = torch.empty(B.alise_paged_decode_attn_workspace_bytes(dev, len(lens), H, max(lens)), dtype=torch.uint8, device="cuda")
        outs = []
        for rep in range(2):
            o = torch.full(qd.shape, float("nan"), dtype=torch.float16, device="cuda")
            B.alise_paged_decode_attn(dev, qd, o, bt, lens_d, max(lens), scale, wsd)
            noise.normal_()
            outs.append(o)
        torch.cuda.synchronize()
        assert torch.equal(outs[0].view(torch.int16), outs[1].view(torch.int16)), "two runs differ"
        assert np.abs(outs[0].cpu().numpy().astype(np.float64) - wd).max() <= ATTN_TOL
