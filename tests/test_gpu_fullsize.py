"""Parity at the full benchmark sizes, in the launch configuration bench.py times.

The whole step (quantize-and-write of the step's tokens, paged attention, page
dequantize) runs on the device exactly as in bench.py; the oracle fills a cache of
its own for the whole batch from the same seeded inputs and attends the whole
batch: every written code and meta byte is compared bit for bit, every element of
the attention output within 2e-3.  The prefill leg is compared on sampled query
tokens (the oracle would need minutes per configuration for all of them).
"""
import numpy as np
import pytest

from paper_2410_23537_amd import workloads as wl

pytestmark = pytest.mark.gpu

ATTN_TOL = 2e-3


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2410_23537_amd import binding
    from paper_2410_23537_amd.decode_step import DecodeStep
    import oracle
    oracle.build()
    return binding, torch, oracle, DecodeStep


def _oracle_cache_of_whole_batch(oracle, st, threads=16):
    """The oracle's own cache of the whole batch, filled from the same seeded inputs by the oracle's writer
    (requests own disjoint pages, so they are written side by side)."""
    from concurrent.futures import ThreadPoolExecutor
    w, pg = st.w, st.pg
    cache = oracle.Cache.empty(pg.num_pages, w.P, w.Hkv, w.D, w.bits, w.G)

    def fill(i):
        L = int(st.lens[i])
        k, v = wl.request_kv(w, st.pool_host, st.offs, i, 0, L, st.gain)
        slots = wl.slots_of(w, pg, i, 0, L)
        for a in range(0, L, 1024):
            oracle.kv_quant_write(cache, k[a:a + 1024], v[a:a + 1024], slots[a:a + 1024])

    with ThreadPoolExecutor(threads) as ex:
        list(ex.map(fill, range(w.B)))
    return cache


def _written_slots(w, pg):
    m = np.zeros((pg.num_pages, w.P), bool)
    for i, L in enumerate(pg.lens):
        s = wl.slots_of(w, pg, i, 0, int(L))
        m[s // w.P, s % w.P] = True
    return m


@pytest.mark.parametrize("name", ["int4", "llama7b", "gqa70b", "opt13b"])
def test_full_size_step_whole_output_against_oracle(env, name):
    """Every written code and meta byte of the whole cache bit for bit, every element of the attention output
    within 2e-3, the dequantized page bit for bit: nothing is sampled."""
    B, torch, oracle, DecodeStep = env
    w = wl.CONFIGS[name]
    print(f"case full-size {name}: B={w.B} H={w.H} Hkv={w.Hkv} bits={w.bits} G={w.G}", flush=True)
    st = DecodeStep(w)
    st.populate()                      # context only; the step's own tokens are written by step()
    st.out.fill_(float("nan"))
    st.step()
    torch.cuda.synchronize()
    out = st.out.cpu().numpy().astype(np.float64)
    assert out.shape == (w.B, w.H, w.D)

    orc = _oracle_cache_of_whole_batch(oracle, st)
    print(f"  oracle cache filled: {int(st.lens.astype(np.int64).sum())} tokens", flush=True)
    written = _written_slots(w, st.pg)
    assert int(written.sum()) == int(st.lens.astype(np.int64).sum())
    cache = st.caches[0]
    step_pages = 4096                   # compare in slabs: the arrays are gigabytes
    for arr in ("k_codes", "v_codes", "k_meta", "v_meta"):
        dev_t, ref = getattr(cache, arr), getattr(orc, arr)
        compared = 0
        for p0 in range(0, st.pg.num_pages, step_pages):
            p1 = min(st.pg.num_pages, p0 + step_pages)
            dev = dev_t[p0:p1].contiguous().cpu().numpy()
            r = ref[p0:p1]
            if arr.endswith("meta"):
                dev, r = dev.view(np.uint16).reshape(p1 - p0, w.Hkv, w.P, -1), r.view(np.uint16).reshape(p1 - p0, w.Hkv, w.P, -1)
            differ = (dev != r).any(axis=-1) & written[p0:p1, None, :]
            assert not differ.any(), f"{arr}: {int(differ.sum())} written (page, head, slot) rows differ in pages {p0}..{p1}"
            compared += int(written[p0:p1].sum()) * w.Hkv
        assert compared == int(st.lens.astype(np.int64).sum()) * w.Hkv
    print("  codes and meta of every written slot bit-exact", flush=True)

    want = oracle.paged_decode_attn(orc, st.q_host, st.pg.block_tables, st.lens, st.scale, num_threads=16)
    assert want.shape == out.shape
    err = np.abs(out - want)                 # NaN (a row the device never wrote) fails the comparison below
    worst = float(np.nanmax(err))
    assert np.isfinite(out).all() and (err <= ATTN_TOL).all(), \
        f"{int((~(err <= ATTN_TOL)).sum())} of {err.size} outputs beyond {ATTN_TOL}; worst {worst}"
    print(f"  all {err.size} attention outputs within {ATTN_TOL}: worst {worst:.3e}", flush=True)

    # the page dequantized in the step
    ko, vo = oracle.kv_dequant_page(orc, st.dq_page)
    rows = written[st.dq_page]
    assert rows.any()
    assert np.array_equal(st.dq_k.cpu().numpy().view(np.uint16)[rows], ko.view(np.uint16)[rows])
    assert np.array_equal(st.dq_v.cpu().numpy().view(np.uint16)[rows], vo.view(np.uint16)[rows])


@pytest.mark.parametrize("name", ["llama7b", "gqa70b", "int4"])
def test_full_size_prefill_sampled_against_oracle(env, name):
    """The prefill leg of bench.py (every 8th request brings its last min(512, L) tokens) on the
    full cache; sampled query tokens are recomputed by the oracle from the same seeded inputs."""
    B, torch, oracle, DecodeStep = env
    w = wl.CONFIGS[name]
    st = DecodeStep(w)
    st.populate(include_step_tokens=True)
    cache = st.caches[0]
    lens = st.lens.astype(np.int64)
    n = np.array([min(512, int(L)) if i % 8 == 0 else 0 for i, L in enumerate(lens)], np.int64)
    q_start = np.concatenate([[0], np.cumsum(n)]).astype(np.int32)
    total = int(q_start[-1])
    print(f"case full-size prefill {name}: {total} query tokens of {int((n > 0).sum())} requests", flush=True)
    rng = np.random.default_rng(w.seed + 5)
    q_np = rng.standard_normal((total, w.H, w.D)).astype(np.float16)
    q = torch.from_numpy(q_np).cuda()
    out = torch.full(q.shape, float("nan"), dtype=torch.float16, device="cuda")
    bt = torch.from_numpy(st.pg.block_tables).cuda()
    lens_d = torch.from_numpy(st.lens.astype(np.int32)).cuda()
    qs = torch.from_numpy(q_start).cuda()
    ws = torch.empty(B.alise_paged_prefill_attn_workspace_bytes(cache, w.B, total, w.H, int(st.lens.max())), dtype=torch.uint8, device="cuda")
    B.alise_paged_prefill_attn(cache, q, out, qs, bt, lens_d, int(st.lens.max()), st.scale, ws)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()

    worst = 0.0
    chunked = [i for i in range(w.B) if n[i] > 0]
    for i in (chunked[0], chunked[len(chunked) // 2], chunked[-1], chunked[int(np.argmax(lens[chunked]))]):
        L, ni = int(lens[i]), int(n[i])
        k, v = wl.request_kv(w, st.pool_host, st.offs, i, 0, L, st.gain)
        nblk = (L + w.P - 1) // w.P
        mini = oracle.Cache.empty(nblk, w.P, w.Hkv, w.D, w.bits, w.G)
        oracle.kv_quant_write(mini, k, v, np.arange(L, dtype=np.int64))
        rows = sorted({0, ni - 1, ni // 2} | {int(r) for r in rng.integers(0, ni, 3)})
        for j in rows:
            # a one-token "chunk" at position L - ni + j: the request cut to that length
            Lj = L - ni + j + 1
            want = oracle.paged_prefill_attn(mini, q_np[q_start[i] + j][None], np.array([0, 1], np.int32),
                                             np.arange(nblk, dtype=np.int32)[None], np.array([Lj], np.int32), st.scale)[0]
            err = np.abs(got[q_start[i] + j] - want).max()
            worst = max(worst, err)
            assert err <= ATTN_TOL, f"request {i} (L={L}) query {j}: max-abs {err}"
    print(f"  worst sampled prefill error {worst:.3e}", flush=True)


def test_full_size_prefill_whole_output_against_oracle(env):
    """The prefill leg of the OPT-13B-shaped configuration, every query token of it: the one configuration whose
    whole prefill output the oracle attends in seconds (2 599 query tokens, 1.3 M (query, key) pairs per head)."""
    B, torch, oracle, DecodeStep = env
    w = wl.CONFIGS["opt13b"]
    st = DecodeStep(w)
    st.populate(include_step_tokens=True)
    cache = st.caches[0]
    lens = st.lens.astype(np.int64)
    n = np.array([min(512, int(L)) if i % 8 == 0 else 0 for i, L in enumerate(lens)], np.int64)
    q_start = np.concatenate([[0], np.cumsum(n)]).astype(np.int32)
    total = int(q_start[-1])
    print(f"case full-size prefill, whole output, opt13b: {total} query tokens", flush=True)
    rng = np.random.default_rng(w.seed + 6)
    q_np = rng.standard_normal((total, w.H, w.D)).astype(np.float16)
    q = torch.from_numpy(q_np).cuda()
    out = torch.full(q.shape, float("nan"), dtype=torch.float16, device="cuda")
    ws = torch.empty(B.alise_paged_prefill_attn_workspace_bytes(cache, w.B, total, w.H, int(st.lens.max())), dtype=torch.uint8, device="cuda")
    B.alise_paged_prefill_attn(cache, q, out, torch.from_numpy(q_start).cuda(), torch.from_numpy(st.pg.block_tables).cuda(),
                               torch.from_numpy(st.lens.astype(np.int32)).cuda(), int(st.lens.max()), st.scale, ws)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    orc = _oracle_cache_of_whole_batch(oracle, st)
    want = oracle.paged_prefill_attn(orc, q_np, q_start, st.pg.block_tables, st.lens, st.scale, num_threads=16)
    err = np.abs(got - want)
    assert np.isfinite(got).all() and (err <= ATTN_TOL).all(), f"worst {np.nanmax(err)}"
    print(f"  all {err.size} prefill outputs within {ATTN_TOL}: worst {err.max():.3e}", flush=True)
