"""Parity at the full benchmark sizes, in the launch configuration bench.py times.

The whole step (quantize-and-write of the step's tokens, paged attention, page
dequantize) runs on the device exactly as in bench.py; the oracle then recomputes
sampled (request, KV head) pairs one by one from the same seeded inputs: codes and
meta of every token of the pair bit for bit, the attention rows of its query heads
within 2e-3.  Whole-output properties (finite, right shape) cover the rest.
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


def _samples(w, lens, n_random, rng):
    """(request, kv head) pairs: the longest and the shortest request, one per length quartile, a few random."""
    order = np.argsort(lens, kind="stable")
    reqs = {int(order[0]), int(order[-1])} | {int(order[int(f * (len(order) - 1))]) for f in (0.25, 0.5, 0.75)}
    reqs |= {int(r) for r in rng.integers(0, w.B, n_random)}
    return [(i, int(rng.integers(0, w.Hkv))) for i in sorted(reqs)]


@pytest.mark.parametrize("name", ["int4", "llama7b", "gqa70b", "opt13b"])
def test_full_size_step_sampled_against_oracle(env, name):
    B, torch, oracle, DecodeStep = env
    w = wl.CONFIGS[name]
    print(f"case full-size {name}: B={w.B} H={w.H} Hkv={w.Hkv} bits={w.bits} G={w.G}", flush=True)
    st = DecodeStep(w)
    st.populate()                      # context only; the step's own tokens are written by step()
    st.out.fill_(float("nan"))
    st.step()
    torch.cuda.synchronize()
    out = st.out.cpu().numpy().astype(np.float64)
    assert out.shape == (w.B, w.H, w.D) and np.isfinite(out).all()

    qper = w.H // w.Hkv
    rng = np.random.default_rng(w.seed + 77)
    cache = st.caches[0]
    worst = 0.0
    for i, hk in _samples(w, st.lens, 4, rng):
        L = int(st.lens[i])
        k, v = wl.request_kv(w, st.pool_host, st.offs, i, 0, L, st.gain)
        nblk = (L + w.P - 1) // w.P
        mini = oracle.Cache.empty(nblk, w.P, 1, w.D, w.bits, w.G)
        oracle.kv_quant_write(mini, k[:, hk:hk + 1], v[:, hk:hk + 1], np.arange(L, dtype=np.int64))
        pages = torch.from_numpy(st.pg.block_tables[i, :nblk].astype(np.int64)).cuda()
        valid = (np.arange(nblk * w.P) < L).reshape(nblk, w.P)
        for name_, arr in (("k_codes", mini.k_codes), ("v_codes", mini.v_codes),
                           ("k_meta", mini.k_meta), ("v_meta", mini.v_meta)):
            dev = getattr(cache, name_)[pages, hk].cpu().numpy()
            ref = arr[:, 0]
            if name_.endswith("meta"):
                dev, ref = dev.view(np.uint16), ref.view(np.uint16)
            assert np.array_equal(dev[valid], ref[valid]), f"{name_} of request {i} head {hk} differ"
        bt = np.arange(nblk, dtype=np.int32)[None]
        want = oracle.paged_decode_attn(mini, st.q_host[i:i + 1, hk * qper:(hk + 1) * qper], bt,
                                        np.array([L], np.int32), st.scale)[0]
        err = np.abs(out[i, hk * qper:(hk + 1) * qper] - want).max()
        worst = max(worst, err)
        assert err <= ATTN_TOL, f"request {i} (L={L}) kv head {hk}: max-abs {err}"
    print(f"  worst sampled attention error {worst:.3e}", flush=True)

    # the page dequantized in the step, against the oracle on the oracle's own codes of that page
    i = int(np.argmax(st.lens))
    L = int(st.lens[i])
    n0 = min(L, w.P)
    k, v = wl.request_kv(w, st.pool_host, st.offs, i, 0, n0, st.gain)
    mini = oracle.Cache.empty(1, w.P, w.Hkv, w.D, w.bits, w.G)
    oracle.kv_quant_write(mini, k, v, np.arange(n0, dtype=np.int64))
    ko, vo = oracle.kv_dequant_page(mini, 0)
    assert np.array_equal(st.dq_k.cpu().numpy().view(np.uint16)[:n0], ko.view(np.uint16)[:n0])
    assert np.array_equal(st.dq_v.cpu().numpy().view(np.uint16)[:n0], vo.view(np.uint16)[:n0])


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
    ws = torch.empty(B.alise_paged_prefill_attn_workspace_bytes(cache, w.B, total, w.H), dtype=torch.uint8, device="cuda")
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
