"""Seeded random shapes within the documented limits: bit width, group size, head_dim, page size, head
counts and lengths drawn independently, so that combinations nobody thought of listing get run.  Every
case: write (codes and meta bit-exact), decode attention, and -- where the shape has a prefill kernel --
prefill attention with ragged chunks, all against the oracle."""
import numpy as np
import pytest

from paper_2410_23537_amd import workloads as wl
from tests import harness

pytestmark = pytest.mark.gpu

ATTN_TOL = 2e-3


def _draw(seed):
    rng = np.random.default_rng([4242, seed])
    bits = int(rng.choice([4, 8]))
    D = int(rng.choice([64, 128, 128, 128]))
    G = int(rng.choice([g for g in (16, 32, 64, 128) if g <= D and g % (128 // bits) == 0]))
    P = int(rng.choice([8, 16, 16, 32, 64, 128, 256]))
    Hkv = int(rng.choice([1, 2, 3, 5]))
    qper = int(rng.choice([1, 1, 2, 3, 4, 8, 16, 20]))
    B = int(rng.integers(1, 7))
    top = int(rng.choice([60, 300, 1200, 3000]))
    lens = rng.integers(0, top + 1, B).astype(np.int32)
    lens[rng.integers(0, B)] = top
    return dict(bits=bits, D=D, G=G, P=P, Hkv=Hkv, H=Hkv * qper), lens


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2410_23537_amd import binding
    import oracle
    oracle.build()
    return binding, torch, oracle


@pytest.mark.parametrize("seed", range(28))
def test_random_shape(env, seed):
    B, torch, oracle = env
    shape, lens = _draw(seed)
    print(f"case random shape seed {seed}: {shape} lens {lens.tolist()}", flush=True)
    w = wl.Workload(f"rnd{seed}", B=len(lens), length_law="fixed:1", seed=9000 + seed, max_len=int(max(1, lens.max())), **shape)
    pg = wl.paging(w, lens)
    pool = wl.value_pool(w, n_min=int(max(1, lens.max())) * w.Hkv * w.D)
    offs, gain = wl.request_offsets(w), wl.k_channel_gain(w)
    orc = harness.fill_oracle_cache(oracle, w, pg, pool, offs, gain)
    dev = harness.fill_device_cache(B, torch, w, pg, pool, offs, gain)
    mask = harness.written_mask(w, pg)
    for name in ("k_codes", "v_codes", "k_meta", "v_meta"):
        d = getattr(dev, name).cpu().numpy()
        o = getattr(orc, name)
        if name.endswith("meta"):
            d, o = d.view(np.uint16), o.view(np.uint16)
        d, o = np.moveaxis(d, 1, 2), np.moveaxis(o, 1, 2)      # [page, off, head, ...]
        assert np.array_equal(d[mask], o[mask]), f"{name}: written slots differ"
        assert np.array_equal(d[~mask], o[~mask]), f"{name}: untouched slots were modified"
    scale = 1.0 / np.sqrt(w.D)
    q = wl.queries(w)
    want = oracle.paged_decode_attn(orc, q, pg.block_tables, pg.lens, scale, num_threads=8)
    got = harness.run_device_attn(B, torch, w, dev, q, pg).astype(np.float64)
    assert np.isfinite(got).all() and not got[lens == 0].any()
    assert np.abs(got - want).max() <= ATTN_TOL

    rng = np.random.default_rng([77, seed])
    chunk = np.minimum(lens, rng.integers(0, 200, len(lens))).astype(np.int64)
    total = int(chunk.sum())
    nbytes = B.alise_paged_prefill_attn_workspace_bytes(dev, len(lens), max(total, 1), w.H, int(max(1, lens.max())))
    assert nbytes > 0                                    # every layout has a prefill path (matrix cores, or the single-query kernels)
    if total == 0:
        return
    q_start = np.concatenate([[0], np.cumsum(chunk)]).astype(np.int32)
    qp_np = rng.standard_normal((total, w.H, w.D)).astype(np.float16)
    wantp = oracle.paged_prefill_attn(orc, qp_np, q_start, pg.block_tables, pg.lens, scale)
    qp = torch.from_numpy(qp_np).cuda()
    op = torch.full(qp.shape, float("nan"), dtype=torch.float16, device="cuda")
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    B.alise_paged_prefill_attn(dev, qp, op, torch.from_numpy(q_start).cuda(), torch.from_numpy(pg.block_tables).cuda(),
                               torch.from_numpy(pg.lens.astype(np.int32)).cuda(), int(max(1, lens.max())), scale, ws)
    torch.cuda.synchronize()
    gotp = op.cpu().numpy().astype(np.float64)
    assert np.isfinite(gotp).all() and np.abs(gotp - wantp).max() <= ATTN_TOL
