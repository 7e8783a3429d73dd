"""ALISE_DEBUG_VALIDATE=1: the calls check the contents of the device arrays they are given and refuse
what would otherwise be undefined behaviour (a slot outside the cache, a slot used twice, a length beyond
the declared maximum, a block-table entry outside the cache, a chunk longer than its request, a page named
twice in a swap) with ALISE_INVALID_ARGUMENT, before anything is launched.  Valid inputs pass and give the
results they give without the checks."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2410_23537_amd import binding
    return binding, torch


def _refused(B, call):
    with pytest.raises(B.AliseError) as e:
        call()
    assert e.value.status == B.ALISE_INVALID_ARGUMENT


def test_device_contents_are_checked_on_request(env, monkeypatch):
    B, torch = env
    Hkv, H, D, P, num_pages = 2, 2, 128, 16, 12
    cache = B.KVCache.allocate(num_pages, P, Hkv, D, 8, 64, fill=0)
    rng = np.random.default_rng(5)
    T = 40
    k = torch.from_numpy(rng.standard_normal((T, Hkv, D)).astype(np.float16)).cuda()
    v = torch.from_numpy(rng.standard_normal((T, Hkv, D)).astype(np.float16)).cuda()
    good_slots = np.concatenate([np.arange(20), 5 * P + np.arange(20)]).astype(np.int64)     # request 0: pages 0-1, request 1: pages 5-6
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    bt = np.array([[0, 1, 0], [5, 6, 0]], np.int32)
    lens = np.array([20, 20], np.int32)
    q = torch.from_numpy(rng.standard_normal((2, H, D)).astype(np.float16)).cuda()
    scale = 1.0 / np.sqrt(D)
    ws = torch.empty(B.alise_paged_decode_attn_workspace_bytes(cache, 2, H, 48), dtype=torch.uint8, device="cuda")

    # the unchecked run is the reference
    B.alise_kv_quant_write(cache, k, v, dev(good_slots))
    ref = torch.empty_like(q)
    B.alise_paged_decode_attn(cache, q, ref, dev(bt), dev(lens), 48, scale, ws)
    torch.cuda.synchronize()

    monkeypatch.setenv("ALISE_DEBUG_VALIDATE", "1")
    # ---- write
    B.alise_kv_quant_write(cache, k, v, dev(good_slots))                    # valid: passes
    skipped = good_slots.copy(); skipped[3] = -1; skipped[7] = -9           # negative slots are skipped tokens, any number of them
    B.alise_kv_quant_write(cache, k, v, dev(skipped))
    bad = good_slots.copy(); bad[11] = num_pages * P                        # first slot past the cache
    _refused(B, lambda: B.alise_kv_quant_write(cache, k, v, dev(bad)))
    bad = good_slots.copy(); bad[30] = bad[2]                               # two tokens into one slot
    _refused(B, lambda: B.alise_kv_quant_write(cache, k, v, dev(bad)))

    # ---- decode attention
    out = torch.full(q.shape, float("nan"), dtype=torch.float16, device="cuda")
    B.alise_paged_decode_attn(cache, q, out, dev(bt), dev(lens), 48, scale, ws)
    torch.cuda.synchronize()
    assert torch.equal(out, ref)
    _refused(B, lambda: B.alise_paged_decode_attn(cache, q, out, dev(bt), dev(np.array([20, 49], np.int32)), 48, scale, ws))   # beyond the declared maximum
    _refused(B, lambda: B.alise_paged_decode_attn(cache, q, out, dev(bt), dev(np.array([-1, 20], np.int32)), 48, scale, ws))
    bad_bt = bt.copy(); bad_bt[1, 1] = num_pages
    _refused(B, lambda: B.alise_paged_decode_attn(cache, q, out, dev(bad_bt), dev(lens), 48, scale, ws))
    bad_bt = bt.copy(); bad_bt[0, 0] = -3
    _refused(B, lambda: B.alise_paged_decode_attn(cache, q, out, dev(bad_bt), dev(lens), 48, scale, ws))
    unused = bt.copy(); unused[:, 2] = 10 ** 6                              # entries no length reaches are never looked at
    B.alise_paged_decode_attn(cache, q, out, dev(unused), dev(lens), 48, scale, ws)
    torch.cuda.synchronize()
    assert torch.equal(out, ref)

    # ---- prefill attention
    qp = torch.from_numpy(rng.standard_normal((12, H, D)).astype(np.float16)).cuda()
    op = torch.empty_like(qp)
    wsp = torch.empty(B.alise_paged_prefill_attn_workspace_bytes(cache, 2, 12, H), dtype=torch.uint8, device="cuda")
    pre = lambda qs, l=lens, t=bt: B.alise_paged_prefill_attn(cache, qp, op, dev(np.array(qs, np.int32)), dev(t), dev(l), 48, scale, wsp)
    pre([0, 5, 12])
    _refused(B, lambda: pre([0, 7, 5]))                                     # boundaries go down
    _refused(B, lambda: pre([0, 5, 13]))                                    # more query tokens than the call brings
    _refused(B, lambda: pre([0, 5, 12], l=np.array([4, 20], np.int32)))     # a chunk longer than its request
    bad_bt = bt.copy(); bad_bt[0, 1] = num_pages + 7
    _refused(B, lambda: pre([0, 5, 12], t=bad_bt))

    # ---- swap
    nbytes = B.alise_kv_swap_bytes(cache, 20)
    buf = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    B.alise_kv_swap_out(cache, dev(np.array([0, 1], np.int32)), 20, buf)
    B.alise_kv_swap_in(cache, dev(np.array([8, 9], np.int32)), 20, buf)
    _refused(B, lambda: B.alise_kv_swap_out(cache, dev(np.array([0, num_pages], np.int32)), 20, buf))
    _refused(B, lambda: B.alise_kv_swap_in(cache, dev(np.array([8, 8], np.int32)), 20, buf))
    torch.cuda.synchronize()
