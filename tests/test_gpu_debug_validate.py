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


@pytest.fixture
def validating(env, monkeypatch):
    """Switches the checks on for one test (the library reads its environment when asked to) and off again."""
    B, _ = env

    def on():
        monkeypatch.setenv("ALISE_DEBUG_VALIDATE", "1")
        B.alise_reload_environment()
    yield on
    monkeypatch.delenv("ALISE_DEBUG_VALIDATE", raising=False)
    B.alise_reload_environment()


def test_device_contents_are_checked_on_request(env, validating):
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

    validating()
    # ---- first show that the checks are on, with inputs that would be harmless if they were launched: a length
    # beyond the declared maximum (the kernels clamp it) and one slot used twice (the second write wins).  If these
    # are not refused the test ends here, before any out-of-range index is handed to a kernel.
    canary = torch.full(q.shape, float("nan"), dtype=torch.float16, device="cuda")
    _refused(B, lambda: B.alise_paged_decode_attn(cache, q, canary, dev(bt), dev(np.array([20, 49], np.int32)), 48, scale, ws))
    twice = good_slots.copy(); twice[30] = twice[2]
    _refused(B, lambda: B.alise_kv_quant_write(cache, k, v, dev(twice)))
    torch.cuda.synchronize()
    assert bool(torch.isnan(canary).all())                                 # nothing was launched
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
    wsp = torch.empty(B.alise_paged_prefill_attn_workspace_bytes(cache, 2, 12, H, 48), dtype=torch.uint8, device="cuda")
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


def test_lengths_beyond_the_cache_capacity(env, validating):
    """The attention workspace is sized by what the cache can hold.  Ten requests that share all 130 pages of a
    cache (20 800 tokens against a capacity of 2 080) would need more split buffers than that: the call must
    not overrun anything -- it writes nothing at all -- and with the checks on it is refused.  Two requests that
    share the pages stay within the bound and are attended to as usual."""
    B, torch = env
    Hkv, H, D, P, num_pages = 2, 2, 128, 16, 130
    cache = B.KVCache.allocate(num_pages, P, Hkv, D, 8, 128, fill=0)
    rng = np.random.default_rng(11)
    T = num_pages * P
    k = torch.from_numpy(rng.standard_normal((T, Hkv, D)).astype(np.float16)).cuda()
    v = torch.from_numpy(rng.standard_normal((T, Hkv, D)).astype(np.float16)).cuda()
    B.alise_kv_quant_write(cache, k, v, torch.arange(T, dtype=torch.int64, device="cuda"))
    scale = 1.0 / np.sqrt(D)

    def run(n_req):
        q = torch.from_numpy(np.repeat(rng.standard_normal((1, H, D)).astype(np.float16), n_req, axis=0)).cuda()
        out = torch.full(q.shape, float("nan"), dtype=torch.float16, device="cuda")
        bt = torch.arange(num_pages, dtype=torch.int32, device="cuda").repeat(n_req, 1).contiguous()
        lens = torch.full((n_req,), T, dtype=torch.int32, device="cuda")
        ws = torch.full((B.alise_paged_decode_attn_workspace_bytes(cache, n_req, H, T),), 0xA5, dtype=torch.uint8, device="cuda")
        guard = torch.full((1 << 20,), 0x5A, dtype=torch.uint8, device="cuda")     # whatever follows the workspace in memory
        B.alise_paged_decode_attn(cache, q, out, bt, lens, T, scale, ws)
        torch.cuda.synchronize()
        assert bool((guard == 0x5A).all())
        return out

    print("case capacity two requests share the pages", flush=True)
    out2 = run(2)
    assert bool(torch.isfinite(out2).all()) and torch.equal(out2[0], out2[1])
    print("case capacity ten requests share the pages", flush=True)
    out10 = run(10)
    assert bool(torch.isnan(out10).all())           # no work was planned, nothing was written
    validating()
    with pytest.raises(B.AliseError) as e:
        run(10)
    assert e.value.status == B.ALISE_INVALID_ARGUMENT


def test_v_scales_beyond_the_matrix_core_range(env, validating):
    """The matrix-core paths (grouped-query decode, chunked prefill) carry weight x V scale as a pair of fp16 numbers, which
    holds for V scales below 256; the vector path has no such limit.  With the checks on, a call that would run on the
    matrix cores over a request whose cached V reaches such a scale is refused; the same cache read by the vector kernel,
    and a request that does not reach the wide group, pass."""
    B, torch = env
    Hkv, D, P, num_pages = 2, 128, 16, 8
    cache = B.KVCache.allocate(num_pages, P, Hkv, D, 8, 64, fill=0)
    rng = np.random.default_rng(7)
    T = 40
    k = rng.standard_normal((T, Hkv, D)).astype(np.float16)
    v = rng.standard_normal((T, Hkv, D)).astype(np.float16)
    v[30, 1, 70], v[30, 1, 71] = 65504.0, -65504.0          # one group of one head of token 30: scale 131008 / 255 = 514
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    B.alise_kv_quant_write(cache, dev(k), dev(v), dev(np.arange(T, dtype=np.int64)))
    bt = dev(np.array([[0, 1, 2]], np.int32))
    scale = 1.0 / np.sqrt(D)
    print("case V scale limit", flush=True)

    def decode(H, L):
        q = dev(rng.standard_normal((1, H, D)).astype(np.float16))
        o = torch.empty_like(q)
        ws = torch.empty(B.alise_paged_decode_attn_workspace_bytes(cache, 1, H, 48), dtype=torch.uint8, device="cuda")
        B.alise_paged_decode_attn(cache, q, o, bt, dev(np.array([L], np.int32)), 48, scale, ws)
        torch.cuda.synchronize()
        return o

    def prefill(H, L, n):
        q = dev(rng.standard_normal((n, H, D)).astype(np.float16))
        o = torch.empty_like(q)
        ws = torch.empty(B.alise_paged_prefill_attn_workspace_bytes(cache, 1, n, H, 48), dtype=torch.uint8, device="cuda")
        B.alise_paged_prefill_attn(cache, q, o, dev(np.array([0, n], np.int32)), bt, dev(np.array([L], np.int32)), 48, scale, ws)
        torch.cuda.synchronize()
        return o

    validating()
    _refused(B, lambda: decode(8, 40))                      # four query heads per KV head: matrix cores, token 30 in reach
    _refused(B, lambda: prefill(2, 40, 8))                  # chunked prefill runs on the matrix cores for this layout
    assert bool(torch.isfinite(decode(8, 30)).all())        # tokens 0 .. 29 only
    assert bool(torch.isfinite(prefill(2, 30, 8)).all())
    assert bool(torch.isfinite(decode(2, 40)).all())        # one query head per KV head: the vector kernel, no limit
