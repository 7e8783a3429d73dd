"""End-to-end parity of a scheduled run on the GPU (ALISE Sec. 3.1 "Preemptive Scheduling",
Sec. 3.2 "Dynamic Swapping" with Alg. 2, over the quantized paged cache of Sec. 3.2 and the
attention of Eq. 1-2): the C++ scheduler plans, the library's kernels run every iteration
(quantize-and-write, chunked prefill, decode attention, offload, upload), and a second run of the
same jobs on the CPU -- the oracle scheduler planning, the oracle's cache and attention
executing, one private cache per job -- must agree: decisions bit for bit, every offloaded
request byte for byte, every attention row within 2e-3.  The loop around the calls is either the
Python one (replay.py) or the C++ one (alise_replay.h); both are held to the same comparison."""
import numpy as np
import pytest

from paper_2410_23537_amd import workloads as wl

pytestmark = pytest.mark.gpu

ATTN_TOL = 2e-3


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2410_23537_amd import binding, replay
    import oracle
    from oracle import sched_oracle
    oracle.build()
    return binding, replay, torch, oracle, sched_oracle


def _mark_tokens(oracle, oc, L):
    """A cache of the same geometry whose bytes are 0xff exactly where the first L tokens of pages 0, 1, ... live."""
    m = oracle.Cache.empty(oc.num_pages, oc.page_size, oc.num_kv_heads, oc.head_dim, oc.bits, oc.group_size)
    t = np.arange(L)
    for arr in (m.k_codes, m.v_codes):
        arr[t // oc.page_size, :, t % oc.page_size] = 0xFF
    for arr in (m.k_meta, m.v_meta):
        arr.view(np.uint16)[t // oc.page_size, :, t % oc.page_size] = 0xFFFF
    return m


SHAPES = {
    "mha_g64": dict(H=4, Hkv=4, D=128, P=16, bits=8, G=64),
    "gqa4_g128_p32": dict(H=8, Hkv=2, D=128, P=32, bits=8, G=128),
    "int4_g32": dict(H=4, Hkv=4, D=128, P=16, bits=4, G=32),
}


class _NativeLoop:
    """The C++ loop of alise_replay.h behind the interface of replay.Replay, for the comparison below."""

    def __init__(self, B, torch, w, cfg, num_pages, max_ctx, data, s, overlap):
        import ctypes
        self._ctypes, self._torch = ctypes, torch
        n = len(data)
        self.base = np.concatenate([[0], np.cumsum([data[i][0].shape[0] for i in range(n)])]).astype(np.int64)
        pad = [np.zeros((max_ctx,) + data[0][c].shape[1:], np.float16) for c in range(3)]      # rows past the last job's tokens
        k, v, q = (torch.from_numpy(np.concatenate([data[i][c] for i in range(n)] + [pad[c]])).cuda() for c in range(3))
        self.cache = B.KVCache.allocate(num_pages, w.P, w.Hkv, w.D, w.bits, w.G, fill=0)
        self.loop = B.NativeReplay(self.cache, w.H, cfg, max_ctx, cfg["max_batch"] * max(s), k, v, q, 1.0 / np.sqrt(w.D), overlap)

    def add_job(self, id, arrival, prompt_len, predicted_len):
        self.loop.add_job(id, arrival, prompt_len, predicted_len, int(self.base[id]))

    def iterate(self):
        d = self.loop.iterate()
        self.loop.synchronize()
        n_pre = d["n_prefill_tokens"]
        pre = [id for id, ph in zip(d["batch"], d["phase"]) if ph == 0]
        dec = [id for id, ph in zip(d["batch"], d["phase"]) if ph == 1]
        # rows: the phase-0 jobs back to back in batch order, then one row per phase-1 job
        assert [d["out_row"][d["batch"].index(id)] for id in dec] == list(range(n_pre, n_pre + len(dec)))
        d.update(prefill_ids=pre, decode_ids=dec, prefill_out=d["out"][:n_pre].clone(),
                 decode_out=d["out"][n_pre:n_pre + len(dec)].clone())
        off = {}
        for id, (addr, n) in d["offloaded"].items():
            raw = (self._ctypes.c_ubyte * n).from_address(addr)
            off[id] = (self._torch.from_numpy(np.frombuffer(raw, np.uint8).copy()), n)
        d["offloaded"] = off
        return d

    def commit(self, elapsed, finished):
        self.loop.commit(elapsed, finished)

    def pages_back(self):
        return self.loop.stats()["free_pages"] == self.cache.num_pages


@pytest.mark.parametrize("shape_name", list(SHAPES))
@pytest.mark.parametrize("overlap", [True, False], ids=["side_stream", "one_stream"])
@pytest.mark.parametrize("loop", ["python_loop", "native_loop"])
def test_scheduled_run_against_the_oracle(env, shape_name, overlap, loop):
    B, replay, torch, oracle, so = env
    sh = SHAPES[shape_name]
    w = wl.Workload(name=shape_name, B=1, length_law="fixed:1", seed=31, max_len=512, **sh)
    n_jobs = 14
    arrival, s, n_true, n_pred = (a.tolist() for a in wl.job_trace(n_jobs, 11, mean_gap=150.0, max_prompt=90, max_output=24))
    cfg = dict(num_queues=3, limit0=1500, age_threshold=6000, max_batch=3, gpu_job_limit=4, t0=2, alpha=1, beta=20)
    print(f"case replay {shape_name} {loop} overlap={overlap}: prompts {s} outputs {n_true} predicted {n_pred}", flush=True)

    # every job's K, V, Q for all of its tokens, seeded
    rng = np.random.default_rng(5)
    data = {}
    for i in range(n_jobs):
        T = s[i] + n_true[i]
        data[i] = ((rng.standard_normal((T, w.Hkv, w.D)) * 1.5 + rng.uniform(-2, 2)).astype(np.float16),
                   rng.standard_normal((T, w.Hkv, w.D)).astype(np.float16),
                   rng.standard_normal((T, w.H, w.D)).astype(np.float16))

    def source(spans):
        return tuple(torch.from_numpy(np.concatenate([data[id][c][t0:t1] for id, t0, t1 in spans])).cuda() for c in range(3))

    max_ctx = max(s[i] + n_true[i] for i in range(n_jobs)) + 1
    pages_per_job = (max_ctx + w.P - 1) // w.P
    num_pages = 2 * (cfg["gpu_job_limit"] + 1) * pages_per_job
    if loop == "native_loop":
        rp = _NativeLoop(B, torch, w, cfg, num_pages, max_ctx, data, s, overlap)
    else:
        rp = replay.Replay(w, B.Scheduler(**cfg), num_pages=num_pages, max_context=max_ctx, kv_source=source, overlap_swaps=overlap)
    osched = so.Scheduler(so.Config(**cfg))
    ocache = {}          # job -> (oracle cache of its own, tokens in it)
    scale = 1.0 / np.sqrt(w.D)

    nxt = sorted(range(n_jobs), key=lambda i: (arrival[i], i))
    k, now, iters, worst = 0, 0, 0, 0.0
    gen = [0] * n_jobs
    n_off = n_up = 0
    while True:
        while k < n_jobs and arrival[nxt[k]] <= now:
            i = nxt[k]
            rp.add_job(i, arrival[i], s[i], n_pred[i])
            osched.add_job(i, arrival[i], s[i], n_pred[i])
            k += 1
        if not osched.jobs:
            if k == n_jobs:
                break
            now = arrival[nxt[k]]
            continue
        want = osched.step()
        got = rp.iterate()
        torch.cuda.synchronize()
        assert got["batch"] == want.batch and got["phase"] == want.phase, f"iteration {iters}"
        assert got["upload"] == want.upload and got["offload"] == want.offload, f"iteration {iters}"
        # ---- what left the GPU, byte for byte (the oracle's cache of the job holds the same tokens)
        for id in want.offload:
            oc, L = ocache[id]
            buf, n = got["offloaded"][id]
            bt = np.arange(oc.num_pages, dtype=np.int32)
            assert n == oracle.kv_swap_bytes(oc, L)
            # whole pages move; the slots of the last page past the job's end hold whatever the page's last owner left
            live = oracle.kv_swap_out(_mark_tokens(oracle, oc, L), bt, L) != 0
            assert live.sum() == L * w.Hkv * 2 * (w.D * w.bits // 8 + 4 * (w.D // w.G))
            assert np.array_equal(buf[:n].numpy()[live], oracle.kv_swap_out(oc, bt, L)[live]), f"offloaded form of job {id}, iteration {iters}"
        n_off += len(want.offload)
        n_up += len(want.upload)
        # ---- the batch on the CPU
        row_p = 0
        for pos, (id, ph) in enumerate(zip(want.batch, want.phase)):
            kk, vv, qq = data[id]
            if ph == 0:
                oc = oracle.Cache.empty((max_ctx + w.P - 1) // w.P, w.P, w.Hkv, w.D, w.bits, w.G)
                L = s[id]
                oracle.kv_quant_write(oc, kk[:L], vv[:L], np.arange(L, dtype=np.int64))
                bt = np.arange(oc.num_pages, dtype=np.int32)[None]
                ref = oracle.paged_prefill_attn(oc, qq[:L], np.array([0, L], np.int32), bt, np.array([L], np.int32), scale)
                dev = got["prefill_out"][row_p:row_p + L].cpu().numpy().astype(np.float64)
                row_p += L
            else:
                oc, L0 = ocache[id]
                L = L0 + 1
                oracle.kv_quant_write(oc, kk[L0:L], vv[L0:L], np.arange(L0, L, dtype=np.int64))
                bt = np.arange(oc.num_pages, dtype=np.int32)[None]
                ref = oracle.paged_decode_attn(oc, qq[L0:L], bt, np.array([L], np.int32), scale)
                r = got["decode_ids"].index(id)
                dev = got["decode_out"][r:r + 1].cpu().numpy().astype(np.float64)
            ocache[id] = (oc, L)
            err = float(np.abs(dev - ref).max())
            worst = max(worst, err)
            assert np.isfinite(dev).all() and err <= ATTN_TOL, f"job {id} iteration {iters}: {err:.3e}"
        elapsed = osched.model_time(want)
        assert got["model_time"] == elapsed
        fin = []
        for id in want.batch:
            gen[id] += 1
            if gen[id] >= n_true[id]:
                fin.append(id)
        osched.commit(want, elapsed, fin)
        rp.commit(elapsed, fin)
        for id in fin:
            del ocache[id]
        now += elapsed
        iters += 1
        assert iters < 5000
    print(f"  {iters} iterations, {n_off} offloads, {n_up} uploads, worst attention error {worst:.2e}", flush=True)
    assert gen == n_true and n_off > 0 and n_up > 0
    # every page came back
    assert rp.pages_back() if loop == "native_loop" else len(rp.free) + len(rp.pending_free) == rp.cache.num_pages


@pytest.mark.parametrize("shape_name", ["gqa4_g128_p32", "int4_g32"])
def test_native_loop_without_host_waits(env, shape_name):
    """The C++ loop never waits for the GPU in the steady state: metadata goes through a ring of pinned staging buffers, host
    buffers of uploads are recycled behind events, freed pages are reused behind events.  A run that is left to run free
    (hundreds of iterations enqueued ahead of the GPU) must give, bit for bit, the outputs and the final cache of a run that
    waits for the GPU after every iteration -- which the test above checks against the oracle."""
    B, _, torch, _, _ = env
    sh = SHAPES[shape_name]
    w = wl.Workload(name=shape_name, B=1, length_law="fixed:1", seed=31, max_len=512, **sh)
    n_jobs = 48
    arrival, s, n_true, n_pred = (a.tolist() for a in wl.job_trace(n_jobs, 23, mean_gap=60.0, max_prompt=120, max_output=40))
    cfg = dict(num_queues=3, limit0=1500, age_threshold=6000, max_batch=4, gpu_job_limit=5, t0=2, alpha=1, beta=20)
    max_ctx = max(a + b for a, b in zip(s, n_true)) + 1
    num_pages = 2 * (cfg["gpu_job_limit"] + cfg["max_batch"] + 1) * ((max_ctx + w.P - 1) // w.P)
    gen = torch.Generator(device="cuda").manual_seed(9)
    rows = 4096
    k = torch.randn((rows + max_ctx, w.Hkv, w.D), dtype=torch.float16, device="cuda", generator=gen) * 1.5
    v = torch.randn((rows + max_ctx, w.Hkv, w.D), dtype=torch.float16, device="cuda", generator=gen)
    q = torch.randn((rows + max_ctx, w.H, w.D), dtype=torch.float16, device="cuda", generator=gen)

    def run(wait):
        cache = B.KVCache.allocate(num_pages, w.P, w.Hkv, w.D, w.bits, w.G, fill=0)
        rp = B.NativeReplay(cache, w.H, cfg, max_ctx, cfg["max_batch"] * max(s), k, v, q, 1.0 / np.sqrt(w.D), True)
        order = sorted(range(n_jobs), key=lambda i: (arrival[i], i))
        nxt, now, produced, log, decisions = 0, 0, [0] * n_jobs, [], []
        while True:
            while nxt < n_jobs and arrival[order[nxt]] <= now:
                i = order[nxt]
                rp.add_job(i, arrival[i], s[i], n_pred[i], (i * 613) % rows)
                nxt += 1
            if rp.num_jobs() == 0:
                if nxt == n_jobs:
                    break
                now = arrival[order[nxt]]
                continue
            d = rp.iterate()
            if wait:
                rp.synchronize()
            n = d["n_prefill_tokens"] + d["n_decode_tokens"]
            log.append(d["out"][:n].clone())                # on the stream the loop runs on: behind this iteration, before the next
            decisions.append((d["batch"], d["phase"], d["upload"], d["offload"], d["out_row"]))
            fin = []
            for id in d["batch"]:
                produced[id] += 1
                if produced[id] >= n_true[id]:
                    fin.append(id)
            rp.commit(d["model_time"], fin)
            now += d["model_time"]
            assert len(log) < 20000
        rp.synchronize()
        torch.cuda.synchronize()
        st = rp.stats()
        assert st["free_pages"] == num_pages and st["live_jobs"] == 0
        rp.close()
        return decisions, torch.cat(log).cpu(), [t.cpu() for t in (cache.k_codes, cache.v_codes, cache.k_meta, cache.v_meta)], st

    print(f"case native loop free-running vs waiting, {shape_name}", flush=True)
    dec_w, out_w, cache_w, st_w = run(True)
    dec_f, out_f, cache_f, st_f = run(False)
    print(f"  {st_f['iterations']} iterations, {st_f['offloads']} offloads, {st_f['uploads']} uploads", flush=True)
    assert st_f["offloads"] >= 10 and st_f["uploads"] >= 10 and st_f["iterations"] > 100
    assert dec_w == dec_f and st_w == st_f
    assert torch.equal(out_w, out_f)
    for a, b in zip(cache_w, cache_f):
        assert torch.equal(a, b)


def test_native_loop_error_paths(env):
    """alise_replay.h: lists that are too short are reported before the scheduler decides (the call can be repeated);
    a cache with too few free pages, or more new tokens than max_iter_tokens, is reported after it has decided, nothing
    is enqueued and the object refuses further work."""
    import ctypes
    B, _, torch, _, _ = env
    lib = B.raw()
    H, Hkv, D, P = 4, 4, 128, 16
    cfg = dict(num_queues=3, limit0=1500, age_threshold=6000, max_batch=2, gpu_job_limit=3, t0=2, alpha=1, beta=20)
    rows = 512
    k = torch.zeros((rows, Hkv, D), dtype=torch.float16, device="cuda")
    q = torch.zeros((rows, H, D), dtype=torch.float16, device="cuda")

    def loop(num_pages, max_iter_tokens=128):
        cache = B.KVCache.allocate(num_pages, P, Hkv, D, 8, 64, fill=0)
        return B.NativeReplay(cache, H, cfg, 100, max_iter_tokens, k, k, q, 0.088)

    print("case native loop error paths", flush=True)
    # --- add_job
    rp = loop(16)
    for bad in [dict(prompt_len=0), dict(prompt_len=100), dict(token_row=-1), dict(prompt_len=129, )]:
        a = dict(id=1, arrival=0, prompt_len=20, predicted_len=5, token_row=0)
        a.update(bad)
        st = lib.alise_replay_add_job(rp._h, a["id"], a["arrival"], a["prompt_len"], a["predicted_len"], a["token_row"])
        assert st == B.ALISE_INVALID_ARGUMENT, bad
    rp.add_job(1, 0, 20, 5, 0)
    assert lib.alise_replay_add_job(rp._h, 1, 0, 20, 5, 0) == B.ALISE_INVALID_ARGUMENT          # the id is live
    # --- lists too short: nothing has changed, the same call with room succeeds
    it = rp._it
    it.batch_cap = 0
    assert lib.alise_replay_iterate(rp._h, k.data_ptr(), k.data_ptr(), q.data_ptr(), rp.out.data_ptr(), ctypes.byref(it)) \
        == B.ALISE_WORKSPACE_TOO_SMALL
    it.batch_cap = cfg["max_batch"]
    d = rp.iterate()
    assert d["batch"] == [1] and d["phase"] == [0] and d["n_prefill_tokens"] == 20
    # commit with an id that was not in the batch: the scheduler's error comes through, nothing changes
    bad_id = (ctypes.c_int64 * 1)(7)
    assert lib.alise_replay_commit(rp._h, 1, bad_id, 1) == B.ALISE_INVALID_ARGUMENT
    rp.commit(d["model_time"], [1])
    rp.synchronize()
    assert rp.stats()["free_pages"] == 16 and rp.num_jobs() == 0
    assert rp.iterate()["batch"] == []              # no live job: nothing to do, no error
    rp.close()
    # --- too few pages for the batch: reported, and the object is finished
    rp = loop(2)
    rp.add_job(1, 0, 40, 5, 0)                      # needs three pages
    with pytest.raises(RuntimeError, match="ALISE_WORKSPACE_TOO_SMALL"):
        rp.iterate()
    with pytest.raises(RuntimeError, match="ALISE_INVALID_ARGUMENT"):
        rp.iterate()
    with pytest.raises(RuntimeError, match="ALISE_INVALID_ARGUMENT"):
        rp.commit(1, [])
    rp.close()
    # --- more new tokens than max_iter_tokens
    rp = loop(16, max_iter_tokens=50)
    rp.add_job(1, 0, 30, 5, 0)
    rp.add_job(2, 0, 30, 5, 100)
    with pytest.raises(RuntimeError, match="ALISE_WORKSPACE_TOO_SMALL"):
        rp.iterate()
    rp.close()
    torch.cuda.synchronize()


@pytest.mark.parametrize("shape_name", ["llama7b", "gqa70b", "int4"])
def test_both_loops_agree_at_the_benchmark_shapes(env, shape_name):
    """The two loops call the same entry points with the same arguments, so on the layouts bench.py times (32 or 64 query
    heads, matrix-core and vector kernels) every decision and every output row of a scheduled run must be the same bit for
    bit, whichever loop drives it, the C++ one running ahead of the GPU."""
    B, replay, torch, _, _ = env
    w = wl.CONFIGS[shape_name]
    n_jobs = 20
    arrival, s, n_true, n_pred = (a.tolist() for a in wl.job_trace(n_jobs, 5, mean_gap=80.0, max_prompt=300, max_output=12))
    cfg = dict(num_queues=3, limit0=3000, age_threshold=20000, max_batch=6, gpu_job_limit=8, t0=2, alpha=1, beta=20)
    max_ctx = max(a + b for a, b in zip(s, n_true)) + 1
    num_pages = 2 * (cfg["gpu_job_limit"] + cfg["max_batch"] + 1) * ((max_ctx + w.P - 1) // w.P)
    gen = torch.Generator(device="cuda").manual_seed(13)
    rows = 2048
    k = torch.randn((rows + max_ctx, w.Hkv, w.D), dtype=torch.float16, device="cuda", generator=gen) * 1.5
    v = torch.randn((rows + max_ctx, w.Hkv, w.D), dtype=torch.float16, device="cuda", generator=gen)
    q = torch.randn((rows + max_ctx, w.H, w.D), dtype=torch.float16, device="cuda", generator=gen)
    base = lambda id: (id * 211) % rows

    def source(spans):
        idx = torch.from_numpy(np.concatenate([np.arange(base(id) + a, base(id) + b) for id, a, b in spans])).cuda()
        return k.index_select(0, idx), v.index_select(0, idx), q.index_select(0, idx)

    def drive(add_job, num_jobs, iterate, commit, rows_of):
        order = sorted(range(n_jobs), key=lambda i: (arrival[i], i))
        nxt, now, produced, log, decisions = 0, 0, [0] * n_jobs, [], []
        while True:
            while nxt < n_jobs and arrival[order[nxt]] <= now:
                add_job(order[nxt])
                nxt += 1
            if num_jobs() == 0:
                if nxt == n_jobs:
                    return decisions, torch.cat(log).cpu()
                now = arrival[order[nxt]]
                continue
            d = iterate()
            log.append(rows_of(d))
            decisions.append((list(d["batch"]), list(d["phase"]), list(d["upload"]), list(d["offload"])))
            fin = []
            for id in d["batch"]:
                produced[id] += 1
                if produced[id] >= n_true[id]:
                    fin.append(id)
            commit(d["model_time"], fin)
            now += d["model_time"]

    print(f"case both loops, {shape_name}", flush=True)
    cache = B.KVCache.allocate(num_pages, w.P, w.Hkv, w.D, w.bits, w.G, fill=0)
    nat = B.NativeReplay(cache, w.H, cfg, max_ctx, cfg["max_batch"] * max(s), k, v, q, 1.0 / np.sqrt(w.D))
    dec_n, out_n = drive(lambda i: nat.add_job(i, arrival[i], s[i], n_pred[i], base(i)), nat.num_jobs, nat.iterate, nat.commit,
                         lambda d: d["out"][:d["n_prefill_tokens"] + d["n_decode_tokens"]].clone())
    nat.synchronize()
    st = nat.stats()
    nat.close()
    py = replay.Replay(w, B.Scheduler(**cfg), num_pages=num_pages, max_context=max_ctx, kv_source=source)

    def rows_py(d):
        parts = [t for t in (d["prefill_out"], d["decode_out"]) if t is not None]
        return torch.cat(parts) if parts else torch.empty((0, w.H, w.D), dtype=torch.float16, device="cuda")
    dec_p, out_p = drive(lambda i: py.add_job(i, arrival[i], s[i], n_pred[i]), py.sched.num_jobs, py.iterate, py.commit, rows_py)
    torch.cuda.synchronize()
    print(f"  {st['iterations']} iterations, {st['offloads']} offloads, {st['uploads']} uploads, {out_n.shape[0]} output rows", flush=True)
    assert dec_n == dec_p
    assert st["offloads"] > 0 and st["uploads"] > 0
    assert out_n.shape == out_p.shape and torch.equal(out_n, out_p)
