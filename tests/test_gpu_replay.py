"""End-to-end parity of a scheduled run on the GPU (ALISE Sec. 3.1 "Preemptive Scheduling",
Sec. 3.2 "Dynamic Swapping" with Alg. 2, over the quantized paged cache of Sec. 3.2 and the
attention of Eq. 1-2): the C++ scheduler plans, the library's kernels run every iteration
(quantize-and-write, chunked prefill, decode attention, offload, upload), and a second run of the
same jobs on the CPU -- the oracle scheduler planning, the oracle's cache and attention
executing, one private cache per job -- must agree: decisions bit for bit, every offloaded
request byte for byte, every attention row within 2e-3."""
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


@pytest.mark.parametrize("shape_name", list(SHAPES))
@pytest.mark.parametrize("overlap", [True, False], ids=["side_stream", "one_stream"])
def test_scheduled_run_against_the_oracle(env, shape_name, overlap):
    B, replay, torch, oracle, so = env
    sh = SHAPES[shape_name]
    w = wl.Workload(name=shape_name, B=1, length_law="fixed:1", seed=31, max_len=512, **sh)
    n_jobs = 14
    arrival, s, n_true, n_pred = (a.tolist() for a in wl.job_trace(n_jobs, 11, mean_gap=150.0, max_prompt=90, max_output=24))
    cfg = dict(num_queues=3, limit0=1500, age_threshold=6000, max_batch=3, gpu_job_limit=4, t0=2, alpha=1, beta=20)
    print(f"case replay {shape_name} overlap={overlap}: prompts {s} outputs {n_true} predicted {n_pred}", flush=True)

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
    rp = replay.Replay(w, B.Scheduler(**cfg), num_pages=2 * (cfg["gpu_job_limit"] + 1) * pages_per_job, max_context=max_ctx,
                       kv_source=source, overlap_swaps=overlap)
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
    assert len(rp.free) + len(rp.pending_free) == rp.cache.num_pages          # every page came back
