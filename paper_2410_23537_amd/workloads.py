"""Seeded synthetic serving workloads for the quantized paged-KV decode path.

This module only *generates inputs* (context lengths, block tables, slot
mappings, fp16 Q/K/V values).  It holds none of the method's arithmetic: no
quantizer, no softmax, no dequantizer.  Both the HIP path and the CPU checker
are fed from here so that they see identical inputs.

The paper evaluates on request traces whose prompt/response lengths follow two
public chat datasets (Sec. 4.1, Workloads); only the *shape* of such traces is
reproduced here -- heavy-tailed synthetic length laws stand in for them, and no
item of either dataset appears anywhere.  The scheduler of the paper (Sec. 3.1)
shows up only as the order of requests in a batch and their context lengths.

Everything is a pure function of (config, seed), uses ``numpy.random.default_rng``
and never touches a GPU.
"""
from __future__ import annotations

from dataclasses import dataclass, replace  # noqa: F401  (replace is re-exported)
from typing import Dict, Tuple

import numpy as np


@dataclass(frozen=True)
class Workload:
    """Shape of one decode step over a paged, quantized KV cache.

    Notation: B requests, H query heads, Hkv KV heads, D head_dim, P page size,
    bits in {4, 8}, G quantization group size (contiguous channels of one
    token's one head vector).
    """
    name: str
    B: int
    H: int
    Hkv: int
    D: int
    P: int
    bits: int
    G: int
    length_law: str          # see context_lens()
    seed: int
    max_len: int
    outlier_frac: float = 0.0   # fraction of K channels scaled by outlier_gain
    outlier_gain: float = 10.0
    prefill_every: int = 0      # every n-th request writes a prefill chunk in the timed step
    prefill_chunk: int = 0

    @property
    def row_code_bytes(self) -> int:
        return self.D * self.bits // 8

    @property
    def groups(self) -> int:
        return self.D // self.G

    @property
    def row_bytes(self) -> int:
        """Compressed bytes of one (token, kv-head): K and V codes plus fp16 scale and zero per group."""
        return 2 * self.row_code_bytes + 2 * self.groups * 4


# The five configurations of the benchmark contract.  Seeds are 1000 + index.
CONFIGS: Dict[str, Workload] = {
    "tiny": Workload("tiny", B=4, H=8, Hkv=8, D=64, P=16, bits=8, G=64,
                     length_law="fixed:17,64,100,255", seed=1001, max_len=255),
    "opt13b": Workload("opt13b", B=64, H=40, Hkv=40, D=128, P=16, bits=8, G=128,
                       length_law="lognormal_priority", seed=1002, max_len=2048),
    "llama7b": Workload("llama7b", B=256, H=32, Hkv=32, D=128, P=16, bits=8, G=64,
                        length_law="bimodal", seed=1003, max_len=4096,
                        prefill_every=8, prefill_chunk=512),
    "gqa70b": Workload("gqa70b", B=128, H=64, Hkv=8, D=128, P=32, bits=8, G=128,
                       length_law="uniform:512,8192", seed=1004, max_len=8192,
                       outlier_frac=0.05),
    "int4": Workload("int4", B=512, H=32, Hkv=32, D=128, P=16, bits=4, G=32,
                     length_law="zipf", seed=1005, max_len=16384),
}


# Variants of the configurations above that the benchmark can also be pointed at (bench.py --workload): not part of
# the contract's five, used to measure kernels that none of the five selects.
CONFIGS["gqa70b_int4"] = replace(CONFIGS["gqa70b"], name="gqa70b_int4", bits=4, G=32)      # the grouped-query kernel on INT4 codes
CONFIGS["gqa70b_int4_g128"] = replace(CONFIGS["gqa70b"], name="gqa70b_int4_g128", bits=4, G=128)


def scaled(w: Workload, B: int, max_len: int, name: str | None = None) -> Workload:
    """Same head geometry and length law, fewer requests and a lower length cap."""
    return replace(w, B=B, max_len=max_len, name=name or f"{w.name}_small")


def context_lens(w: Workload) -> np.ndarray:
    """Context length L_i of every request, *including* the token written in this step.

    Laws: ``fixed:a,b,..``; ``lognormal_priority`` (median 300, sigma 1, clipped to
    [1, max_len], then ordered by a noisy shortest-predicted-first key -- the batch
    order a length-predicting priority scheduler would produce); ``bimodal`` (70 %
    uniform 16..256, 30 % uniform 1024..4096, both clipped to max_len);
    ``uniform:a,b``; ``zipf`` (exponent 1.2, clipped -- not truncated -- to
    [1, max_len], so the mass beyond the cap sits on the cap).
    """
    rng = np.random.default_rng([w.seed, 1])
    law = w.length_law
    if law.startswith("fixed:"):
        vals = np.array([int(x) for x in law[6:].split(",")], dtype=np.int64)
        L = np.resize(vals, w.B)
    elif law == "lognormal_priority":
        L = np.rint(np.exp(rng.normal(np.log(300.0), 1.0, w.B))).astype(np.int64)
        L = np.clip(L, 1, w.max_len)
        key = L * np.exp(rng.normal(0.0, 0.1, w.B))
        L = L[np.argsort(key, kind="stable")]
    elif law == "bimodal":
        short = rng.integers(16, 257, w.B)
        long_ = rng.integers(1024, 4097, w.B)
        pick = rng.random(w.B) < 0.7
        L = np.where(pick, short, long_)
    elif law.startswith("uniform:"):
        a, b = (int(x) for x in law[8:].split(","))
        L = rng.integers(a, b + 1, w.B)
    elif law == "zipf":
        L = rng.zipf(1.2, w.B)
    else:
        raise ValueError(f"unknown length law {law!r}")
    return np.clip(L, 1, w.max_len).astype(np.int32)


@dataclass
class Paging:
    """Block tables of one batch.  Physical pages are a random permutation dealt
    out in logical order; every unused block-table entry names ``poison_page``,
    a real page nobody owns, so that a stray read stays in bounds."""
    lens: np.ndarray            # int32 [B]
    block_tables: np.ndarray    # int32 [B, max_blocks]
    num_pages: int              # pages in the cache, including the poison page
    poison_page: int
    max_blocks: int


def paging(w: Workload, lens: np.ndarray | None = None) -> Paging:
    lens = context_lens(w) if lens is None else np.asarray(lens, dtype=np.int32)
    rng = np.random.default_rng([w.seed, 2])
    nblk = (lens.astype(np.int64) + w.P - 1) // w.P
    total = int(nblk.sum())
    num_pages = total + 1
    perm = rng.permutation(num_pages).astype(np.int32)
    poison = int(perm[-1])
    max_blocks = max(1, int(nblk.max(initial=0)))
    bt = np.full((len(lens), max_blocks), poison, dtype=np.int32)
    start = 0
    for i, n in enumerate(nblk):
        bt[i, :n] = perm[start:start + n]
        start += int(n)
    return Paging(lens, bt, num_pages, poison, max_blocks)


def slots_of(w: Workload, pg: Paging, i: int, t0: int, t1: int) -> np.ndarray:
    """Slot indices (page * P + offset) of tokens t0..t1-1 of request i."""
    t = np.arange(t0, t1, dtype=np.int64)
    return pg.block_tables[i, t // w.P].astype(np.int64) * w.P + (t % w.P)


# --------------------------------------------------------------------------
# values

_POOL_SPAN = 1 << 24


def value_pool(w: Workload, n_min: int | None = None) -> np.ndarray:
    """A long seeded vector of fp16 N(0,1) samples from which every request's
    K and V are cut at seeded offsets.  Within one request the samples are
    i.i.d.; different requests may overlap in the pool, which changes nothing
    for a path that treats requests independently."""
    if n_min is None:
        n_min = int(w.max_len) * w.Hkv * w.D
    rng = np.random.default_rng([w.seed, 3])
    n = n_min + _POOL_SPAN
    out = np.empty(n, dtype=np.float16)
    step = 1 << 24
    for s in range(0, n, step):
        e = min(n, s + step)
        out[s:e] = rng.standard_normal(e - s, dtype=np.float32).astype(np.float16)
    return out


def request_offsets(w: Workload) -> Tuple[np.ndarray, np.ndarray]:
    """Pool offsets (K, V) of every request, in elements; multiples of 8 so that a
    slice of the pool is a 16-byte aligned fp16 tensor."""
    rng = np.random.default_rng([w.seed, 4])
    return (rng.integers(0, _POOL_SPAN // 8, w.B, dtype=np.int64) * 8,
            rng.integers(0, _POOL_SPAN // 8, w.B, dtype=np.int64) * 8)


def k_channel_gain(w: Workload) -> np.ndarray:
    """fp32 [Hkv, D] multiplier on K: ``outlier_frac`` of the channels of each KV
    head (a fixed subset, the same for every token) carry ``outlier_gain``."""
    gain = np.ones((w.Hkv, w.D), dtype=np.float32)
    if w.outlier_frac > 0:
        rng = np.random.default_rng([w.seed, 5])
        n = max(1, int(round(w.outlier_frac * w.D)))
        for h in range(w.Hkv):
            gain[h, rng.choice(w.D, n, replace=False)] = w.outlier_gain
    return gain


def request_kv(w: Workload, pool: np.ndarray, offs: Tuple[np.ndarray, np.ndarray],
               i: int, t0: int, t1: int, gain: np.ndarray | None = None
               ) -> Tuple[np.ndarray, np.ndarray]:
    """fp16 K and V of tokens t0..t1-1 of request i, each [t1-t0, Hkv, D]."""
    row = w.Hkv * w.D
    ko = int(offs[0][i]) + t0 * row
    vo = int(offs[1][i]) + t0 * row
    n = (t1 - t0) * row
    k = pool[ko:ko + n].reshape(t1 - t0, w.Hkv, w.D)
    v = pool[vo:vo + n].reshape(t1 - t0, w.Hkv, w.D)
    if gain is not None and w.outlier_frac > 0:
        k = (k.astype(np.float32) * gain[None]).astype(np.float16)
    return k, v


def queries(w: Workload) -> np.ndarray:
    """fp16 Q [B, H, D] ~ N(0,1)."""
    rng = np.random.default_rng([w.seed, 6])
    return rng.standard_normal((w.B, w.H, w.D), dtype=np.float32).astype(np.float16)


def step_tokens(w: Workload, lens: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """(request, position) of every token the *timed* quantize-and-write call stores:
    the decode token L_i-1 of every request and, when the workload has a prefill
    part, the last min(prefill_chunk, L_i-1) context tokens of every
    ``prefill_every``-th request."""
    req, pos = [], []
    for i, L in enumerate(lens):
        L = int(L)
        if L <= 0:
            continue
        t0 = L - 1
        if w.prefill_every and i % w.prefill_every == 0:
            t0 = max(0, L - 1 - w.prefill_chunk)
        req.append(np.full(L - t0, i, dtype=np.int32))
        pos.append(np.arange(t0, L, dtype=np.int32))
    if not req:
        return np.zeros(0, np.int32), np.zeros(0, np.int32)
    return np.concatenate(req), np.concatenate(pos)


def algorithmic_bytes_attn(w: Workload, lens: np.ndarray) -> int:
    """Bytes a decode-attention call must move: compressed K/V rows of every
    attended token, the block-table entries and lengths it needs, Q in, O out."""
    lens = lens.astype(np.int64)
    kv = int(lens.sum()) * w.Hkv * w.row_bytes
    bt = int(((lens + w.P - 1) // w.P).sum()) * 4
    return kv + bt + len(lens) * 4 + 2 * len(lens) * w.H * w.D * 2


def algorithmic_bytes_write(w: Workload, T: int) -> int:
    """Bytes a quantize-and-write call must move: fp16 K and V in, codes and
    meta out, one slot index per token."""
    return T * w.Hkv * (4 * w.D + w.row_bytes) + T * 8


def algorithmic_bytes_dequant(w: Workload, n_pages: int = 1) -> int:
    return n_pages * w.P * w.Hkv * (w.row_bytes + 4 * w.D)


# ---------------------------------------------------------------- job traces for the scheduler

def job_trace(n_jobs: int, seed: int, mean_gap: float = 40.0, max_prompt: int = 512, max_output: int = 256,
              pred_error: float = 0.1, underestimates: float = 0.15, prompt_median: float = 60.0, output_median: float = 40.0):
    """A seeded stream of serving jobs, stand-in for the chat traces the paper replays: Poisson
    arrivals (exponential gaps of `mean_gap` ticks), log-normal prompt and output lengths (the given
    medians, sigma 1) clipped to [1, max], a length prediction that is off by a normal relative error of `pred_error`, and a
    fraction `underestimates` of jobs whose prediction is a quarter of the truth (the short
    mispredictions the demote-and-double rule exists for).  Returns int64 arrays
    (arrival, prompt_len, output_len, predicted_len).  Holds no scheduler arithmetic."""
    rng = np.random.default_rng([seed, n_jobs])
    arrival = np.floor(np.cumsum(rng.exponential(mean_gap, n_jobs))).astype(np.int64)
    s = np.clip(np.round(np.exp(rng.normal(np.log(prompt_median), 1.0, n_jobs))), 1, max_prompt).astype(np.int64)
    n = np.clip(np.round(np.exp(rng.normal(np.log(output_median), 1.0, n_jobs))), 1, max_output).astype(np.int64)
    pred = np.maximum(1, np.round(n * (1.0 + pred_error * rng.standard_normal(n_jobs)))).astype(np.int64)
    low = rng.random(n_jobs) < underestimates
    pred[low] = np.maximum(1, n[low] // 4)
    return arrival, s, n, pred
