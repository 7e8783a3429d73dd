"""The oracle's own fp16 <-> fp32 conversions against numpy's IEEE binary16."""
import numpy as np


def test_h2f_exhaustive(oracle_mod):
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float32)
    got = np.array([oracle_mod.h2f(int(b)) for b in bits], dtype=np.float32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))


def test_f2h_rne_random_and_edges(oracle_mod):
    rng = np.random.default_rng(7)
    xs = np.concatenate([
        rng.standard_normal(20000).astype(np.float32),
        (rng.standard_normal(5000) * 1e-5).astype(np.float32),          # subnormal results
        (rng.standard_normal(5000) * 3e4).astype(np.float32),           # near overflow
        np.array([0.0, -0.0, 65504.0, 65519.99, 65520.0, 1e9, -1e9, 2.0**-24, 2.0**-25,
                  2.0**-25 * 1.0001, 3 * 2.0**-25, 2.0**-14, 2.0**-14 - 2.0**-25], np.float32),
    ])
    # exact ties between neighbouring fp16 values, to exercise ties-to-even
    h = rng.integers(0x0001, 0x7bff, 4000).astype(np.uint16)
    lo = h.view(np.float16).astype(np.float64)
    hi = (h + 1).astype(np.uint16).view(np.float16).astype(np.float64)
    xs = np.concatenate([xs, ((lo + hi) / 2).astype(np.float32)])
    with np.errstate(over="ignore"):
        want = xs.astype(np.float16).view(np.uint16)
    got = np.array([oracle_mod.f2h_rne(float(x)) for x in xs], dtype=np.uint16)
    assert np.array_equal(got, want)
