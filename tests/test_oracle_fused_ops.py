"""Pins for the oracle's fused residual add + LayerNorm and bias + ReLU (ALISE Sec. 3.3
"Implementation": fused kernels for LayerNorm and ReLU; Sec. 2 "Transformer Architecture":
LayerNorm and residual connection around the attention and FFN modules).  CPU only.

Pins: hand-derived rows (tests/golden/layernorm_worked_examples.txt); PyTorch's layer_norm in
fp64; numpy's correctly rounded fp64 -> fp16 conversion for the one-rounding sums; closed
forms and invariants of the definition (a constant row returns beta; zero mean and unit
variance of the normalized row; invariance under a shift of the row and, with eps = 0, under
a positive scaling; rows are independent; the affine part is affine)."""
import os

import numpy as np
import pytest
import torch

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "layernorm_worked_examples.txt")


def _rows():
    out = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        f = [c.strip() for c in line.split(";")]
        vec = lambda s: np.array([float(t) for t in s.split()], np.float64)
        out.append(dict(x=vec(f[0]), res=None if f[1] == "-" else vec(f[1]), gamma=vec(f[2]), beta=vec(f[3]),
                        eps=float(f[4]), h=vec(f[5]), y=vec(f[6])))
    return out


@pytest.mark.parametrize("row", _rows(), ids=lambda r: "x=" + " ".join(f"{v:g}" for v in r["x"]))
def test_hand_derived_rows(oracle_mod, row):
    h, y = oracle_mod.add_layernorm(row["x"][None].astype(np.float16),
                                    None if row["res"] is None else row["res"][None].astype(np.float16),
                                    row["gamma"].astype(np.float16), row["beta"].astype(np.float16), row["eps"])
    assert np.array_equal(h[0].astype(np.float64), row["h"])
    assert np.abs(y[0] - row["y"]).max() < 1e-14


def _problem(rows, hidden, seed, with_res=True):
    rng = np.random.default_rng(seed)
    x = (rng.standard_normal((rows, hidden)) * rng.uniform(0.1, 4.0, (rows, 1))).astype(np.float16)
    res = (rng.standard_normal((rows, hidden)) * 2.0 + rng.uniform(-3, 3, (rows, 1))).astype(np.float16) if with_res else None
    gamma = (1.0 + 0.2 * rng.standard_normal(hidden)).astype(np.float16)
    beta = (0.3 * rng.standard_normal(hidden)).astype(np.float16)
    return x, res, gamma, beta


@pytest.mark.parametrize("shape", [(7, 64), (3, 5120), (5, 1000), (2, 8), (4, 1)])
@pytest.mark.parametrize("with_res", [True, False])
def test_against_torch_layer_norm(oracle_mod, shape, with_res):
    x, res, gamma, beta = _problem(*shape, seed=11, with_res=with_res)
    eps = 1e-5
    h, y = oracle_mod.add_layernorm(x, res, gamma, beta, eps)
    # the sum of two fp16 numbers is exact in fp64, and numpy rounds fp64 -> fp16 correctly (to nearest even)
    h_ref = x.astype(np.float64) + (res.astype(np.float64) if with_res else 0.0)
    h_ref = h_ref.astype(np.float16)
    assert np.array_equal(h.view(np.uint16), h_ref.view(np.uint16))
    want = torch.nn.functional.layer_norm(torch.from_numpy(h_ref.astype(np.float64)), (shape[1],),
                                          torch.from_numpy(gamma.astype(np.float64)), torch.from_numpy(beta.astype(np.float64)), eps)
    assert np.abs(y - want.numpy()).max() < 1e-11


def test_sum_is_rounded_once_to_nearest_even(oracle_mod):
    one = np.ones(4, np.float16)
    zero = np.zeros(4, np.float16)
    # 2048 + 1 = 2049 lies halfway between 2048 and 2050: ties to even -> 2048; 2050 + 1 = 2051 -> 2052
    x = np.array([[2048, 2050, 1, -2048]], np.float16)
    r = np.array([[1, 1, 2.0 ** -11, -1]], np.float16)
    h, _ = oracle_mod.add_layernorm(x, r, one, zero, 1e-5)
    assert h[0].astype(np.float64).tolist() == [2048.0, 2052.0, 1.0, -2048.0]
    # overflow of the sum rounds to infinity like any fp16 rounding
    h, _ = oracle_mod.add_layernorm(np.array([[60000, 1, 1, 1]], np.float16), np.array([[60000, 1, 1, 1]], np.float16), one, zero, 1e-5)
    assert np.isinf(h[0, 0])


def test_constant_row_returns_beta(oracle_mod):
    x, _, gamma, beta = _problem(1, 96, seed=5)
    x[:] = np.float16(1.375)
    _, y = oracle_mod.add_layernorm(x, None, gamma, beta, 1e-5)
    assert np.array_equal(y[0], beta.astype(np.float64))


def test_normalized_row_has_zero_mean_and_unit_variance(oracle_mod):
    x, res, _, _ = _problem(6, 2048, seed=9)
    one, zero = np.ones(2048, np.float16), np.zeros(2048, np.float16)
    _, y = oracle_mod.add_layernorm(x, res, one, zero, 0.0)
    assert np.abs(y.mean(axis=1)).max() < 1e-13
    assert np.abs(y.var(axis=1) - 1.0).max() < 1e-12
    # with eps the variance of the output is var / (var + eps)
    h, y2 = oracle_mod.add_layernorm(x, res, one, zero, 0.5)
    v = h.astype(np.float64).var(axis=1)
    assert np.abs(y2.var(axis=1) - v / (v + 0.5)).max() < 1e-12


def test_shift_and_scale_invariance(oracle_mod):
    rng = np.random.default_rng(3)
    x = rng.integers(-64, 64, (3, 128)).astype(np.float16)          # small integers: shifts and doublings are exact in fp16
    gamma = (1.0 + 0.2 * rng.standard_normal(128)).astype(np.float16)
    beta = (0.3 * rng.standard_normal(128)).astype(np.float16)
    _, y = oracle_mod.add_layernorm(x, None, gamma, beta, 0.0)
    _, y_shift = oracle_mod.add_layernorm(x, np.full_like(x, 100.0), gamma, beta, 0.0)      # h = x + 100, exact
    assert np.abs(y - y_shift).max() < 1e-12
    _, y_scale = oracle_mod.add_layernorm((x * np.float16(4)).astype(np.float16), None, gamma, beta, 0.0)
    assert np.abs(y - y_scale).max() < 1e-12
    _, y_neg = oracle_mod.add_layernorm(-x, None, gamma, np.zeros_like(beta), 0.0)         # odd in h once beta is gone
    _, y_pos = oracle_mod.add_layernorm(x, None, gamma, np.zeros_like(beta), 0.0)
    assert np.abs(y_neg + y_pos).max() < 1e-12


def test_rows_are_independent_and_channels_permute(oracle_mod):
    x, res, gamma, beta = _problem(5, 256, seed=21)
    h, y = oracle_mod.add_layernorm(x, res, gamma, beta, 1e-5)
    h1, y1 = oracle_mod.add_layernorm(x[2:3], res[2:3], gamma, beta, 1e-5)
    assert np.array_equal(h[2:3], h1) and np.array_equal(y[2:3], y1)
    perm = np.random.default_rng(2).permutation(256)
    _, yp = oracle_mod.add_layernorm(x[:, perm], res[:, perm], gamma[perm], beta[perm], 1e-5)
    assert np.abs(yp - y[:, perm]).max() < 1e-12                   # only the order of the two sums changes


def test_affine_part(oracle_mod):
    x, res, gamma, beta = _problem(3, 64, seed=33)
    one, zero = np.ones(64, np.float16), np.zeros(64, np.float16)
    _, n = oracle_mod.add_layernorm(x, res, one, zero, 1e-5)
    _, y = oracle_mod.add_layernorm(x, res, gamma, beta, 1e-5)
    assert np.abs(y - (gamma.astype(np.float64) * n + beta.astype(np.float64))).max() < 1e-13


# ---------------------------------------------------------------- bias + ReLU

def test_bias_relu_against_numpy(oracle_mod):
    rng = np.random.default_rng(8)
    x = (rng.standard_normal((9, 333)) * 3).astype(np.float16)
    b = rng.standard_normal(333).astype(np.float16)
    want = np.maximum(x.astype(np.float64) + b.astype(np.float64), 0.0).astype(np.float16)
    got = oracle_mod.bias_relu(x, b)
    assert np.array_equal(got.view(np.uint16), want.view(np.uint16))
    assert np.array_equal(oracle_mod.bias_relu(x, None).view(np.uint16), np.maximum(x, np.float16(0)).view(np.uint16))


def test_bias_relu_special_values(oracle_mod):
    x = np.array([[-0.0, 0.0, -1.0, 1.0, 2048.0, 2050.0, 65504.0, -65504.0, 6e-8]], np.float16)
    b = np.array([0.0, -0.0, 1.0, -1.0, 1.0, 1.0, 65504.0, 65504.0, -6e-8], np.float16)
    got = oracle_mod.bias_relu(x, b)
    assert got.view(np.uint16).tolist() == [[0, 0, 0, 0, 0x6800, 0x6802, 0x7c00, 0, 0]]       # +0 for -0 and for exact cancellation; 2049 -> 2048, 2051 -> 2052; overflow -> inf


def test_bias_relu_is_idempotent_without_bias(oracle_mod):
    rng = np.random.default_rng(1)
    x = rng.standard_normal((4, 50)).astype(np.float16)
    y = oracle_mod.bias_relu(x, None)
    assert np.array_equal(oracle_mod.bias_relu(y, None), y)
    assert (y >= 0).all() and np.array_equal(y[x > 0], x[x > 0])


def test_d2h_rounds_once(oracle_mod):
    # 1 + 2^-11 + 2^-30 is just above the halfway point between 1 and 1 + 2^-10: one rounding goes up,
    # a detour through fp32 (which drops the 2^-30) would land on the tie and go down to 1
    assert oracle_mod.d2h(1.0 + 2.0 ** -11 + 2.0 ** -30) == 0x3c01
    assert oracle_mod.d2h(1.0 + 2.0 ** -11) == 0x3c00
    assert oracle_mod.d2h(-65520.0) == 0xfc00 and oracle_mod.d2h(65519.9) == 0x7bff
    assert oracle_mod.d2h(2.0 ** -25) == 0 and oracle_mod.d2h(2.0 ** -25 * 1.0001) == 1       # half of the smallest subnormal: tie to even
    for v in (0.1, -3.14159, 1e-6, 123.456, 5.96e-8, 6.1e-5):
        assert oracle_mod.d2h(v) == int(np.float64(v).astype(np.float16).view(np.uint16))
