"""GPU parity of the fused residual add + LayerNorm and bias + ReLU (ALISE Sec. 3.3
"Implementation"; Sec. 2 "Transformer Architecture") against the CPU oracle, through the C ABI.

The residual sum h and the ReLU output are exact sums rounded once: compared bit for bit.
The LayerNorm output is an fp32 evaluation rounded once to fp16, the oracle's an fp64 one:
the bar is half a unit in the last place of fp16 plus the error of the fp32 arithmetic,
16 fp32 units on the terms of the formula,

    |y - y_oracle| <= ulp16(y_oracle) / 2 + 2^-20 * (|gamma| * (max|h| + |mean|) / sqrt(var + eps) + |y_oracle|),

and nearly all outputs must be the correctly rounded value itself."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2410_23537_amd import binding
    import oracle
    oracle.build()
    return binding, torch, oracle


def _ulp16(v):
    a = np.abs(v)
    e = np.floor(np.log2(np.maximum(a, 2.0 ** -14)))
    return 2.0 ** (e - 10)


def _ln_problem(rows, hidden, seed):
    rng = np.random.default_rng([seed, rows, hidden])
    x = (rng.standard_normal((rows, hidden)) * rng.uniform(0.05, 6.0, (rows, 1))).astype(np.float16)
    # a residual stream with a few outlier channels and a per-row offset, as transformer activations have
    res = (rng.standard_normal((rows, hidden)) * 1.5 + rng.uniform(-4, 4, (rows, 1))).astype(np.float16)
    res[:, rng.integers(0, hidden, max(1, hidden // 256))] *= np.float16(12.0)
    gamma = (1.0 + 0.3 * rng.standard_normal(hidden)).astype(np.float16)
    beta = (0.5 * rng.standard_normal(hidden)).astype(np.float16)
    return x, res, gamma, beta


def _check_ln(oracle, x, res, gamma, beta, eps, h_got, y_got):
    h_want, y_want = oracle.add_layernorm(x, res, gamma, beta, eps)
    if h_got is not None:
        assert np.array_equal(h_got.view(np.uint16), h_want.view(np.uint16)), "the residual sum must be bit-exact"
    h64 = h_want.astype(np.float64)
    mean = h64.mean(axis=1, keepdims=True)
    rstd = 1.0 / np.sqrt(h64.var(axis=1, keepdims=True) + eps)
    spread = (np.abs(h64).max(axis=1, keepdims=True) + np.abs(mean)) * rstd
    tol = 0.5 * _ulp16(y_want) + 2.0 ** -20 * (np.abs(gamma.astype(np.float64)) * spread + np.abs(y_want))
    err = np.abs(y_got.astype(np.float64) - y_want)
    assert np.isfinite(y_got).all()
    assert (err <= tol).all(), f"worst excess {np.max(err - tol):.3e} at {np.unravel_index(np.argmax(err - tol), err.shape)}"
    exact = np.mean(y_got.view(np.uint16) == y_want.astype(np.float16).view(np.uint16))
    assert exact >= 0.99, f"only {exact:.4f} of the outputs are the correctly rounded value"


LN_SHAPES = [(1, 8), (5, 64), (7, 512), (13, 1000), (9, 1024), (3, 1032), (6, 2048), (5, 2560), (33, 4096), (17, 5120),
             (3, 6144), (4, 7168), (3, 9216), (2, 12288), (2, 16384), (1025, 128), (0, 256)]


@pytest.mark.parametrize("shape", LN_SHAPES, ids=lambda s: f"{s[0]}x{s[1]}")
@pytest.mark.parametrize("mode", ["residual", "plain"])
def test_add_layernorm_against_oracle(env, shape, mode):
    B, torch, oracle = env
    rows, hidden = shape
    print(f"case add_layernorm {rows}x{hidden} {mode}", flush=True)
    x, res, gamma, beta = _ln_problem(rows, hidden, seed=77)
    if mode == "plain":
        res = None
    eps = 1e-5
    xd, gd, bd = torch.from_numpy(x).cuda(), torch.from_numpy(gamma).cuda(), torch.from_numpy(beta).cuda()
    rd = None if res is None else torch.from_numpy(res).cuda()
    # outputs with a guard row behind them
    hbuf = torch.full((rows + 1, hidden), 7.0, dtype=torch.float16, device="cuda")
    ybuf = torch.full((rows + 1, hidden), 9.0, dtype=torch.float16, device="cuda")
    B.alise_add_layernorm(xd, rd, gd, bd, eps, hbuf[:rows], ybuf[:rows])
    torch.cuda.synchronize()
    assert (hbuf[rows:] == 7.0).all() and (ybuf[rows:] == 9.0).all(), "wrote past the last row"
    if rows:
        _check_ln(oracle, x, res, gamma, beta, eps, hbuf[:rows].cpu().numpy(), ybuf[:rows].cpu().numpy())


def test_add_layernorm_in_place_and_without_the_sum(env):
    B, torch, oracle = env
    x, res, gamma, beta = _ln_problem(19, 5120, seed=5)
    gd, bd = torch.from_numpy(gamma).cuda(), torch.from_numpy(beta).cuda()
    # the usual decoder-layer call: the residual stream is updated in place, the normalized row replaces x
    xd, rd = torch.from_numpy(x).cuda(), torch.from_numpy(res).cuda()
    B.alise_add_layernorm(xd, rd, gd, bd, 1e-5, rd, xd)
    torch.cuda.synchronize()
    _check_ln(oracle, x, res, gamma, beta, 1e-5, rd.cpu().numpy(), xd.cpu().numpy())
    # no h_out at all
    xd, rd = torch.from_numpy(x).cuda(), torch.from_numpy(res).cuda()
    y = torch.empty_like(xd)
    B.alise_add_layernorm(xd, rd, gd, bd, 1e-5, None, y)
    torch.cuda.synchronize()
    _check_ln(oracle, x, res, gamma, beta, 1e-5, None, y.cpu().numpy())
    assert np.array_equal(xd.cpu().numpy(), x) and np.array_equal(rd.cpu().numpy(), res)      # inputs untouched


def test_add_layernorm_degenerate_rows(env):
    B, torch, oracle = env
    hidden = 256
    rng = np.random.default_rng(4)
    gamma = (1.0 + 0.3 * rng.standard_normal(hidden)).astype(np.float16)
    beta = (0.5 * rng.standard_normal(hidden)).astype(np.float16)
    x = np.zeros((4, hidden), np.float16)
    x[0] = 3.25                                   # a constant row: y = beta
    x[1, 0] = 1000.0                              # one spike
    x[2] = np.float16(6e-8)                       # subnormals, constant
    x[3] = (rng.standard_normal(hidden) * 2.0 ** -12).astype(np.float16)      # tiny values: eps dominates the variance
    y = torch.empty((4, hidden), dtype=torch.float16, device="cuda")
    B.alise_add_layernorm(torch.from_numpy(x).cuda(), None, torch.from_numpy(gamma).cuda(), torch.from_numpy(beta).cuda(),
                          1e-5, None, y)
    torch.cuda.synchronize()
    got = y.cpu().numpy()
    assert np.array_equal(got[0], beta) and np.array_equal(got[2], beta)
    _check_ln(oracle, x, None, gamma, beta, 1e-5, None, got)


RELU_SHAPES = [(1, 8), (3, 64), (1000, 8), (7, 2056), (33, 20480), (5, 4096), (257, 1024), (4099, 24), (0, 64)]


@pytest.mark.parametrize("shape", RELU_SHAPES, ids=lambda s: f"{s[0]}x{s[1]}")
@pytest.mark.parametrize("mode", ["bias", "plain", "in_place"])
def test_bias_relu_against_oracle(env, shape, mode):
    B, torch, oracle = env
    rows, cols = shape
    print(f"case bias_relu {rows}x{cols} {mode}", flush=True)
    rng = np.random.default_rng([9, rows, cols])
    x = (rng.standard_normal((rows, cols)) * 3).astype(np.float16)
    if rows:
        specials = np.array([-0.0, 0.0, 6e-8, -6e-8, 65504.0, -65504.0, 2048.0, 2050.0], np.float16)
        x[0, :8] = specials
    b = None if mode == "plain" else rng.standard_normal(cols).astype(np.float16)
    if b is not None:
        b[:8] = np.array([0.0, -0.0, -6e-8, 6e-8, 65504.0, 65504.0, 1.0, 1.0], np.float16)
    want = oracle.bias_relu(x, b)
    buf = torch.full((rows + 1, cols), 5.0, dtype=torch.float16, device="cuda")
    bd = None if b is None else torch.from_numpy(b).cuda()
    if mode == "in_place":
        buf[:rows] = torch.from_numpy(x).cuda()
        B.alise_bias_relu(buf[:rows], bd, buf[:rows])
    else:
        B.alise_bias_relu(torch.from_numpy(x).cuda(), bd, buf[:rows])
    torch.cuda.synchronize()
    assert (buf[rows:] == 5.0).all(), "wrote past the last row"
    assert np.array_equal(buf[:rows].cpu().numpy().view(np.uint16), want.view(np.uint16))


@pytest.mark.parametrize("n16", [0, 1, 255, 256 * 8 * 3 + 5, 1 << 20, (1 << 22) + 12345])
def test_read_probe_folds_every_word_once(env, n16):
    """The streaming-read probe returns the exclusive-or of all 32-bit words of the buffer: every
    16-byte unit is read exactly once, whatever the size is relative to the grid and its unrolling."""
    B, torch, _ = env
    rng = np.random.default_rng([77, n16])
    host = rng.integers(0, 1 << 32, size=n16 * 4, dtype=np.uint32)
    src = torch.from_numpy(host.view(np.int32)).cuda()
    out = torch.full((1,), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
    B.alise_hbm_read_probe(src, out)
    torch.cuda.synchronize()
    want = int(np.bitwise_xor.reduce(host)) if n16 else 0
    assert int(out.cpu().numpy().view(np.uint32)[0]) == want


def test_issue_probe_runs_in_all_three_modes(env):
    """The issue probe (matrix instructions, vector instructions, both) is a timing utility: it must run, end, and
    leave its sink alone."""
    B, torch, _ = env
    sink = torch.full((1,), 3.5, dtype=torch.float32, device="cuda")
    for mode in (1, 2, 3):
        B.alise_issue_overlap_probe(mode, 50, sink)
    B.alise_issue_overlap_probe(3, 0, sink)
    torch.cuda.synchronize()
    assert float(sink[0]) == 3.5
