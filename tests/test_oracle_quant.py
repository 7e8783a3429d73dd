"""Pins for the oracle's quantizer, writer and page dequantizer (ALISE Sec. 3.2,
"KV Compression").  Nothing here touches a GPU or the HIP library.

Pins used: the hand-derived worked examples under tests/golden/, an exact
rational re-derivation (every rounding done from first principles on
``fractions.Fraction``), the half-step error bound, and structural invariants of
an affine quantizer.
"""
import os
from fractions import Fraction

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "quant_worked_examples.txt")


def _golden_rows():
    rows = []
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        b, xs, sh, z, codes, dq = [s.strip() for s in line.split(";")]
        rows.append((int(b), [float(t) for t in xs.split()], int(sh, 16), int(z),
                     [int(t) for t in codes.split()],
                     None if dq == "-" else [int(t, 16) for t in dq.split()]))
    return rows


@pytest.mark.parametrize("row", _golden_rows())
def test_worked_examples(oracle_mod, row):
    bits, xs, scale_hex, zero, codes, dq = row
    x = np.array(xs, np.float16)
    assert np.array_equal(x.astype(np.float64), np.array(xs))  # the examples are exact fp16 values
    c, sh, zh = oracle_mod.quant_group(x, bits)
    assert sh == scale_hex
    assert zh == int(np.float16(zero).view(np.uint16))
    assert list(c) == codes
    # the same group through the oracle's writer and its page dequantizer: one KV head whose vector is this group,
    # written to the second slot of a two-slot page (K carries the group, V its mirror image, so a mix-up shows)
    n = len(xs)
    cache = oracle_mod.Cache.empty(1, 2, 1, n, bits, n, fill=0xEE)
    oracle_mod.kv_quant_write(cache, x.reshape(1, 1, n), x[::-1].reshape(1, 1, n), np.array([1], np.int64))
    assert cache.k_meta[0, 0, 1, 0].view(np.uint16).tolist() == [scale_hex, int(np.float16(zero).view(np.uint16))]
    stored = cache.k_codes[0, 0, 1]
    unpacked = stored if bits == 8 else np.stack([stored & 15, stored >> 4], axis=-1).reshape(-1)
    assert list(unpacked) == codes
    if dq is not None:
        kd, vd = oracle_mod.kv_dequant_page(cache, 0)
        assert [int(v) for v in kd[1, 0].view(np.uint16)] == dq          # the hand-derived column, not a restatement
        assert [int(v) for v in vd[1, 0].view(np.uint16)] == dq[::-1]


# ---------------------------------------------------------------------------
# exact rational re-derivation: roundings implemented on Fractions, no float ops

def _round_to_format(v: Fraction, sig_bits: int, emin: int) -> Fraction:
    """Round a rational to a binary format with `sig_bits` significant bits and
    minimum normal exponent `emin` (gradual underflow), nearest, ties to even."""
    if v == 0:
        return Fraction(0)
    s = -1 if v < 0 else 1
    a = abs(v)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1                      # 2^e <= a < 2^(e+1)
    e = max(e, emin)
    ulp = Fraction(2) ** (e - (sig_bits - 1))
    n = a / ulp
    fl = n.numerator // n.denominator
    rem = n - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        fl += 1
    return s * fl * ulp


def _f32(v):
    return _round_to_format(Fraction(v), 24, -126)


def _f16(v):
    return _round_to_format(Fraction(v), 11, -14)


def _rint_even(v: Fraction) -> int:
    fl = v.numerator // v.denominator
    rem = v - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        fl += 1
    return int(fl)


def _exact_quant(xs, bits):
    """The quantizer with every operation carried out exactly and rounded explicitly."""
    qmax = (1 << bits) - 1
    x = [Fraction(float(v)) for v in xs]
    mn = min(min(x), Fraction(0))
    mx = max(max(x), Fraction(0))
    r = _f32(mx - mn)
    l32 = _f32(r / qmax)
    h = _f16(l32)
    if h < l32:                                     # next binary16 above
        e = h.numerator.bit_length() - h.denominator.bit_length() if h else -100
        if h and Fraction(2) ** e > h:
            e -= 1
        e = max(e, -14)
        h = h + Fraction(2) ** (e - 10)
    h = max(h, Fraction(2) ** -14)
    inv = _f32(1 / h)
    z = min(max(_rint_even(_f32(-mn * inv)), 0), qmax)
    codes = [min(max(_rint_even(_f32(v * inv + z)), 0), qmax) for v in x]   # one rounding: fused
    return codes, h, z


def _groups(rng, n, G, outliers=True):
    x = rng.standard_normal((n, G)).astype(np.float32)
    if outliers:
        mask = rng.random((n, G)) < 0.05
        x = np.where(mask, x * 10, x)
    x[: n // 8] = np.abs(x[: n // 8])            # all non-negative groups
    x[n // 8: n // 4] = -np.abs(x[n // 8: n // 4])   # all non-positive groups
    return x.astype(np.float16)


@pytest.mark.parametrize("bits,G", [(8, 128), (8, 64), (4, 32), (8, 16), (4, 128)])
def test_exact_rational_rederivation(oracle_mod, bits, G):
    rng = np.random.default_rng(100 + bits + G)
    xs = _groups(rng, 60, G)
    xs[0] = 0
    xs[1] = np.float16(6e-8)                      # subnormal inputs -> floor of the scale
    xs[2, :] = np.float16(0.3)                    # constant group
    xs[3] = (rng.standard_normal(G) * 3000).astype(np.float16)   # large magnitudes
    for x in xs:
        c, sh, zh = oracle_mod.quant_group(x, bits)
        codes, h, z = _exact_quant(x, bits)
        assert Fraction(float(np.uint16(sh).view(np.float16))) == h
        assert float(np.uint16(zh).view(np.float16)) == z
        assert list(map(int, c)) == codes


@pytest.mark.parametrize("bits,G", [(8, 128), (8, 64), (4, 32)])
def test_half_step_bound_and_structure(oracle_mod, bits, G):
    rng = np.random.default_rng(200 + bits + G)
    qmax = (1 << bits) - 1
    xs = _groups(rng, 3000, G)
    worst = 0.0
    for x in xs:
        c, sh, zh = oracle_mod.quant_group(x, bits)
        lam = float(np.uint16(sh).view(np.float16))
        z = float(np.uint16(zh).view(np.float16))
        xf = x.astype(np.float64)
        c = c.astype(np.int64)
        assert 0 <= z <= qmax and z == int(z)
        assert c.min() >= 0 and c.max() <= qmax
        xhat = lam * (c - z)
        err = np.abs(xf - xhat) / lam
        worst = max(worst, err.max())
        # x = 0 maps to the zero-point and back to exactly 0
        x0 = np.concatenate([x, [np.float16(0)]])
        c0, sh0, zh0 = oracle_mod.quant_group(x0, bits)
        assert (sh0, zh0) == (sh, zh) and c0[-1] == z
        # monotone
        order = np.argsort(xf, kind="stable")
        assert np.all(np.diff(c[order]) >= 0)
        if xf.min() < 0:
            assert c[np.argmin(xf)] == 0
        if xf.min() >= 0 and xf.max() > 0 and sh > 0x0400:
            assert c[np.argmax(xf)] == qmax
        # the stored scale is the smallest fp16 >= range/qmax
        rng_ = max(xf.max(), 0) - min(xf.min(), 0)
        l32 = float(np.float32(np.float32(rng_) / np.float32(qmax)))
        assert lam >= l32
        below = float(np.uint16(sh - 1).view(np.float16))
        assert below < l32 or sh == 0x0400
    assert worst <= 0.5 + 1e-4


@pytest.mark.parametrize("bits", [4, 8])
def test_power_of_two_scaling_invariance(oracle_mod, bits):
    rng = np.random.default_rng(31 + bits)
    for _ in range(300):
        x = rng.standard_normal(32).astype(np.float16)
        k = int(rng.integers(-4, 6))
        c1, s1, z1 = oracle_mod.quant_group(x, bits)
        c2, s2, z2 = oracle_mod.quant_group((x.astype(np.float32) * 2.0 ** k).astype(np.float16), bits)
        # fp16 inputs in the normal range scale exactly; skip groups holding subnormals
        if np.any((np.abs(x) < 2.0 ** -9) & (x != 0)):
            continue
        assert np.array_equal(c1, c2) and z1 == z2
        assert float(np.uint16(s2).view(np.float16)) == float(np.uint16(s1).view(np.float16)) * 2.0 ** k


def _np_unpack(codes_packed, bits, D):
    if bits == 8:
        return codes_packed
    lo = codes_packed & 0xF
    hi = codes_packed >> 4
    return np.stack([lo, hi], axis=-1).reshape(*codes_packed.shape[:-1], D)


@pytest.mark.parametrize("bits,G,D", [(8, 64, 64), (4, 32, 128), (8, 32, 128)])
def test_writer_layout_and_page_dequant(oracle_mod, bits, G, D):
    """Writer puts every (token, head) row at its slot in the canonical layout;
    INT4 packs channel 2i low / 2i+1 high; untouched slots keep their fill; the page
    dequantizer equals lambda*(code - zero) rounded to fp16."""
    rng = np.random.default_rng(5 + bits + D)
    P, Hkv, pages, T = 16, 3, 7, 40
    cache = oracle_mod.Cache.empty(pages, P, Hkv, D, bits, G, fill=0xAB)
    k = rng.standard_normal((T, Hkv, D)).astype(np.float16)
    v = (rng.standard_normal((T, Hkv, D)) * 2 + 0.5).astype(np.float16)
    slots = rng.permutation(pages * P)[:T].astype(np.int64)
    slots[5] = -1                                    # skipped token
    oracle_mod.kv_quant_write(cache, k, v, slots)
    written = np.zeros((pages, P), bool)
    for t in range(T):
        if slots[t] < 0:
            continue
        pg, off = divmod(int(slots[t]), P)
        written[pg, off] = True
        for h in range(Hkv):
            for src, codes, meta in ((k, cache.k_codes, cache.k_meta), (v, cache.v_codes, cache.v_meta)):
                row = _np_unpack(codes[pg, h, off], bits, D)
                for g in range(D // G):
                    c, sh, zh = oracle_mod.quant_group(src[t, h, g * G:(g + 1) * G], bits)
                    assert np.array_equal(row[g * G:(g + 1) * G], c)
                    assert meta[pg, h, off, g, 0].view(np.uint16) == sh
                    assert meta[pg, h, off, g, 1].view(np.uint16) == zh
    assert np.all(cache.k_codes[~written[:, None, :].repeat(Hkv, 1)] == 0xAB)
    assert np.all(cache.v_codes[~written[:, None, :].repeat(Hkv, 1)] == 0xAB)
    # page dequantizer, all slots of a page (written or not)
    pg = int(slots[0] // P)
    kd, vd = oracle_mod.kv_dequant_page(cache, pg)
    for out, codes, meta in ((kd, cache.k_codes, cache.k_meta), (vd, cache.v_codes, cache.v_meta)):
        u = _np_unpack(codes[pg], bits, D).astype(np.float32)            # [Hkv, P, D]
        lam = np.repeat(meta[pg, ..., 0].astype(np.float32), G, axis=-1)
        z = np.repeat(meta[pg, ..., 1].astype(np.float32), G, axis=-1)
        want = (lam * (u - z)).astype(np.float16).transpose(1, 0, 2)      # [P, Hkv, D]
        assert np.array_equal(out.view(np.uint16), want.view(np.uint16))


def test_dequant_of_zero_point_is_zero(oracle_mod):
    cache = oracle_mod.Cache.empty(1, 16, 2, 64, 8, 64)
    cache.k_codes[:] = 77
    cache.v_codes[:] = 77
    cache.k_meta[..., 0] = 0.37
    cache.k_meta[..., 1] = 77
    cache.v_meta[..., 0] = 1.5
    cache.v_meta[..., 1] = 77
    kd, vd = oracle_mod.kv_dequant_page(cache, 0)
    assert not kd.any() and not vd.any()
