"""Pins for the oracle's AMAT quantiser, slicing and dequantisation (CPU only).

Nothing here compares the oracle with itself: each check is an exhaustive integer
identity, a closed form, or a special case whose answer is known in advance.
"""
import itertools

import numpy as np
import pytest

from oracle import slicemoe_oracle as O


def _qmat_from_codes(q, zp, scale, group, b_high=8, b_low=4):
    return O.QMat(np.asarray(q, np.uint8), np.asarray(zp, np.uint8), np.asarray(scale, np.float32),
                  group, b_high, b_low)


@pytest.mark.parametrize("b_high,b_low", [(8, 4), (6, 3), (4, 2)])
def test_slices_recombine_to_original_code_exhaustive(b_high, b_low):
    # Section 4.2 equation: q_low = floor(q_high / 2^shift); the LSB slice holds the rest.
    n = 1 << b_high
    shift = b_high - b_low
    q = np.arange(n, dtype=np.uint8)[None, :]
    m = _qmat_from_codes(q, [[0]], [[1.0]], n, b_high, b_low)
    for code in range(n):
        assert int(m.msb()[0, code]) == code // (2 ** shift)
        assert (int(m.msb()[0, code]) << shift) | int(m.lsb()[0, code]) == code
        assert int(m.lsb()[0, code]) < 2 ** shift


def test_golden_worked_example():
    # tests/golden/amat_example.txt: derived by hand from the Section 4.2 equation.
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "amat_example.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    for q, zp, s, hi, lo in rows:
        m = _qmat_from_codes([[int(q)]], [[int(zp)]], [[float(s)]], 1)
        assert m.dequant(O.HIGH)[0, 0] == float(hi)
        assert m.dequant(O.LOW)[0, 0] == float(lo)


def test_amat_identity_exhaustive_all_code_zeropoint_pairs():
    # 16*((q>>4)-(zp>>4)) - (q-zp) == (zp&15) - (q&15) for all 65,536 pairs, so
    # low - high = s*((zp&15)-(q&15)) and |low - high| <= 15 s exactly.
    s = 0.5
    q = np.tile(np.arange(256, dtype=np.uint8), (256, 1))
    zp = np.arange(256, dtype=np.uint8)[:, None]
    m = _qmat_from_codes(q, zp, np.full((256, 1), s, np.float32), 256)
    hi, lo = m.dequant(O.HIGH), m.dequant(O.LOW)
    for z in range(256):
        for c in range(256):
            assert hi[z, c] == s * (c - z)
            assert lo[z, c] == 16 * s * (c // 16 - z // 16)
            assert lo[z, c] - hi[z, c] == s * ((z % 16) - (c % 16))
    assert np.max(np.abs(lo - hi)) == 15 * s


def test_truncating_codes_only_is_far_worse_negative_control():
    # Table 1: truncating codes while keeping the full zero-point ("Trunc") destroys the
    # low-bit model, AMAT does not.  On synthetic weights the dequant error of the
    # codes-only variant is of order 16*zp*s, AMAT's is bounded by 15 s.
    rng = np.random.default_rng(0)
    W = (rng.standard_normal((64, 256)) * 0.02).astype(np.float32)
    m = O.quantize(W, 64)
    s = np.repeat(m.scale.astype(np.float64), 64, axis=1)
    zp = np.repeat(m.zp.astype(np.int64), 64, axis=1)
    trunc_only = 16 * s * ((m.q >> 4).astype(np.int64) - zp)          # zero-point NOT truncated
    err_trunc = np.sqrt(np.mean((trunc_only - W) ** 2))
    err_amat = np.sqrt(np.mean((m.dequant(O.LOW) - W) ** 2))
    assert err_trunc > 5 * err_amat
    # AMAT-low vs AMAT-high in units of the scale: difference of two uniform 0..15 digits
    r = np.sqrt(np.mean(((m.dequant(O.LOW) - m.dequant(O.HIGH)) / s) ** 2))
    assert 5.0 < r < 8.0                                              # sqrt(2*(256-1)/12) = 6.52
    # and within ~2x RMS of an independently quantised 4-bit model ("Base" rows of Table 1)
    base4 = O.quantize(W, 64, b_high=4, b_low=2)
    err_base = np.sqrt(np.mean((base4.dequant(O.HIGH) - W) ** 2))
    assert err_amat < 2.5 * err_base


@pytest.mark.parametrize("scale_dtype", ["f32", "bf16"])
@pytest.mark.parametrize("K,G", [(256, 64), (160, 64), (96, 32)])
def test_quantiser_recovers_exact_grid(scale_dtype, K, G):
    # If w = s0*(j - z0) with s0 a power of two and codes 0 and 255 present in every group,
    # min-max quantisation must return exactly s0, z0 and j (different per row AND per group,
    # which also fixes the group axis).
    rng = np.random.default_rng(1)
    N = 5
    ng = -(-K // G)
    j = rng.integers(0, 256, size=(N, K))
    z0 = rng.integers(0, 256, size=(N, ng))
    e0 = rng.integers(-12, -3, size=(N, ng))
    W = np.zeros((N, K), np.float32)
    for n in range(N):
        for g in range(ng):
            lo, hi = g * G, min(K, (g + 1) * G)
            j[n, lo] = 0
            j[n, hi - 1] = 255
            W[n, lo:hi] = (2.0 ** e0[n, g]) * (j[n, lo:hi] - z0[n, g])
    m = O.quantize(W, G, scale_dtype=scale_dtype)
    assert m.zp.shape == (N, ng) and m.scale.shape == (N, ng)
    assert np.array_equal(m.q, j.astype(np.uint8))
    assert np.array_equal(m.zp, z0.astype(np.uint8))
    assert np.array_equal(m.scale, (2.0 ** e0).astype(np.float32))
    assert np.array_equal(m.dequant(O.HIGH), W.astype(np.float64))


def test_quantiser_special_groups():
    W = np.zeros((3, 64), np.float32)
    W[1, :] = np.linspace(0.5, 1.0, 64)        # all positive: range is widened down to 0
    W[2, :] = -np.linspace(0.5, 1.0, 64)       # all negative: range is widened up to 0
    m = O.quantize(W, 64)
    assert m.scale[0, 0] == 1.0 and m.zp[0, 0] == 0 and not m.q[0].any()
    assert m.zp[1, 0] == 0 and m.q[1].max() == 255
    assert m.zp[2, 0] == 255 and m.q[2].min() == 0
    # an exact 0.0 weight always dequantises to exactly 0 at HIGH
    W2 = (np.random.default_rng(2).standard_normal((4, 128)) * 0.02).astype(np.float32)
    W2[:, ::7] = 0.0
    m2 = O.quantize(W2, 32, scale_dtype="bf16")
    assert np.all(m2.dequant(O.HIGH)[:, ::7] == 0.0)


@pytest.mark.parametrize("scale_dtype,bound_hi", [("f32", 1.0), ("bf16", 1.5)])
def test_dequant_error_bounds_on_synthetic_weights(scale_dtype, bound_hi):
    rng = np.random.default_rng(3)
    W = (rng.standard_normal((128, 512)) * 0.02).astype(np.float32)
    m = O.quantize(W, 128, scale_dtype=scale_dtype)
    s = np.repeat(m.scale.astype(np.float64), 128, axis=1)
    eh = np.abs(m.dequant(O.HIGH) - W) / s
    el = np.abs(m.dequant(O.LOW) - W) / s
    assert eh.max() <= bound_hi
    assert np.median(eh) < 0.3                  # round-to-nearest: uniform on [0, 0.5]
    assert el.max() <= 15.0 + bound_hi
    assert 0 <= m.q.min() and m.q.max() <= 255 and m.q.dtype == np.uint8


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -7, 1.0 + 3 * 2 ** -8, 3.1415927, -2.5e-5], np.float32)
    r = O.round_to_bf16(x)
    assert r[0] == 1.0 and r[1] == 1.0              # tie -> even mantissa
    assert r[2] == np.float32(1.0 + 2 ** -7)
    assert r[3] == np.float32(1.0 + 2 ** -6)        # tie -> even
    import torch
    assert np.array_equal(r, torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy())


def test_lower_bit_nests():
    # MAT63 / MAT42: same identities with shift 3 / 2.
    for b_high, b_low in [(6, 3), (4, 2)]:
        shift = b_high - b_low
        n = 1 << b_high
        q = np.tile(np.arange(n, dtype=np.uint8), (n, 1))
        zp = np.arange(n, dtype=np.uint8)[:, None]
        m = _qmat_from_codes(q, zp, np.full((n, 1), 0.25, np.float32), n, b_high, b_low)
        d = (m.dequant(O.LOW) - m.dequant(O.HIGH)) / 0.25
        for z, c in itertools.product(range(n), range(n)):
            assert d[z, c] == (z % (1 << shift)) - (c % (1 << shift))


@pytest.mark.parametrize("b_high,b_low", [(8, 4), (6, 3), (4, 2)])
def test_symmetric_variant_pins(b_high, b_low):
    # Symmetric integer quantisation (Section 6.1 item 1) in the unsigned store: what must hold whatever
    # the implementation -- the zero-point sits at mid-range, the largest magnitude of a group lands on
    # the last signed level, negating the weights mirrors every code about the zero-point, an exact
    # signed grid is recovered, and the error is at most half a step.
    rng = np.random.default_rng(5)
    half, G = 1 << (b_high - 1), 32
    W = rng.standard_normal((6, 96)).astype(np.float32)
    W[0, :32] = 0.0                                        # flat group
    m = O.quantize(W, G, b_high, b_low, symmetric=True)
    n = O.quantize(-W, G, b_high, b_low, symmetric=True)
    assert np.all(m.zp == half) and np.all(n.zp == half)
    assert np.array_equal(m.scale, n.scale)
    assert np.array_equal(m.q.astype(int) - half, -(n.q.astype(int) - half))
    assert m.q.min() >= 1                                  # level -2^(b-1) is never used
    assert np.all(m.q[0, :32] == half) and m.scale[0, 0] == 1.0
    Wg, qg = W.reshape(6, 3, G), m.q.reshape(6, 3, G).astype(int) - half
    j = np.abs(Wg).argmax(axis=2)
    top = np.take_along_axis(qg, j[:, :, None], axis=2)[:, :, 0]
    assert np.all(np.abs(top)[1:] == half - 1)
    assert np.array_equal(np.sign(top), np.sign(np.take_along_axis(Wg, j[:, :, None], axis=2)[:, :, 0]))
    err = np.abs(m.dequant(O.HIGH) - W.astype(np.float64)).reshape(6, 3, G)
    assert np.all(err <= 0.5 * m.scale[:, :, None].astype(np.float64) * (1 + 1e-6))
    # an exact grid: signed integers times a power-of-two step come back unchanged
    c = rng.integers(-(half - 1), half, size=(4, 64))
    c[:, 0] = half - 1
    c[:, 32] = -(half - 1)
    g = O.quantize((c * 0.25).astype(np.float32), G, b_high, b_low, symmetric=True)
    assert np.array_equal(g.q.astype(int) - half, c) and np.all(g.scale == 0.25)
    assert np.array_equal(g.dequant(O.HIGH), c * 0.25)
    # the low-bit model of the symmetric store is the truncated code against the truncated mid-point
    shift = b_high - b_low
    assert np.array_equal(g.dequant(O.LOW), 0.25 * (1 << shift) * ((g.q.astype(int) >> shift) - (half >> shift)))
