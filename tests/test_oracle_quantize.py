"""Pins for the oracle's quantizer (Section 3.1.1; relative scale of Section 4.2).

Nothing here re-uses the oracle to check itself: the expected values are closed forms, invariants from the
definition (|x - x'| <= rel_eb * range), numpy reductions along the axis the paper names, or hand-picked grids
whose codes are known by construction.
"""
import numpy as np
import pytest

import workloads as W

K, V = 0, 1


def _tile(rng, scale=1.0):
    return (rng.standard_normal((64, 128)) * scale).astype(np.float16)


@pytest.mark.parametrize("rel_eb,n", [(5e-3, 101), (1e-2, 51), (2e-2, 26), (0.25, 3), (0.5, 2), (0.125, 5)])
def test_n_sym(oracle, rel_eb, n):
    # bins of width 2*rel_eb*range cover [min, max] with 1/(2 rel_eb) + 1 levels
    assert oracle.n_sym(rel_eb) == n


def test_n_sym_rejects(oracle):
    assert oracle.n_sym(0.6) < 0
    assert oracle.n_sym(0.0) < 0
    assert oracle.n_sym(1.0 / 1024) < 0  # would need more than 256 levels (codes are unsigned 8-bit)


@pytest.mark.parametrize("which", [K, V])
@pytest.mark.parametrize("rel_eb", [5e-3, 1e-2, 2e-2, 0.1])
def test_error_bound_every_element(oracle, which, rel_eb):
    rng = np.random.default_rng(11)
    for scale in (1.0, 1e-3, 300.0, 6e-6):
        x = _tile(rng, scale)
        x[5, :] *= 7  # an outlier token
        x[:, 9] *= 11  # an outlier channel
        x = np.clip(x, -60000, 60000).astype(np.float16)
        codes, mm = oracle.quantize_block(which, x, rel_eb)
        xd = oracle.dequantize_block(which, codes, mm, rel_eb)
        x64 = x.astype(np.float64)
        axis = 0 if which == K else 1  # K: per channel over the 64 tokens; V: per token over the 128 channels
        rng_unit = x64.max(axis=axis, keepdims=True) - x64.min(axis=axis, keepdims=True)
        eb = rel_eb * rng_unit
        assert np.all(np.abs(x64 - xd) <= eb * (1 + 1e-4) + 1e-30)
        assert codes.max() <= oracle.n_sym(rel_eb) - 1


@pytest.mark.parametrize("which", [K, V])
def test_units_and_minmax_follow_the_named_axis(oracle, which):
    rng = np.random.default_rng(3)
    x = _tile(rng)
    x *= np.linspace(1, 30, 128, dtype=np.float16)[None, :]  # distinct channel scales
    x *= np.linspace(1, 5, 64, dtype=np.float16)[:, None]  # distinct token scales
    codes, mm = oracle.quantize_block(which, x, 1e-2)
    axis = 0 if which == K else 1
    assert mm.shape == ((128, 2) if which == K else (64, 2))
    np.testing.assert_array_equal(mm[:, 0].view(np.float16), x.min(axis=axis))
    np.testing.assert_array_equal(mm[:, 1].view(np.float16), x.max(axis=axis))
    # minimum maps to code 0, maximum to the top level, in every unit
    amin, amax = x.argmin(axis=axis), x.argmax(axis=axis)
    for u in range(mm.shape[0]):
        lo = codes[amin[u], u] if which == K else codes[u, amin[u]]
        hi = codes[amax[u], u] if which == K else codes[u, amax[u]]
        assert lo == 0 and hi == 50


def test_block_mode_is_one_unit(oracle):
    rng = np.random.default_rng(4)
    x = _tile(rng)
    codes, mm = oracle.quantize_block(K, x, 1e-2, k_mode=1)
    assert mm.shape == (1, 2)
    assert mm[0, 0].view(np.float16) == x.min() and mm[0, 1].view(np.float16) == x.max()
    xd = oracle.dequantize_block(K, codes, mm, 1e-2, k_mode=1)
    rngv = float(x.max()) - float(x.min())
    assert np.all(np.abs(x.astype(np.float64) - xd) <= 1e-2 * rngv * (1 + 1e-4))


@pytest.mark.parametrize("which", [K, V])
def test_integer_grid_round_trips_exactly(oracle, which):
    # every unit spans [0, 50]; with rel_eb = 1e-2 the bin width is 1, so integer inputs are their own codes
    rng = np.random.default_rng(5)
    k = rng.integers(0, 51, (64, 128))
    if which == K:
        k[0, :], k[1, :] = 0, 50
    else:
        k[:, 0], k[:, 1] = 0, 50
    x = k.astype(np.float16)
    codes, mm = oracle.quantize_block(which, x, 1e-2)
    np.testing.assert_array_equal(codes, k.astype(np.uint8))
    xd = oracle.dequantize_block(which, codes, mm, 1e-2)
    assert np.max(np.abs(xd - k)) < 1e-5


def test_round_half_to_even(oracle):
    # rel_eb = 0.125: bin width = 0.25 * range exactly; range 4 -> width 1; halves go to the even level
    x = np.zeros((64, 128), np.float16)
    x[:, :] = 4.0
    x[0, :] = 0.0
    x[1, :], x[2, :], x[3, :], x[4, :] = 0.5, 1.5, 2.5, 3.5
    codes, _ = oracle.quantize_block(K, x, 0.125)
    assert codes[1, 0] == 0 and codes[2, 0] == 2 and codes[3, 0] == 2 and codes[4, 0] == 4
    assert codes[0, 0] == 0 and codes[5, 0] == 4


def test_constant_unit_and_signed_zero(oracle):
    x = np.full((64, 128), 3.25, np.float16)
    x[:, 7] = np.float16(-0.0)
    x[::2, 7] = np.float16(0.0)
    for which in (K, V):
        xx = x.copy()
        if which == V:
            xx[:] = 3.25
            xx[7, :] = np.float16(-0.0)
            xx[7, ::2] = np.float16(0.0)
        codes, mm = oracle.quantize_block(which, xx, 1e-2)
        assert np.all(codes == 0)
        xd = oracle.dequantize_block(which, codes, mm, 1e-2)
        np.testing.assert_array_equal(xd, xx.astype(np.float64))
        assert mm[7, 0] == 0 and mm[7, 1] == 0  # stored as +0


def test_non_finite_is_rejected(oracle):
    x = np.ones((64, 128), np.float16)
    x[3, 3] = np.inf
    with pytest.raises(ValueError):
        oracle.quantize_block(K, x, 1e-2)
    x[3, 3] = np.nan
    with pytest.raises(ValueError):
        oracle.quantize_block(V, x, 1e-2)


def test_fp16_conversion_is_exact_on_all_finite_patterns(oracle):
    # dequantizing code 0 returns the unit minimum: sweep every finite binary16 pattern through that path
    pats = np.arange(0, 0x10000, dtype=np.uint32).astype(np.uint16)
    pats = pats[np.isfinite(pats.view(np.float16))]
    assert len(pats) == 63488 and len(pats) % 64 == 0
    for i in range(0, len(pats), 64):
        # V-style units (per token): make each token constant so that min == the pattern under test
        x = np.repeat(pats[i:i + 64, None], 128, axis=1).view(np.float16)
        codes, mm = oracle.quantize_block(V, x, 1e-2)
        assert not codes.any()
        xd = oracle.dequantize_block(V, codes, mm, 1e-2)
        np.testing.assert_array_equal(xd, x.astype(np.float64))


def test_histogram_equals_bincount(oracle):
    K_, V_ = W.make_kv(1, 2, 256, 7)
    codes, _ = oracle.tensor_quantize(K, K_, 1e-2)
    h = oracle.histogram(codes)
    np.testing.assert_array_equal(h, np.bincount(codes.reshape(-1), minlength=256).astype(np.uint64))
    assert h.sum() == 1 * 2 * 256 * 128


def test_tensor_quantize_matches_block_by_block_gather(oracle):
    # layout pin: block (b,h,j) of [B,S,H,128] is X[b, 64j:64j+64, h, :]
    K_, V_ = W.make_kv(2, 3, 200, 9)  # 3 full blocks, 8 tokens left over
    for which, X in ((K, K_), (V, V_)):
        codes, mm = oracle.tensor_quantize(which, X, 2e-2)
        assert codes.shape[0] == 2 * 3 * 3
        i = 0
        for b in range(2):
            for h in range(3):
                for j in range(3):
                    c1, m1 = oracle.quantize_block(which, X[b, 64 * j:64 * j + 64, h, :], 2e-2)
                    np.testing.assert_array_equal(codes[i], c1)
                    np.testing.assert_array_equal(mm[i], m1)
                    i += 1


def test_float_to_half_matches_numpy_on_a_dense_sweep(oracle):
    """The oracle's own binary32 -> binary16 rounding against numpy's, on every half value, the midpoints between
    neighbours (ties), just above and below them, and the overflow and underflow edges."""
    halves = np.arange(0, 0x7c00, dtype=np.uint16).view(np.float16).astype(np.float32)
    mids = (halves[:-1].astype(np.float64) + halves[1:].astype(np.float64)) / 2.0
    cand = [halves, mids.astype(np.float32), np.nextafter(mids.astype(np.float32), np.float32(np.inf)),
            np.nextafter(mids.astype(np.float32), np.float32(-np.inf)),
            np.array([65504.0, 65519.99, 65520.0, 65520.01, 1e6, 2.0**-25, np.nextafter(np.float32(2.0**-25), np.float32(1)),
                      2.0**-26, 0.0, 3.0e-8, 5.9604645e-08], np.float32)]
    xs = np.concatenate(cand)
    xs = np.concatenate([xs, -xs])
    rng = np.random.default_rng(3)
    pick = rng.choice(len(xs), 6000, replace=False)
    with np.errstate(over="ignore"):
        for x in xs[pick]:
            assert oracle.float_to_half_bits(x) == int(np.float32(x).astype(np.float16).view(np.uint16)), float(x)


def test_fp16_reconstruction_is_one_rounding_of_the_binary32_value(oracle):
    rng = np.random.default_rng(11)
    for which, k_mode in ((K, 0), (K, 1), (V, 0)):
        x = (rng.standard_normal((64, 128)) * rng.lognormal(0, 1.0, 128)).astype(np.float16)
        codes, mm = oracle.quantize_block(which, x, 1e-2, k_mode=k_mode)
        rec = oracle.reconstruct_block_fp16(which, codes, mm, 1e-2, k_mode=k_mode)
        mmf = mm.view(np.float16).astype(np.float32)
        step = (np.float32(2.0) * np.float32(1e-2)) * (mmf[:, 1] - mmf[:, 0])
        if which == V:
            mn, st = mmf[:, 0][:, None], step[:, None]
        elif k_mode == 1:
            mn, st = mmf[0, 0], step[0]
        else:
            mn, st = mmf[:, 0][None, :], step[None, :]
        expect = (mn + codes.astype(np.float32) * st).astype(np.float16)   # numpy: float32 ops, then one rounding
        np.testing.assert_array_equal(rec.view(np.uint16), expect.view(np.uint16))
        # and it stays within the error bound plus half a binary16 ulp of the input
        exact = oracle.dequantize_block(which, codes, mm, 1e-2, k_mode=k_mode)
        assert np.abs(rec.astype(np.float64) - exact).max() <= np.abs(exact).max() * 2.0**-11
