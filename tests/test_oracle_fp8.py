"""Pins of the 8-bit GEMM checker (oracle/fp8_oracle.py) to things other than itself: the code
points the OFP8 specification names, a library's own E4M3 conversion, bounds that follow from
the format, and exact rational arithmetic."""
from fractions import Fraction

import numpy as np
import torch

from oracle import fp8_oracle as F


def test_code_points_named_by_the_format():
    # OFP8 E4M3: bias 7, max normal S.1111.110 = 448, min normal S.0001.000 = 2^-6,
    # max subnormal S.0000.111 = 0.875 * 2^-6, min subnormal S.0000.001 = 2^-9, NaN S.1111.111
    dec = F.e4m3_decode(np.arange(256, dtype=np.uint8))
    assert dec[0x7E] == 448.0 and dec[0xFE] == -448.0
    assert dec[0x08] == 2.0 ** -6 and dec[0x07] == 0.875 * 2.0 ** -6 and dec[0x01] == 2.0 ** -9
    assert dec[0x38] == 1.0 and dec[0x40] == 2.0 and dec[0x3C] == 1.5 and dec[0xB8] == -1.0
    assert dec[0x00] == 0.0 and dec[0x80] == 0.0 and np.signbit(dec[0x80])
    assert np.isnan(dec[0x7F]) and np.isnan(dec[0xFF])
    assert np.isfinite(dec).sum() == 254                      # no infinities, two NaN codes
    pos = dec[:0x7F]
    assert np.all(np.diff(pos) > 0)                           # code order is value order


def test_decode_and_encode_against_a_library_conversion():
    codes = torch.arange(256, dtype=torch.uint8)
    lib = codes.view(torch.float8_e4m3fn).to(torch.float32).numpy().astype(np.float64)
    mine = F.e4m3_decode(codes.numpy())
    assert np.array_equal(np.isnan(lib), np.isnan(mine))
    ok = ~np.isnan(lib)
    assert np.array_equal(lib[ok], mine[ok]) and np.array_equal(np.signbit(lib[ok]), np.signbit(mine[ok]))

    rng = np.random.default_rng(5)
    pos = mine[:0x7F]
    halfway = (pos[:-1] + pos[1:]) / 2                        # every tie, exactly representable in binary32
    x = np.concatenate([
        rng.normal(0, 1, 20000), rng.normal(0, 100, 20000), rng.uniform(-448, 448, 20000),
        rng.normal(0, 2.0 ** -8, 5000),                       # subnormal range and below
        halfway, -halfway, np.nextafter(halfway, 0), np.nextafter(halfway, 1e9),
        pos, -pos, [0.0, -0.0, 448.0, -448.0, 2.0 ** -10, 2.0 ** -10 * 1.0001, 2.0 ** -11]]).astype(np.float32)
    x = x[np.abs(x) <= 448.0]                                 # the library does not saturate above 448
    lib_codes = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = F.e4m3_encode(x)
    assert np.array_equal(got, lib_codes)


def test_ties_go_to_the_even_code_and_large_values_saturate():
    assert F.e4m3_encode(np.float32(1.0625)) == 0x38          # between 1.0 (0x38) and 1.125 (0x39)
    assert F.e4m3_encode(np.float32(1.1875)) == 0x3A          # between 1.125 (0x39) and 1.25 (0x3a)
    assert F.e4m3_encode(np.float32(2.0 ** -10)) == 0x00      # half of the smallest subnormal: to even (zero)
    assert F.e4m3_encode(np.float32(3 * 2.0 ** -10)) == 0x02  # between codes 1 and 2
    assert F.e4m3_encode(np.float32(-1.0625)) == 0xB8
    for v, c in ((448.0, 0x7E), (449.0, 0x7E), (464.0, 0x7E), (1e6, 0x7E), (np.inf, 0x7E), (-1e6, 0xFE)):
        assert F.e4m3_encode(np.float32(v)) == c
    assert F.e4m3_encode(np.float32(np.nan)) == 0x7F


def test_row_quantisation_bounds():
    rng = np.random.default_rng(11)
    x = rng.normal(0, 1, (37, 200)).astype(np.float32)
    x[3] = 0.0                                                # an all-zero row
    x[4] *= 1e-6
    x[5] *= 1e4
    x[6, 1:] = 0.0                                            # one non-zero entry
    codes, scale = F.quantize_rows(x)
    assert codes.dtype == np.uint8 and scale.dtype == np.float32 and scale[3] == 1.0 and not codes[3].any()
    amax = np.abs(x).max(axis=1)
    nz = amax > 0
    assert np.allclose(scale[nz], amax[nz] / 448.0, rtol=1e-6)
    assert np.all((codes[nz] & 0x7F).max(axis=1) == 0x7E)     # the largest entry of a row maps to +-448
    back = F.e4m3_decode(codes) * scale[:, None].astype(np.float64)
    err = np.abs(back - x)
    # round to nearest with 3 mantissa bits: relative error <= 2^-4 for normals (>= 2^-6 * scale),
    # absolute error <= 2^-10 * scale below
    bound = np.maximum(np.abs(x) * 2.0 ** -4, scale[:, None] * 2.0 ** -10) * (1 + 1e-5)
    assert np.all(err <= bound)
    assert np.array_equal(np.signbit(back)[x != 0], np.signbit(x)[x != 0])


def test_product_against_rational_arithmetic():
    rng = np.random.default_rng(3)
    M, N, K = 5, 4, 24
    a = rng.normal(0, 1, (M, K)).astype(np.float32)
    w = rng.normal(0, 0.05, (N, K)).astype(np.float32)
    ac, sa = F.quantize_rows(a)
    wc, sw = F.quantize_rows(w)
    got = F.gemm_fp8(ac, sa, wc, sw)

    def frac_of(code):                                       # E4M3 value as an exact fraction, from the bit fields
        code = int(code)
        s = -1 if code & 0x80 else 1
        e, m = (code >> 3) & 0xF, code & 7
        return s * (Fraction(m, 8) * Fraction(1, 64) if e == 0 else Fraction(8 + m, 8) * Fraction(2) ** (e - 7))

    for m in range(M):
        for n in range(N):
            acc = sum(frac_of(ac[m, k]) * frac_of(wc[n, k]) for k in range(K))
            want = float(acc * Fraction(float(sa[m])) * Fraction(float(sw[n])))
            assert abs(got[m, n] - want) <= 1e-12 * max(1.0, abs(want))
    # and the quantised product approximates the exact one to the format's precision
    exact = a.astype(np.float64) @ w.astype(np.float64).T
    scale = np.sqrt((a.astype(np.float64) ** 2).sum(1))[:, None] * np.sqrt((w.astype(np.float64) ** 2).sum(1))[None, :]
    assert np.max(np.abs(got - exact) / scale) < 0.08
    # transposed operands give the transposed product (rows of W are output features)
    assert np.allclose(F.gemm_fp8(wc, sw, ac, sa), got.T, rtol=1e-12, atol=0)


# ---------------------------------------------------------------- the projections of a layer

from oracle import lazyllm_oracle as O
from paper_2407_14057_amd import synth


def test_projection_is_exact_when_nothing_needs_rounding():
    """Operands whose rows quantise without loss (entries are E4M3 values times a power of two,
    largest magnitude 448 * 2^j) must give the plain product, with and without the folded
    RMSNorm: a dropped or misplaced scale, a gain folded on the wrong axis or a missing 1/rms
    would show."""
    rng = np.random.default_rng(21)
    vals = F.e4m3_decode(np.arange(0x7F, dtype=np.uint8))
    M, N, K = 7, 9, 40
    a = rng.choice(vals, (M, K)) * rng.choice([-1.0, 1.0], (M, K))
    a[:, 0] = 448.0
    a *= 2.0 ** rng.integers(-6, 3, (M, 1))
    w = rng.choice(vals, (N, K)) * rng.choice([-1.0, 1.0], (N, K))
    w[:, 3] = -448.0
    w *= 2.0 ** rng.integers(-12, -4, (N, 1))
    assert np.allclose(O.projection_8bit(a, w), a @ w.T, rtol=1e-12, atol=0)
    # with a gain: entries of w * gain must stay E4M3 values relative to the row's peak, so the
    # weights are taken from the values >= 0.5, the gains from {1/4, 1/2, 1, 2, 4}, and the peak
    # (448 under the largest gain) is planted in column 3
    big = vals[vals >= 0.5]
    w = rng.choice(big, (N, K)) * rng.choice([-1.0, 1.0], (N, K))
    gain = 2.0 ** rng.integers(-2, 3, K).astype(np.float64)
    gain[3] = 4.0
    w[:, 3] = -448.0
    w *= 2.0 ** rng.integers(-12, -4, (N, 1))
    eps = 1e-5
    got = O.projection_8bit(a, w, gain, eps)
    want = O.rmsnorm(a, gain, eps) @ w.T
    assert np.allclose(got, want, rtol=1e-12, atol=0)
    assert not np.allclose(got, O.rmsnorm(a, np.ones(K), eps) @ w.T, rtol=1e-3, atol=0)


def test_layer_with_8bit_projections_is_close_to_the_exact_layer_but_not_equal():
    shape = synth.TINY
    w = synth.weights_to_host_bits(synth.make_weights(shape, 5, "cpu", gain_jitter=0.25))
    lw = O.LayerWeights(w, 1, np.float64)
    rng = np.random.default_rng(4)
    m = 48
    h = O.round_to_bf16(rng.normal(0, 1, (m, shape.d_model)))
    pos = np.arange(m)
    ref = O.decoder_layer(h, pos, lw, shape.n_heads, shape.head_dim, shape.rms_eps, shape.rope_theta)
    got = O.decoder_layer(h, pos, lw, shape.n_heads, shape.head_dim, shape.rms_eps, shape.rope_theta, gemm8=True)
    for name, r, g, tol in (("h", ref[0], got[0], 0.05), ("k", ref[1], got[1], 0.08), ("v", ref[2], got[2], 0.08)):
        rel = np.sqrt(np.mean((g - r) ** 2) / np.mean(r ** 2))
        assert 1e-4 < rel < tol, (name, rel)                         # quantised, but to the format's precision
    assert abs(got[3].sum() - 1.0) < 1e-9                            # Eq. 1 is still a mean of distributions
    # fusing the rows of several weight matrices into one product changes nothing (scales are per row)
    sep = np.concatenate([O.projection_8bit(h, lw.wq, lw.attn_norm, 1e-5), O.projection_8bit(h, lw.wk, lw.attn_norm, 1e-5)], axis=1)
    fused = O.projection_8bit(h, np.concatenate([lw.wq, lw.wk], axis=0), lw.attn_norm, 1e-5)
    assert np.array_equal(sep, fused)
