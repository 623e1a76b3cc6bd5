"""Pins for the oracle's 8-bit (e4m3) row quantiser (CPU only)."""
import numpy as np
import torch

from oracle import mp_oracle as O


def _bf16(a):
    return torch.tensor(np.asarray(a), dtype=torch.float32).to(torch.bfloat16).to(torch.float64).numpy()


def test_value_table_is_the_e4m3_format():
    # against the library's own decoding of every finite non-negative code
    codes = torch.arange(0, 127, dtype=torch.uint8)
    ref = codes.view(torch.float8_e4m3fn).to(torch.float64).numpy()
    np.testing.assert_array_equal(O.e4m3_magnitudes(), ref)
    assert O.e4m3_magnitudes()[126] == 448.0 and O.e4m3_magnitudes()[1] == 2.0 ** -9


def test_codes_equal_library_conversion_of_the_scaled_row():
    rng = np.random.default_rng(0)
    X = _bf16(rng.normal(size=(200, 128)) * np.exp(rng.normal(size=(200, 1)) * 3))
    X[3] = 0.0                                  # an all-zero row
    X[4, 5:] = 0.0                              # a row with one large and many zero entries
    codes, scale = O.quantize_rows_e4m3(X)
    assert scale.dtype == np.float32 and codes.dtype == np.uint8
    amax = np.abs(X).max(1)
    np.testing.assert_array_equal(scale[amax > 0], (amax[amax > 0].astype(np.float32) / np.float32(448)))
    assert scale[3] == 1.0 and (codes[3] == 0).all()
    # independent conversion: torch's float32 -> float8_e4m3fn (round to nearest even) of the same quotients
    y = torch.tensor(X, dtype=torch.float32) / torch.tensor(scale)[:, None]
    assert float(y.abs().max()) < 449.0          # the fp32 quotient may exceed 448 by an ulp; both sides round it to 448
    ref = y.to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    same = codes == ref
    # (-0.0 and 0.0: the sign bit of a zero quotient may differ in representation only)
    assert (same | (((codes & 0x7f) == 0) & ((ref & 0x7f) == 0))).all()
    # the largest entry of every row maps to +-448 exactly
    np.testing.assert_array_equal(np.abs(O.dequantize_rows_e4m3(codes, scale)).max(1)[amax > 0],
                                  448.0 * scale[amax > 0].astype(np.float64))


def test_ties_go_to_the_even_code_and_overshoot_clamps():
    tab = O.e4m3_magnitudes()
    # a row whose largest entry is 448 has scale 1: entries are quantised as they are
    mids = (tab[40:60] + tab[41:61]) / 2            # exact midpoints between neighbouring values (bf16-representable here)
    row = np.concatenate([[448.0], mids, -mids])
    row = np.pad(row, (0, 128 - row.shape[0]))
    codes, scale = O.quantize_rows_e4m3(row[None])
    assert scale[0] == 1.0
    got = codes[0, 1:21].astype(int)
    want = np.array([c if c % 2 == 0 else c + 1 for c in range(40, 60)])
    np.testing.assert_array_equal(got, want)
    np.testing.assert_array_equal(codes[0, 21:41].astype(int), want | 0x80)


def test_dequantised_rows_are_close_and_exactly_representable():
    rng = np.random.default_rng(1)
    X = _bf16(rng.normal(size=(64, 128)) * 3)
    codes, scale = O.quantize_rows_e4m3(X)
    D = O.dequantize_rows_e4m3(codes, scale)
    # relative step of e4m3 is 2^-3: half of it bounds the rounding error of normal values; subnormal
    # values (below 2^-6 of the code range) are off by at most half a subnormal step, 2^-10 * scale
    err = np.abs(D - X)
    bound = np.maximum(np.abs(X) * 2.0 ** -4, 2.0 ** -10 * scale[:, None]) * (1 + 1e-6)
    assert (err <= bound).all()
    assert (D.astype(np.float32).astype(np.float64) * 0 == 0).all()


def test_key_residuals_use_the_cluster_centroid_and_shrink_the_error():
    rng = np.random.default_rng(2)
    cen = _bf16(rng.normal(size=(8, 128)) * 20)                      # far-apart cluster centroids
    which = rng.integers(0, 8, size=300)
    K = _bf16(cen[which] + rng.normal(size=(300, 128)) * 0.3)
    codes, scale = O.quantize_keys_e4m3(K, cen[which])
    # the codes are those of the fp32 difference, by the library's conversion
    r = torch.tensor(K, dtype=torch.float32) - torch.tensor(cen[which], dtype=torch.float32)
    y = r / torch.tensor(scale)[:, None]
    ref = y.to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert ((codes == ref) | (((codes & 0x7f) == 0) & ((ref & 0x7f) == 0))).all()
    np.testing.assert_array_equal(scale, (r.abs().amax(1) / 448).numpy())
    D = O.dequantize_keys_e4m3(codes, scale, cen[which])
    np.testing.assert_array_equal(D - cen[which], O.dequantize_rows_e4m3(codes, scale))
    # the error is a sixteenth of the residual, not of the key
    direct = O.dequantize_rows_e4m3(*O.quantize_rows_e4m3(K))
    assert np.abs(D - K).max() < 0.15 and np.abs(direct - K).max() > 1.0
    # a key that equals its centroid is stored exactly
    codes0, scale0 = O.quantize_keys_e4m3(cen[:3], cen[:3])
    assert (codes0 & 0x7f == 0).all() and (scale0 == 1).all()
    np.testing.assert_array_equal(O.dequantize_keys_e4m3(codes0, scale0, cen[:3]), cen[:3])
