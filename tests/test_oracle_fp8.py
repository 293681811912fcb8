"""Pins of the oracle's 8-bit K/V storage (OCP FP8 E4M3 with one power-of-two scale per unit):
the code table against the format's definition, the encoder against a brute-force nearest-value
search with ties to even, the scale rule, and attention on a quantised cache against attention on
its decoded values."""
import math

import numpy as np
import pytest

from oracle import ref


def _table():
    return np.array([ref.fp8_e4m3_decode(c) for c in range(256)], dtype=np.float64)


def test_code_table_landmarks():
    t = _table()
    # the format's fixed points: zero, smallest subnormal, smallest normal, one, two, largest finite
    assert t[0x00] == 0.0 and t[0x80] == 0.0 and math.copysign(1.0, t[0x80]) == -1.0
    assert t[0x01] == 2.0 ** -9 and t[0x07] == 7 * 2.0 ** -9
    assert t[0x08] == 2.0 ** -6
    assert t[0x38] == 1.0 and t[0x40] == 2.0 and t[0x3C] == 1.5
    assert t[0x7E] == 448.0 and t[0xFE] == -448.0
    assert np.isnan(t[0x7F]) and np.isnan(t[0xFF])
    pos = t[:0x7F]
    assert np.all(np.diff(pos) > 0)                       # strictly increasing with the code
    assert np.array_equal(t[0x80:0xFF], -pos)             # the sign bit mirrors
    # 3 mantissa bits: neighbours inside a binade differ by 2^(e-3)
    for e in range(1, 15):
        seg = t[e * 8:(e + 1) * 8 + (0 if e == 15 else 1)]
        assert np.allclose(np.diff(seg[:8]), 2.0 ** (e - 7 - 3))


def test_encode_inverts_decode_for_every_finite_code():
    t = _table()
    for c in range(256):
        if np.isnan(t[c]):
            continue
        assert ref.fp8_e4m3_encode(t[c]) == c


def _nearest_code(a, t):
    """Brute force over the 127 non-negative finite values: nearest, ties to the even code."""
    pos = t[:0x7F]
    d = np.abs(pos - a)
    best = np.flatnonzero(d == d.min())
    if len(best) == 1:
        return int(best[0])
    return int(best[0] if best[0] % 2 == 0 else best[1])


def test_encode_is_round_to_nearest_even():
    t = _table()
    rng = np.random.default_rng(3)
    vals = np.concatenate([
        rng.uniform(0, 448, 3000), rng.uniform(0, 2.0 ** -5, 2000), 2.0 ** rng.uniform(-12, 8.8, 3000),
        (t[:0x7E] + t[1:0x7F]) / 2,                       # every tie between neighbours
        (t[:0x7E] + t[1:0x7F]) / 2 * (1 + 2.0 ** -20), (t[:0x7E] + t[1:0x7F]) / 2 * (1 - 2.0 ** -20),
    ]).astype(np.float32)
    for v in vals:
        a = float(v)
        if a > 448.0:
            continue
        want = _nearest_code(a, t)
        assert ref.fp8_e4m3_encode(a) == want, (a, want)
        assert ref.fp8_e4m3_encode(-a) == (want | 0x80)


def test_unit_scale_is_the_smallest_power_of_two_that_fits():
    rng = np.random.default_rng(5)
    x = (rng.standard_normal((3, 2, 50, 128)) * np.array([1e-3, 1.0, 37.0])[:, None, None, None]).astype(np.float32)
    x[0, 1] = 0.0                                         # an all-zero unit
    x[1, 0, 0, 0] = 448.0 * 4                             # exactly on the boundary: 448 * 2^2
    x[1, 0] = np.clip(x[1, 0], -448.0 * 4, 448.0 * 4)
    codes, scale = ref.quantize_fp8(x)
    for s in range(3):
        for h in range(2):
            amax = float(np.abs(x[s, h]).max())
            sc = float(scale[s, h])
            if amax == 0.0:
                assert sc == 1.0 and not codes[s, h].any()
                continue
            assert math.log2(sc) == round(math.log2(sc))
            assert amax <= 448.0 * sc and amax > 448.0 * sc / 2
    assert scale[1, 0] == 4.0 and codes[1, 0, 0, 0] == 0x7E
    # decoded values: within half a grid step (relative 2^-4 for normal numbers, 2^-10 * scale absolute below)
    y = ref.dequantize_fp8(codes, scale).astype(np.float64)
    err = np.abs(y - x)
    bound = np.maximum(np.abs(x) * 2.0 ** -4, 2.0 ** -10 * scale[:, :, None, None])
    assert np.all(err <= bound)
    # and they are exactly the table values times the scale
    t = _table()
    assert np.array_equal(y, t[codes] * scale[:, :, None, None].astype(np.float64))


def test_rows_quantised_with_given_scales_agree_with_the_unit_quantiser_and_saturate():
    """Rows that join later: inside the range the codes are those quantize_fp8 gives with the same scale
    (checked against the nearest-value search too); beyond it they take +-448, never a NaN code."""
    rng = np.random.default_rng(23)
    x = (rng.standard_normal((2, 2, 40, 128)) * np.array([0.3, 11.0])[:, None, None, None]).astype(np.float32)
    codes, scale = ref.quantize_fp8(x)
    assert np.array_equal(ref.quantize_fp8_scaled(x, scale), codes)
    t = _table()
    row = x[1, 1, :1].copy().reshape(1, 1, 1, 128)
    sc = scale[1:2, 1:2]
    row[0, 0, 0, :6] = np.array([448.0, 449.0, 1e9, -448.0, -460.0, -3e38], dtype=np.float32) * sc[0, 0]
    got = ref.quantize_fp8_scaled(row, sc)[0, 0, 0]
    assert list(got[:6]) == [0x7E, 0x7E, 0x7E, 0xFE, 0xFE, 0xFE]
    for j in range(6, 128):
        assert got[j] & 0x7F == _nearest_code(abs(float(row[0, 0, 0, j]) / float(sc[0, 0])), t)
    # a scale other than the unit's own: plain division, then the same rounding
    other = np.full((2, 2), 0.25, dtype=np.float32)
    y = ref.quantize_fp8_scaled(x[:, :, :2], other)
    for v, c in zip(x[0, 0, 0, :32], y[0, 0, 0, :32]):
        assert c == ref.fp8_e4m3_encode(min(max(float(v) / 0.25, -448.0), 448.0))


def test_attention_on_a_quantised_cache_is_attention_on_its_decoded_values():
    """Brute force in numpy on the decoded cache, against the oracle's sparse attention fed the same values."""
    rng = np.random.default_rng(11)
    S, Hkv, G, N, d, B = 1, 2, 2, 96, 128, 4
    K = rng.standard_normal((S, Hkv, N, d)).astype(np.float32)
    V = rng.standard_normal((S, Hkv, N, d)).astype(np.float32)
    q = rng.standard_normal((S, Hkv * G, d)).astype(np.float32)
    ids = rng.integers(0, B, (S, Hkv, N)).astype(np.int32)
    off, ln, idx, Ks, Vs = ref.build_bucket_index(ids, K, V, B, 0)
    K8, ks = ref.quantize_fp8(Ks)
    V8, vs = ref.quantize_fp8(Vs)
    Kd, Vd = ref.dequantize_fp8(K8, ks), ref.dequantize_fp8(V8, vs)
    # the oracle's attention reads keys by position through idx: decoded rows back in position order
    Kp, Vp = np.zeros_like(K), np.zeros_like(V)
    for h in range(Hkv):
        m = idx[0, h] >= 0
        Kp[0, h, idx[0, h][m]] = Kd[0, h][m]
        Vp[0, h, idx[0, h][m]] = Vd[0, h][m]
    sel = np.array([[[1, 3], [0, 2]]], dtype=np.int32)
    scale = np.float32(1.0 / math.sqrt(d))
    out, lse = ref.sparse_decode_attention(q, Kp, Vp, off, ln, idx, sel, scale)
    t = _table()
    for h in range(Hkv):
        rows = np.concatenate([np.arange(off[0, h, b], off[0, h, b] + ln[0, h, b]) for b in sel[0, h]])
        kk = t[K8[0, h, rows]] * float(ks[0, h])
        vv = t[V8[0, h, rows]] * float(vs[0, h])
        for g in range(G):
            a = float(scale) * (kk @ q[0, h * G + g].astype(np.float64))
            w = np.exp(a - a.max())
            np.testing.assert_allclose(out[0, h * G + g], (w / w.sum()) @ vv, rtol=1e-6, atol=1e-7)
            np.testing.assert_allclose(lse[0, h * G + g], a.max() + math.log(w.sum()), rtol=1e-6)
