"""CPU pins of the E4M3 oracle: against the format's definition, a library's independent conversion and brute force."""
import numpy as np
import torch

from oracle import fp8, nn

ALL = np.arange(256, dtype=np.uint8)


def test_decode_matches_the_format_definition():
    v = fp8.e4m3_decode(ALL)
    # landmarks of the OCP E4M3 table: zero, smallest subnormal 2^-9, largest subnormal 7 * 2^-9, smallest normal 2^-6,
    # one, two, the largest finite value 448 = 1.75 * 2^8, and the two NaN codes; no infinities anywhere
    assert v[0x00] == 0.0 and v[0x80] == 0.0 and np.signbit(v[0x80])
    assert v[0x01] == 2.0 ** -9 and v[0x07] == 7 * 2.0 ** -9 and v[0x08] == 2.0 ** -6
    assert v[0x38] == 1.0 and v[0x40] == 2.0 and v[0x3C] == 1.5 and v[0x7E] == 448.0 and v[0xFE] == -448.0
    assert np.isnan(v[0x7F]) and np.isnan(v[0xFF]) and np.isfinite(np.delete(v, [0x7F, 0xFF])).all()
    # the codes of one sign are ordered like their values (what makes it a floating-point format)
    pos = v[:0x7F]
    assert (np.diff(pos) > 0).all() and np.array_equal(v[0x80:0xFF], -pos)
    # generic rule, written out once more from the definition, bit by bit
    for c in range(256):
        s, e, m = c >> 7, (c >> 3) & 15, c & 7
        if e == 15 and m == 7:
            continue
        mag = m * 2.0 ** -9 if e == 0 else (1 + m / 8) * 2.0 ** (e - 7)
        assert v[c] == (-mag if s else mag)


def test_decode_and_encode_match_an_independent_library_conversion():
    v = fp8.e4m3_decode(ALL)
    t = torch.from_numpy(ALL.copy()).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    assert np.array_equal(np.isnan(v), np.isnan(t)) and np.array_equal(v[~np.isnan(v)], t[~np.isnan(t)])
    rng = np.random.default_rng(3)
    x = np.concatenate([rng.standard_normal(100000).astype(np.float32) * s for s in (1e-3, 0.02, 1.0, 30.0, 300.0)])
    ref = torch.from_numpy(x).clamp(-448, 448).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(fp8.e4m3_encode(x), ref)


def test_encode_rounds_to_nearest_ties_to_even_and_saturates():
    v = fp8.e4m3_decode(ALL)
    ok = ~np.isnan(v)
    assert np.array_equal(fp8.e4m3_encode(v[ok].astype(np.float32)), ALL[ok])            # representable values are fixed points
    pos = v[:0x7F]
    for c in range(0x7E):
        lo, hi = pos[c], pos[c + 1]
        mid = np.float32((lo + hi) / 2)                                                  # exact in fp32
        even = c if c % 2 == 0 else c + 1
        assert fp8.e4m3_encode(mid) == even, (c, mid)
        assert fp8.e4m3_encode(np.nextafter(mid, np.float32(0))) == c
        assert fp8.e4m3_encode(np.nextafter(mid, np.float32(1e9))) == c + 1
        assert fp8.e4m3_encode(-mid) == (even | 0x80)
    sat = np.float32([448.0, 449.0, 464.0, 465.0, 1e30, np.inf])
    assert (fp8.e4m3_encode(sat) == 0x7E).all() and (fp8.e4m3_encode(-sat) == 0xFE).all()
    assert fp8.e4m3_encode(np.float32(np.nan)) == 0x7F
    assert fp8.e4m3_encode(np.float32(2.0 ** -10)) == 0x00 and fp8.e4m3_encode(np.nextafter(np.float32(2.0 ** -10), np.float32(1))) == 0x01
    # a worked example by hand: 0.3 lies between 0.28125 (0x29) and 0.3125 (0x2A), nearer the latter
    assert fp8.e4m3_encode(np.float32(0.3)) == 0x2A and fp8.e4m3_decode(np.uint8(0x2A)) == 0.3125


def test_conv_e4m3_equals_brute_force_on_hand_decoded_values():
    rng = np.random.default_rng(5)
    xc = rng.integers(0, 0x70, (2, 5, 6, 4)).astype(np.uint8) | (rng.integers(0, 2, (2, 5, 6, 4)).astype(np.uint8) << 7)
    wc = rng.integers(0, 0x60, (3, 3, 3, 4)).astype(np.uint8) | (rng.integers(0, 2, (3, 3, 3, 4)).astype(np.uint8) << 7)
    table = [(-1.0 if c & 0x80 else 1.0) * ((c & 7) * 2.0 ** -9 if (c >> 3) & 15 == 0 else (1 + (c & 7) / 8) * 2.0 ** (((c >> 3) & 15) - 7))
             for c in range(256)]
    xv = np.vectorize(lambda c: table[c])(xc).astype(np.float64)
    wv = np.vectorize(lambda c: table[c])(wc).astype(np.float64)
    scale = np.float64([0.5, 2.0, 0.125]); bias = np.float64([0.25, -1.0, 3.0])
    for stride, pad in ((1, 1), (2, 0)):
        ref = nn.direct_conv(xv, wv, stride, pad) * scale + bias
        got = fp8.conv_e4m3(xc, wc, scale, bias, stride, pad, nn.ACT_NONE)
        assert np.allclose(got, ref, rtol=1e-13, atol=1e-13)
        relu = fp8.conv_e4m3(xc, wc, scale, bias, stride, pad, nn.ACT_RELU)
        assert np.array_equal(relu, np.maximum(got, 0.0))
    # residual before / after the activation
    rc = rng.integers(0, 0x70, (2, 5, 6, 3)).astype(np.uint8)
    rv = np.vectorize(lambda c: table[c])(rc) * 0.75
    base = nn.direct_conv(xv, wv, 1, 1) * scale + bias
    assert np.allclose(fp8.conv_e4m3(xc, wc, scale, bias, 1, 1, nn.ACT_RELU, rc, 0.75, nn.RES_BEFORE_ACT), np.maximum(base + rv, 0), atol=1e-13)
    assert np.allclose(fp8.conv_e4m3(xc, wc, scale, bias, 1, 1, nn.ACT_RELU, rc, 0.75, nn.RES_AFTER_ACT), np.maximum(base, 0) + rv, atol=1e-13)
    # what is stored: the fp32 product with the inverse scale, encoded
    assert np.array_equal(fp8.store_e4m3(np.float64([0.6, -1000.0, 3.0]), 0.5), np.uint8([0x2A, 0xFE, 0x3C]))
