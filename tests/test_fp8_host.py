"""The library's host-side E4M3 conversion and weight packing against the oracle (no GPU)."""
import numpy as np
import pytest

from oracle import fp8
from paper_2502_01277_amd import binding

ALL = np.arange(256, dtype=np.uint8)


def test_library_host_conversion_is_the_oracles():
    rng = np.random.default_rng(11)
    x = np.concatenate([rng.standard_normal(200000).astype(np.float32) * s for s in (1e-3, 0.02, 1.0, 30.0, 300.0)] +
                       [np.float32([0.0, -0.0, 448, 449, 464, 465, 1e30, -1e30, np.inf, -np.inf, np.nan, 2.0 ** -10, 1.5 * 2.0 ** -9, 7.5 * 2.0 ** -9])])
    for inv in (1.0, 0.37, 16.0):
        ref = fp8.e4m3_encode(x * np.float32(inv))
        assert np.array_equal(binding.quantize_e4m3(x, inv), ref)
    v = fp8.e4m3_decode(ALL)
    pos = v[:0x7F]
    mids = ((pos[:-1] + pos[1:]) / 2).astype(np.float32)
    assert np.array_equal(binding.quantize_e4m3(mids), fp8.e4m3_encode(mids))
    got = binding.dequantize_e4m3(ALL, 0.5)
    assert np.array_equal(np.isnan(got), np.isnan(v)) and np.array_equal(got[~np.isnan(v)], (v[~np.isnan(v)] * 0.5).astype(np.float32))


@pytest.mark.parametrize("dtype,es,kstep", [("f8", 1, 128), ("bf16", 2, 64), ("f32", 4, 32)])
def test_weight_packing_layout(dtype, es, kstep):
    rng = np.random.default_rng(2)
    cout, kh, kw, cin = 70, 3, 3, 16
    raw = rng.integers(1, 255, (cout, kh, kw, cin * es)).astype(np.uint8)            # any bytes: packing only moves them
    packed = binding.conv_pack(raw.reshape(cout, kh, kw, cin, es).view({1: np.uint8, 2: np.uint16, 4: np.float32}[es]).reshape(cout, kh, kw, cin), dtype)
    k = kh * kw * cin
    kp = (k + kstep - 1) // kstep * kstep
    rows = binding.lib().octo_op_conv_padded_cout(cout)
    assert rows == 128 and packed.size == rows * kp * es + 512
    m = packed[:rows * kp * es].reshape(rows, kp * es)
    assert np.array_equal(m[:cout, :k * es], raw.reshape(cout, k * es))
    assert not m[:cout, k * es:].any() and not m[cout:].any() and not packed[rows * kp * es:].any()
