"""Pins of the oracle's number formats: bf16 rounding, block quantizers, nibble packing.

Citations: Sec. 3.1 (Quant_n equation, block size 256, BFloat16 gradients), Sec. 3.3 (INT4 projection).
"""
import numpy as np
import pytest
import torch

from oracle import qgalore as Q
from oracle import brute


def test_bf16_all_patterns_round_trip():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    vals = Q.bf16_bits_to_f64(bits)
    finite = np.isfinite(vals)
    assert np.array_equal(Q.bf16_rne(vals[finite]), vals[finite])
    assert np.array_equal(Q.f64_to_bf16_bits(vals[finite]), bits[finite])


def test_bf16_matches_library_cast_on_fp32_inputs():
    rs = np.random.default_rng(1)
    x = np.concatenate([
        rs.standard_normal(200000).astype(np.float32),
        (rs.standard_normal(50000) * 1e-30).astype(np.float32),
        (rs.standard_normal(50000) * 1e30).astype(np.float32),
        (rs.standard_normal(20000) * 1e-39).astype(np.float32),     # bf16 subnormals
    ])
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(Q.bf16_rne(x.astype(np.float64)), want)


def test_bf16_ties_to_even_and_single_rounding():
    # 1 + 2^-8 is halfway between 1 and 1+2^-7: goes to the even mantissa (1.0)
    assert Q.bf16_rne(np.array([1.0 + 2.0 ** -8]))[0] == 1.0
    # 1 + 3*2^-8 is halfway between 1+2^-7 and 1+2^-6: goes to even (1+2^-6)
    assert Q.bf16_rne(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6
    # just above the tie (not representable in fp32): a double rounding through fp32 would give 1.0
    assert Q.bf16_rne(np.array([1.0 + 2.0 ** -8 + 2.0 ** -40]))[0] == 1.0 + 2.0 ** -7
    # brute-force helper agrees
    rs = np.random.default_rng(2)
    for v in rs.standard_normal(2000) * 10.0 ** rs.integers(-6, 6, 2000):
        assert brute.bf16(float(v)) == Q.bf16_rne(np.array([v]))[0]


@pytest.mark.parametrize("bits", [4, 8])
def test_quant_round_trip_error_bound(bits):
    # |dequant(quant(x)) - x| <= s/2 up to the fp32 rounding of the scaled value
    rs = np.random.default_rng(3)
    x = (rs.standard_normal((64, 700)) * 0.02).astype(np.float32)
    if bits == 8:
        q, s = Q.quant_int8(x)
        d = Q.dequant_int8(q, s)
        sfull = np.repeat(s.astype(np.float64), 256, axis=1)[:, :700]
    else:
        x = x[:, :512]
        pk, s = Q.quant_int4(x)
        d = Q.dequant_int4(pk, s, 64, 512)
        sfull = np.repeat(s.astype(np.float64), 256).reshape(64, 512)
    err = np.abs(d - x.astype(np.float64))
    slack = 1.0 + Q.QMAX[bits] * 2.0 ** -21
    assert np.all(err <= 0.5 * sfull * slack)
    # and the error is not trivially small: a wrong rounding mode (floor) would exceed s/2
    assert err.max() > 0.45 * sfull.max() * 0.5


@pytest.mark.parametrize("bits", [4, 8])
def test_quant_absmax_maps_to_qmax(bits):
    rs = np.random.default_rng(4)
    x = rs.standard_normal((8, 512)).astype(np.float32)
    qmax = Q.QMAX[bits]
    if bits == 8:
        q, s = Q.quant_int8(x)
        blocks = q.reshape(8, 2, 256)
        xb = x.reshape(8, 2, 256)
    else:
        q, s = Q.quant_int4_codes(x)
        blocks = q.reshape(16, 256)[:, None, :]
        xb = x.reshape(16, 256)[:, None, :]
    am = np.argmax(np.abs(xb), axis=-1)
    top = np.take_along_axis(blocks, am[..., None], axis=-1)[..., 0]
    sign = np.sign(np.take_along_axis(xb, am[..., None], axis=-1)[..., 0])
    assert np.array_equal(top, (sign * qmax).astype(np.int8))
    assert np.abs(q).max() == qmax          # symmetric: -qmax-1 is never produced


def test_quant_special_blocks():
    x = np.zeros((3, 512), dtype=np.float32)
    x[1, :256] = 0.5                 # constant block
    x[2, 300] = -3.0                 # a single non-zero in the second block
    q, s = Q.quant_int8(x)
    assert np.all(q[0] == 0) and np.all(s[0] == 0)                       # zero block: s = 0, codes 0
    assert np.all(q[1, :256] == 127) and s[1, 0] == np.float32(0.5 / 127)
    assert q[2, 300] == -127 and np.count_nonzero(q[2]) == 1
    assert np.all(Q.dequant_int8(q, s)[0] == 0)
    c4, s4 = Q.quant_int4_codes(x)
    assert np.all(c4[0] == 0) and c4[2, 300] == -7 and np.all(c4[1, :256] == 7)
    assert s4.shape == (6,) and s4[0] == 0


@pytest.mark.parametrize("bits", [4, 8])
def test_quant_idempotent(bits):
    rs = np.random.default_rng(5)
    x = (rs.standard_normal((16, 512)) * 0.02).astype(np.float32)
    if bits == 8:
        q, s = Q.quant_int8(x)
        q2, s2 = Q.quant_int8(Q.dequant_int8(q, s).astype(np.float32))
    else:
        q, s = Q.quant_int4_codes(x)
        d = Q.dequant_int4(Q.pack_int4(q), s, 16, 512).astype(np.float32)
        q2, s2 = Q.quant_int4_codes(d)
    assert np.array_equal(q, q2)
    assert np.all(np.abs(s2.astype(np.float64) - s) <= np.spacing(s))


def test_quant_short_last_block():
    rs = np.random.default_rng(6)
    x = rs.standard_normal((4, 300)).astype(np.float32)
    q, s = Q.quant_int8(x)
    assert s.shape == (4, 2)
    assert np.array_equal(s[:, 1], (np.abs(x[:, 256:]).max(axis=1).astype(np.float64) / 127).astype(np.float32))
    y = rs.standard_normal((3, 100)).astype(np.float32)          # 300 elements: one full + one short flat block
    c, s4 = Q.quant_int4_codes(y)
    assert s4.shape == (2,)
    assert s4[1] == np.float32(np.abs(y.reshape(-1)[256:]).max().astype(np.float64) / 7)


def test_quant_matches_python_loops():
    rs = np.random.default_rng(7)
    x = (rs.standard_normal((3, 300)) * 0.02).astype(np.float32)
    q, s = Q.quant_int8(x)
    bq, bs = brute.quant_int8_rows(x.tolist())
    assert q.tolist() == bq
    assert [[float(v) for v in row] for row in s] == bs
    c, s4 = Q.quant_int4_codes(x)
    bc, bs4 = brute.quant_int4_flat(x.tolist())
    assert c.tolist() == bc and [float(v) for v in s4] == bs4


def test_int4_pack_all_pairs():
    codes = np.array([(a, b) for a in range(-7, 8) for b in range(-7, 8)], dtype=np.int8).reshape(-1)
    pk = Q.pack_int4(codes)
    assert pk.size == codes.size // 2
    assert np.array_equal(Q.unpack_int4(pk, codes.size), codes)
    # layout: even flat element in the low nibble, stored nibble = code + 8
    assert Q.pack_int4(np.array([-7, 7], dtype=np.int8))[0] == (1 | (15 << 4))
    assert Q.pack_int4(np.array([3], dtype=np.int8))[0] == (11 | (8 << 4))
    with pytest.raises(ValueError):
        Q.pack_int4(np.array([9]))
