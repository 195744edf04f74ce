"""Pins of the oracle's 8-bit Adam states (Sec. 3.5 names an 8-bit Adam as the inner optimizer; the format is this
build's design): table structure, nearest-entry quantization by brute force, the error bound of the data type, and
the behaviour of Adam under it."""
import numpy as np

from oracle import qgalore as Q


def test_table_structure():
    u, s = Q.state8_table(False).astype(np.float64), Q.state8_table(True).astype(np.float64)
    assert u.size == 256 and s.size == 255
    assert np.all(np.diff(u) > 0) and np.all(np.diff(s) > 0)
    assert u[0] == 0 and u[-1] == 1 and np.isclose(u[1], 1e-7) and s[127] == 0 and s[0] == -1 and s[-1] == 1
    assert np.array_equal(s, -s[::-1]) and np.isclose(s[128], 1e-6)
    # 2^L entries spaced linearly over each decade, the last one on the decade's top
    for L in range(8):
        lvl = u[2 ** L: 2 ** (L + 1)]
        top = 10.0 ** -(7 - L)
        assert np.isclose(lvl[-1], top, rtol=1e-6) and lvl[0] > top / 10
        if L > 0:
            assert np.allclose(np.diff(lvl), 0.9 * top / 2 ** L, rtol=1e-4)
    # fraction bits: the relative step never exceeds 0.9 / (0.1 * 2^L + 0.9) of the value inside a level
    assert np.max(np.diff(u[128:]) / u[128:-1]) < 0.07


def test_quantization_is_nearest_entry_with_ties_down():
    g = np.random.default_rng(0)
    for signed in (True, False):
        tab = Q.state8_table(signed).astype(np.float64)
        x = g.standard_normal(256) * np.logspace(0, -8, 256)
        if not signed:
            x = np.abs(x)
        codes, scales = Q.state8_quant(x, signed)
        a = np.float32(np.abs(x.astype(np.float32)).max())
        assert scales.shape == (1,) and scales[0] == a
        xn = (x.astype(np.float32) * (np.float32(1) / a)).astype(np.float64)
        first_mid = 0.5 * (tab[0] + tab[1])
        for i in range(256):                                        # brute force over the whole table
            if not signed and 0 < xn[i] <= first_mid:
                assert codes[i] == 1                                # a positive second moment never rounds to zero
                continue
            d = np.abs(tab - xn[i])
            assert d[codes[i]] <= d.min() * (1 + 1e-6) + 1e-12
        # a value exactly on a midpoint goes to the lower entry
        mid = Q._state8_mids(Q.state8_table(signed))
        y = np.concatenate([[1.0], mid[[3, 100, 200]].astype(np.float64)])
        if not signed:
            y = np.abs(y)
        c2, _ = Q.state8_quant(np.pad(y, (0, 252)), signed)
        want = np.searchsorted(mid, y.astype(np.float32), side="left")
        assert np.array_equal(c2[:4], want) and np.all(tab[c2[1:4]] <= y[1:4])


def test_round_trip_error_bound_and_blocks():
    g = np.random.default_rng(1)
    x = g.standard_normal(1000) * 3.0
    x[256:512] = 0.0                                                # an all-zero block
    for signed, data in ((True, x), (False, x * x)):
        codes, scales = Q.state8_quant(data, signed)
        assert scales.size == 4 and scales[1] == 0 and np.all(codes[256:512] == (127 if signed else 0))
        back = Q.state8_dequant(codes, scales, signed)
        top = 6 if signed else 7
        for b in (0, 2, 3):
            sl = slice(b * 256, min((b + 1) * 256, 1000))
            a = float(scales[b])
            mag = np.abs(data[sl]) / a
            # level of each value: decade (10^-(E+1), 10^-E]; the step there is 0.9 * 10^-E / 2^(top-E)
            E = np.clip(np.floor(-np.log10(np.maximum(mag, 1e-30)) + 1e-12), 0, top)
            step = 0.9 * 10.0 ** -E / 2.0 ** (top - E)
            small = mag < 10.0 ** -top
            bound = np.where(small, 10.0 ** -top, 0.5 * step * 1.0001) * a + 1e-6 * a
            assert np.all(np.abs(back[sl] - data[sl]) <= bound)
    assert np.array_equal(Q.state8_quant(back, False)[0], codes)      # a representable state is a fixed point


def test_adam_with_8bit_states_tracks_fp_adam_and_saturates():
    """Constant gradient: the bias-corrected direction is 1 from the first step and stays there; against Adam with
    exact states the 8-bit run stays within the data type's resolution."""
    hp = Q.HParams()
    g = np.random.default_rng(2)
    R = g.standard_normal((4, 128)) * 0.01
    Mq, Ms = Q.state8_quant(np.zeros(R.size), True)
    Vq, Vs = Q.state8_quant(np.zeros(R.size), False)
    M = np.zeros_like(R); V = np.zeros_like(R)
    for t in range(1, 40):
        Mq, Ms, Vq, Vs, N8, M8, V8 = Q.lowrank_adam8(R, Mq, Ms, Vq, Vs, t, hp)
        M, V, N = Q.lowrank_adam(R, M, V, t, hp)
        assert np.abs(N8 - N).max() < 0.15
    big = np.abs(R) > 1e-3
    assert np.allclose(np.abs(N8[big]), 1.0, atol=0.15) and np.array_equal(np.sign(N8[big]), np.sign(R[big]))
    assert np.abs(Q.state8_dequant(Mq, Ms, True).reshape(R.shape) - M)[big].max() <= 0.05 * np.abs(M).max()
    # one step is exactly: dequantize, exact Adam, quantize
    Mq2, Ms2, Vq2, Vs2, N2, M2, V2 = Q.lowrank_adam8(R, Mq, Ms, Vq, Vs, 40, hp)
    Md, Vd = Q.state8_dequant(Mq, Ms, True).reshape(R.shape), Q.state8_dequant(Vq, Vs, False).reshape(R.shape)
    b1, b2 = float(np.float32(0.9)), float(np.float32(0.999))
    assert np.allclose(M2, b1 * Md + (1 - b1) * R, rtol=1e-15) and np.allclose(V2, b2 * Vd + (1 - b2) * R * R, rtol=1e-15)
    assert np.array_equal(Q.state8_quant(M2, True)[0], Mq2)


def test_midpoints_are_wider_apart_than_float_buckets_of_15_bits():
    """A property of the format the library's encoder builds on: cut the positive floats by their top 15 bits (8
    exponent + 7 mantissa bits); between the first midpoint and 1 no such bucket holds more than one midpoint of the
    unsigned table or of the positive half of the signed one, so a value's code is the count of midpoints below its
    bucket's lower edge plus at most one."""
    for signed in (False, True):
        tab = Q.state8_table(signed).astype(np.float32)
        mids = np.asarray(Q._state8_mids(tab), dtype=np.float32)
        pm = mids[127:254] if signed else mids[:255]
        assert np.all(np.diff(pm) > 0) and pm[0] > 0
        k0 = int(np.float32(pm[0]).view(np.uint32)) >> 16
        k1 = int(np.float32(1.0).view(np.uint32)) >> 16
        edges = (np.arange(k0, k1 + 2, dtype=np.uint32) << np.uint32(16)).view(np.float32)
        below = np.searchsorted(pm, edges, side="left")
        assert np.diff(below).max() == 1
        assert (k0, k1) == ((13574, 16256) if signed else (13142, 16256))


def test_a_persistently_small_gradient_keeps_a_bounded_direction():
    """An element whose gradient stays far below its block's largest (between the floors of the two tables: its
    first moment survives quantization, its second moment would round to zero) over 60 steps: Adam's direction for
    it must stay of order one.  With V flushed to zero every step the quotient would come from the newest gradient
    alone, m / sqrt((1 - beta2) g^2) ~ 30 at large t; storing a positive V at the smallest positive entry instead
    bounds it (and errs towards the smaller step)."""
    hp = Q.HParams()
    R = np.full(256, 1e-2)
    small = [3, 100, 200]
    R[small] = [1e-2 * 1e-4, -1e-2 * 3e-5, 1e-2 * 5e-6]           # 1e-4, 3e-5, 5e-6 of the block maximum
    Mq, Ms = Q.state8_quant(np.zeros(256), True)
    Vq, Vs = Q.state8_quant(np.zeros(256), False)
    worst = 0.0
    for t in range(1, 61):
        Mq, Ms, Vq, Vs, N, M1, V1 = Q.lowrank_adam8(R, Mq, Ms, Vq, Vs, t, hp)
        worst = max(worst, float(np.abs(N[small]).max()))
        assert np.all(Vq[small] >= 1)                               # never flushed
        assert np.allclose(N[[0, 1, 2]], 1.0, atol=0.1)             # the ordinary elements: direction 1
    assert worst <= 1.5, worst
    assert np.all(Mq[small] != 127)                                 # their first moments did survive
    # the format rule itself: any positive value takes code >= 1, zero keeps code 0, nearest-entry otherwise
    x = np.zeros(256); x[0] = 1.0; x[1] = 1e-9; x[2] = 4e-8; x[3] = 6e-8; x[4] = 1.4e-7
    c, _ = Q.state8_quant(x, False)
    assert list(c[:6]) == [255, 1, 1, 1, 1, 0]
