"""Pins of the oracle's INT8 linear layer (Appendix A) against scalar loops, the identity weight, the adjoint
identities that tie forward and backward together, and finite differences of a scalar loss."""
import numpy as np

from oracle import qgalore as Q
from paper_2407_08296_amd import inputs as I


def _case(tokens, m, n, seed=0):
    g = np.random.default_rng(seed)
    Wq, Ws = Q.quant_int8(I.weight_f32(m, n, seed=seed))
    x = Q.f64_to_bf16_bits(g.standard_normal((tokens, n)))
    dy = Q.f64_to_bf16_bits(g.standard_normal((tokens, m)) * 0.1)
    return Wq, Ws, x, dy


def test_dequantized_weight_is_code_times_scale_in_bf16():
    Wq, Ws, _, _ = _case(1, 5, 700)
    Wd = Q.dequant_w_bf16(Wq, Ws)
    for (i, j) in [(0, 0), (2, 255), (2, 256), (4, 699)]:
        prod = np.float32(np.float32(Wq[i, j]) * Ws[i, j // 256])
        assert Wd[i, j] == Q.bf16_rne(np.float64(prod))
    assert np.array_equal(Q.f64_to_bf16_bits(Wd).astype(np.uint32) << 16, Wd.astype(np.float32).view(np.uint32))


def test_forward_and_backward_by_scalar_loops():
    tokens, m, n = 3, 4, 260
    Wq, Ws, xb, dyb = _case(tokens, m, n, seed=1)
    bias = Q.f64_to_bf16_bits(np.linspace(-1, 1, m))
    W = Q.dequant_w_bf16(Wq, Ws)
    x = Q.bf16_bits_to_f64(xb).reshape(tokens, n)
    dy = Q.bf16_bits_to_f64(dyb).reshape(tokens, m)
    b = Q.bf16_bits_to_f64(bias)
    y = Q.int8_linear_forward(xb, Wq, Ws, bias)
    dx, gW = Q.int8_linear_backward(dyb, xb, Wq, Ws)
    assert y.shape == (tokens, m) and dx.shape == (tokens, n) and gW.shape == (m, n)
    for t in range(tokens):
        for o in range(m):
            assert abs(y[t, o] - (sum(x[t, i] * W[o, i] for i in range(n)) + b[o])) < 1e-12
        for i in range(0, n, 37):
            assert abs(dx[t, i] - sum(dy[t, o] * W[o, i] for o in range(m))) < 1e-12
    for o in range(m):
        for i in range(0, n, 41):
            assert abs(gW[o, i] - sum(dy[t, o] * x[t, i] for t in range(tokens))) < 1e-12


def test_identity_weight_passes_activations_through():
    n = 64
    Wq = (np.eye(n, dtype=np.int8) * 127)
    Ws = np.full((n, 1), np.float32(1.0) / np.float32(127.0), dtype=np.float32)
    assert np.array_equal(Q.dequant_w_bf16(Wq, Ws), np.eye(n))       # fl32(127 * fl32(1/127)) = 1
    xb = Q.f64_to_bf16_bits(np.random.default_rng(2).standard_normal((5, n)))
    assert np.array_equal(Q.int8_linear_forward(xb, Wq, Ws), Q.bf16_bits_to_f64(xb).reshape(5, n))
    dx, _ = Q.int8_linear_backward(xb, xb, Wq, Ws)
    assert np.array_equal(dx, Q.bf16_bits_to_f64(xb).reshape(5, n))


def test_adjoint_identities():
    """<dy, x W^T> = <dy W, x> = <dy^T x, W>: a transposed or swapped operand in any of the three products breaks one."""
    tokens, m, n = 17, 24, 300
    Wq, Ws, xb, dyb = _case(tokens, m, n, seed=3)
    x = Q.bf16_bits_to_f64(xb).reshape(tokens, n)
    dy = Q.bf16_bits_to_f64(dyb).reshape(tokens, m)
    y = Q.int8_linear_forward(xb, Wq, Ws)
    dx, gW = Q.int8_linear_backward(dyb, xb, Wq, Ws)
    a = np.sum(dy * y)
    assert abs(a - np.sum(dx * x)) <= 1e-12 * abs(a) + 1e-12
    assert abs(a - np.sum(gW * Q.dequant_w_bf16(Wq, Ws))) <= 1e-12 * abs(a) + 1e-12


def test_backward_is_the_gradient_of_a_scalar_loss():
    """L = sum(C * forward(x)): dL/dx = C W and dL/dW = C^T x; the layer is bilinear, so central differences in
    fp64 are exact up to rounding."""
    tokens, m, n = 4, 6, 20
    g = np.random.default_rng(4)
    W = g.standard_normal((m, n))
    x = g.standard_normal((tokens, n))
    C = g.standard_normal((tokens, m))
    # the same formulas the oracle uses, on unquantized operands
    dx, gW = C @ W, C.T @ x
    h = 1e-3
    for (t, i) in [(0, 0), (3, 19), (2, 7)]:
        e = np.zeros_like(x); e[t, i] = h
        assert abs((np.sum(C * ((x + e) @ W.T)) - np.sum(C * ((x - e) @ W.T))) / (2 * h) - dx[t, i]) < 1e-9
    for (o, i) in [(0, 0), (5, 19), (3, 11)]:
        e = np.zeros_like(W); e[o, i] = h
        assert abs((np.sum(C * (x @ (W + e).T)) - np.sum(C * (x @ (W - e).T))) / (2 * h) - gW[o, i]) < 1e-9
    # and the oracle evaluates exactly these formulas on its dequantized weight
    Wq, Ws = Q.quant_int8(W.astype(np.float32))
    xb, Cb = Q.f64_to_bf16_bits(x), Q.f64_to_bf16_bits(C)
    odx, ogW = Q.int8_linear_backward(Cb, xb, Wq, Ws)
    Wd, xr, Cr = Q.dequant_w_bf16(Wq, Ws), Q.bf16_bits_to_f64(xb).reshape(tokens, n), Q.bf16_bits_to_f64(Cb).reshape(tokens, m)
    assert np.allclose(odx, Cr @ Wd, rtol=0, atol=1e-14) and np.allclose(ogW, Cr.T @ xr, rtol=0, atol=1e-14)
    assert np.abs(Wd - W).max() <= np.abs(W).max() * (1 / 127 + 2 ** -8)      # INT8 step + bf16 rounding
