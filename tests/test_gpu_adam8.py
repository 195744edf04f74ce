"""GPU parity of the 8-bit Adam states against the CPU oracle.

Bars: the quantizer on given fp32 input is bit-exact (codes and scales: the same fp32 decisions on both sides);
the dequantizer is bit-exact; after an Adam step the library's fp32 moments differ from the oracle's fp64 ones by
an ulp or so before they are quantized, so a value that sits on a table midpoint may take the neighbouring code:
>= 99.99 % of the codes identical and none further than one entry away; scales within 1e-6 relative; N within 1e-3
relative Frobenius (the bar of the fp32-state path).
"""
import numpy as np
import pytest
import torch

from oracle import qgalore as Q
from paper_2407_08296_amd import qgalore as qg

pytestmark = pytest.mark.gpu
DEV = "cuda"
HP = Q.HParams()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def host(t):
    return t.detach().cpu().numpy()


@pytest.mark.parametrize("count", [256, 1000, 4, 128 * 521, 1024 * 4096])
@pytest.mark.parametrize("signed", [True, False])
def test_state8_quant_and_dequant_bit_exact(count, signed):
    g = np.random.default_rng([count, int(signed)])
    x = (g.standard_normal(count) * np.exp(g.uniform(-12, 2, count))).astype(np.float32)   # many decades
    if not signed:
        x = np.abs(x)
    if count >= 1000:
        x[256:512] = 0.0                                         # an all-zero block
        x[700] = np.float32(Q._state8_mids(Q.state8_table(signed))[150]) * np.abs(x[512:768]).max()
    codes, scales = qg.state8_quant(dev(x), signed)
    oc, os_ = Q.state8_quant(x, signed)
    assert np.array_equal(host(scales), os_)
    assert np.array_equal(host(codes), oc)
    back = qg.state8_dequant(codes, scales, signed)
    assert np.array_equal(host(back).astype(np.float64), Q.state8_dequant(oc, os_, signed))


@pytest.mark.parametrize("r,n", [(128, 512), (144, 264), (48, 521), (1024, 4096)])
def test_lowrank_adam8_steps(r, n):
    """Three steps, teacher-forced from the oracle's states (a differing code would otherwise propagate)."""
    g = np.random.default_rng([r, n])
    count = r * n
    Mq, Ms = Q.state8_quant(np.zeros(count), True)
    Vq, Vs = Q.state8_quant(np.zeros(count), False)
    hp = qg.hparams()
    for t in (1, 2, 3):
        R = (g.standard_normal((r, n)) * np.exp(g.uniform(-6, 0, (r, n))) * 1e-2).astype(np.float32)
        dMq, dMs, dVq, dVs = dev(Mq), dev(Ms), dev(Vq), dev(Vs)
        N = torch.empty((r, n), dtype=torch.bfloat16, device=DEV)
        qg.lowrank_adam8(dev(R), dMq, dMs, dVq, dVs, N, t, hp)
        Mq, Ms, Vq, Vs, oN, _, _ = Q.lowrank_adam8(R, Mq, Ms, Vq, Vs, t, HP)
        for got, want in ((host(dMq), Mq), (host(dVq), Vq)):
            d = got.astype(np.int32) - want.astype(np.int32)
            assert np.abs(d).max() <= 1 and np.mean(d == 0) >= 0.9999, (np.abs(d).max(), np.mean(d == 0))
        assert np.allclose(host(dMs), Ms, rtol=1e-6, atol=0) and np.allclose(host(dVs), Vs, rtol=1e-6, atol=0)
        gN = Q.bf16_bits_to_f64(host(N.view(torch.int16)).view(np.uint16)).reshape(r, n)
        oNb = Q.bf16_rne(oN)
        if t == 1:
            # from zero states N = R / (|R| + eps): compare where |R| is well above eps = 1e-8 (see the fp32 path)
            far = np.abs(R) > 1e-6
            assert np.linalg.norm((gN - oNb)[far]) <= 1e-3 * np.linalg.norm(oNb[far])
        else:
            assert np.linalg.norm(gN - oNb) <= 1e-3 * np.linalg.norm(oNb)
