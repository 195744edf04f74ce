"""The step at the edge of its documented size range: m * n just below 2^32 (the element index of the stochastic
rounding stream and the 32-bit offsets of the kernels' buffer loads end there), and the smallest shapes the calls
accept.  The large case is generated on the device (4.3e9 elements: 8.6 GB of gradient, 4.3 GB of codes); the oracle
recomputes whole column blocks from what the device holds, the step being column-separable (Sec. 3.5)."""
import numpy as np
import pytest
import torch

from oracle import qgalore as Q
from paper_2407_08296_amd import inputs as I
from paper_2407_08296_amd import qgalore as qg

pytestmark = pytest.mark.gpu
HP = Q.HParams()
DEV = "cuda"


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def host(t):
    return t.detach().cpu().numpy()


def rel_fro(a, b):
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(np.asarray(a, dtype=np.float64) - b) / max(np.linalg.norm(b), 1e-300))


def bits(t):
    return host(t.contiguous().view(torch.int16)).view(np.uint16)


def test_step_just_below_the_index_limit():
    """m * n = 2^32 - 2^23: every row and column block exists, the last element's index is 2^32 - 2^23 - 1.  Warm
    moments, t = 3; first, middle and last column block against the oracle, all 32768 rows of each."""
    m, n, r, t, seed = 32768, 130816, 128, 3, 0x1234_5678_9ABC_DEF0
    assert m * n < 2 ** 32 and (m + 128) * n >= 2 ** 32
    gen = torch.Generator(device=DEV); gen.manual_seed(5)
    Pq_h, Ps_h = Q.quant_int4(I.projection_f32(m, r))
    Pq, Ps = dev(Pq_h), dev(Ps_h)
    G = torch.empty((m, n), dtype=torch.bfloat16, device=DEV)
    Wq = torch.empty((m, n), dtype=torch.int8, device=DEV)
    Ws = torch.empty((m, n // 256), dtype=torch.float32, device=DEV)
    A = torch.randn((m, 16), generator=gen, device=DEV) * 0.01
    B = torch.randn((n, 16), generator=gen, device=DEV) * 0.01
    rows = 2048
    for i in range(0, m, rows):                       # in row chunks: the fp32 temporaries stay at 1 GB
        g = torch.randn((rows, n), generator=gen, device=DEV) * 1e-4
        g.addmm_(A[i:i + rows], B.t())
        G[i:i + rows] = g.to(torch.bfloat16)
        q, s = qg.quant_int8(torch.randn((rows, n), generator=gen, device=DEV) * 0.02)
        Wq[i:i + rows], Ws[i:i + rows] = q, s
        del g, q, s
    M = torch.randn((r, n), generator=gen, device=DEV) * 5e-5
    V = (torch.randn((r, n), generator=gen, device=DEV) * 5e-5) ** 2 + 1e-12
    ng = n // 256
    blocks = sorted({0, ng // 2, ng - 1})
    before = {}
    for g in blocks:                                  # the oracle's inputs: what the device holds before the step
        sl = slice(g * 256, (g + 1) * 256)
        before[g] = dict(G=bits(G[:, sl]), Wq=host(Wq[:, sl].contiguous()), Ws=host(Ws[:, g:g + 1].contiguous()),
                         M=host(M[:, sl].contiguous()), V=host(V[:, sl].contiguous()))
    R = torch.empty((r, n), dtype=torch.float32, device=DEV)
    N = torch.empty((r, n), dtype=torch.bfloat16, device=DEV)
    s = qg.MatrixState(m, n, r, Pq, Ps, G, Wq, Ws, M, V, R, N)
    print("launching the grouped step on", m, "x", n, flush=True)
    qg.step_many(qg.StepPlan([s]), qg.hparams(), seed, t)
    torch.cuda.synchronize()
    for g in blocks:
        sl = slice(g * 256, (g + 1) * 256)
        b = before[g]
        o = Q.step(b["Wq"], b["Ws"], b["G"], Pq_h, Ps_h, b["M"], b["V"], t, HP, seed=seed, r=r, n_total=n, col0=g * 256)
        eR = rel_fro(host(R[:, sl]), o["R"])
        eN = rel_fro(Q.bf16_bits_to_f64(bits(N[:, sl])), Q.bf16_rne(o["N"]))
        assert eR <= 1e-4 and eN <= 1e-3, (g, eR, eN)          # K = 32768 terms accumulated in fp32
        assert rel_fro(host(M[:, sl]), o["M"]) <= 1e-4 and rel_fro(host(V[:, sl]), o["V"]) <= 2e-4
        d = host(Wq[:, sl].contiguous()).astype(np.int32) - o["Wq"].astype(np.int32)
        assert np.abs(d).max() <= 1
        same = float(np.mean(d == 0))
        assert same >= 0.9999, (g, same)
        sg, so = host(Ws[:, g:g + 1].contiguous()).astype(np.float64), o["Ws"].astype(np.float64)
        assert np.all(np.abs(sg - so) <= 5e-4 * np.abs(so))
        print(f"block {g}: R {eR:.2e} N {eN:.2e} identical codes {same:.6f}", flush=True)


@pytest.mark.parametrize("m,n,r", [(8, 8, 8), (8, 1, 8), (9, 257, 8), (256, 256, 256)])
def test_smallest_shapes(m, n, r):
    """The smallest shapes the step accepts (r a multiple of 8, r <= m; any n >= 1), r = m included: one workgroup,
    mostly padding."""
    t, seed = 2, 3
    Wq, Ws = Q.quant_int8(I.weight_f32(m, n))
    Pq, Ps = Q.quant_int4(I.projection_f32(m, r))
    Gb = I.gradient_bf16(m, n, t)
    rs = np.random.default_rng(1)
    M0 = (rs.standard_normal((r, n)) * 5e-5).astype(np.float32)
    V0 = ((rs.standard_normal((r, n)) * 5e-5) ** 2 + 1e-12).astype(np.float32)
    o = Q.step(Wq, Ws, Gb, Pq, Ps, M0, V0, t, HP, seed=seed, r=r)
    dWq, dWs, dM, dV = dev(Wq), dev(Ws), dev(M0), dev(V0)
    dR = torch.empty((r, n), dtype=torch.float32, device=DEV)
    dN = torch.empty((r, n), dtype=torch.bfloat16, device=DEV)
    qg.step(dev(Pq), dev(Ps), dev(Gb), dWq, dWs, dM, dV, dR, dN, m, n, r, qg.hparams(), seed, t)
    torch.cuda.synchronize()
    assert rel_fro(host(dR), o["R"]) <= 2e-5
    assert rel_fro(host(dM), o["M"]) <= 2e-5 and rel_fro(host(dV), o["V"]) <= 4e-5
    d = host(dWq).astype(np.int32) - o["Wq"].astype(np.int32)
    assert np.abs(d).max() <= 1 and np.mean(d != 0) <= 1e-2      # few elements: one differing code is a large share
    assert np.allclose(host(dWs), o["Ws"], rtol=1e-5, atol=0)
