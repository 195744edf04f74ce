"""The pieces in the order a training iteration uses them (Sec. 3.5, Fig. 3; Appendix A), on one small layer:

    forward of the INT8 linear layer  ->  loss gradient dy  ->  backward (grad_W = G)
    [every `interval` steps: subspace refresh from G, cosine check, interval policy (Sec. 3.2)]
    optimizer step: project, Adam, back-project, INT8 update with stochastic rounding

Every library call of an iteration starts from the ORACLE's state and inputs (teacher forcing: one differing INT8
code never heals), and each result is held to the bar of its own parity test.  The loop regresses the layer onto a
fixed teacher weight, so the oracle's loss must also go down: the pieces compose into something that trains.
"""
import numpy as np
import pytest
import torch

from oracle import qgalore as Q
from paper_2407_08296_amd import inputs as I
from paper_2407_08296_amd import qgalore as qg

pytestmark = pytest.mark.gpu
DEV = "cuda"


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def host(t):
    return t.detach().cpu().numpy()


def bits_t(bits, shape):
    return dev(np.ascontiguousarray(bits).view(np.int16).reshape(shape))


def bf16_host(t):
    return Q.bf16_bits_to_f64(host(t.view(torch.int16)).view(np.uint16)).reshape(tuple(t.shape))


def test_forward_backward_refresh_step_loop():
    tokens, m, n, r = 96, 384, 512, 64
    # lr and alpha large enough for the loss to move in a dozen steps; everything else the paper's defaults
    hp_o = Q.HParams(lr=2e-2, alpha=0.25)
    hp_g = qg.hparams(lr=2e-2, alpha=0.25)
    g = np.random.default_rng(0)
    W_teacher = I.weight_f32(m, n, seed=7).astype(np.float64)
    Wq, Ws = Q.quant_int8(I.weight_f32(m, n, seed=8))
    Pq, Ps = Q.quant_int4(I.projection_f32(m, r))
    M = np.zeros((r, n), np.float32)
    V = np.zeros((r, n), np.float32)
    pol_g = qg.Policy(4, 0, 1, 1, 0.4, 0.0)
    pol_o = Q.Policy(interval=4, k=1, threshold=0.4, next_refresh=1)
    losses, refreshes = [], 0
    for t in range(1, 14):
        xb = Q.f64_to_bf16_bits(g.standard_normal((tokens, n)))
        x = Q.bf16_bits_to_f64(xb).reshape(tokens, n)
        target = x @ W_teacher.T
        xd, Wqd, Wsd = bits_t(xb, (tokens, n)), dev(Wq), dev(Ws)

        # forward
        oy = Q.int8_linear_forward(xb, Wq, Ws)
        gy = bf16_host(qg.int8_linear_forward(xd, Wqd, Wsd))
        assert np.all(np.abs(gy - oy) <= 2.0 ** -8 * np.abs(oy) + 1e-5)
        yb = Q.bf16_rne(oy)                                   # the activation as the layer stores it
        losses.append(0.5 * np.mean(np.sum((yb - target) ** 2, axis=1)))
        dyb = Q.f64_to_bf16_bits((yb - target) / tokens)

        # backward
        odx, oG = Q.int8_linear_backward(dyb, xb, Wq, Ws)
        gdx, gG = qg.int8_linear_backward(bits_t(dyb, (tokens, m)), xd, Wqd, Wsd, m, n)
        for got, want in ((bf16_host(gdx), odx), (bf16_host(gG), oG)):
            assert np.all(np.abs(got - want) <= 2.0 ** -8 * np.abs(want) + 1e-7)
            assert np.mean(got == Q.bf16_rne(want)) >= 0.99
        Gb = Q.f64_to_bf16_bits(oG)                           # the gradient as stored, from the oracle
        Gd = bits_t(Gb, (m, n))

        # subspace refresh when due (the first one at step 1, as GaLore does)
        if t == pol_o.next_refresh:
            oPq, oPs, ocos = Q.subspace_refresh_check(Pq, Ps, Gb, m, n, r, iters=1)
            gPq, gPs, gcos, ginfo, _ = qg.subspace_refresh(dev(Pq), dev(Ps), Gd, m, n, r, 1)
            assert int(host(ginfo)[0]) == 0
            assert abs(float(host(gcos)[0]) - ocos) <= 2e-3
            e_g = np.linalg.norm(Q.project(host(gPq), host(gPs), Gb, m, n, r)) ** 2
            e_o = np.linalg.norm(Q.project(oPq, oPs, Gb, m, n, r)) ** 2
            assert abs(e_g - e_o) <= 1e-3 * e_o
            doubled_o = pol_o.update(float(np.float32(ocos)))
            doubled_g = qg.policy_update(pol_g, float(host(gcos)[0]))
            if abs(ocos - 0.4) > 5e-3:                        # away from the threshold the decisions agree
                assert doubled_g == doubled_o and pol_g.next_refresh == pol_o.next_refresh
            else:
                pol_g.interval, pol_g.streak, pol_g.next_refresh = pol_o.interval, pol_o.streak, pol_o.next_refresh
            Pq, Ps = oPq, oPs
            refreshes += 1

        # optimizer step (the fused two-launch form)
        o = Q.step(Wq, Ws, Gb, Pq, Ps, M, V, t, hp_o, seed=3, r=r)
        dWq, dWs, dM, dV = dev(Wq), dev(Ws), dev(M), dev(V)
        dN = torch.empty((r, n), dtype=torch.bfloat16, device=DEV)
        qg.step(dev(Pq), dev(Ps), Gd, dWq, dWs, dM, dV, None, dN, m, n, r, hp_g, 3, t)
        d = host(dWq).astype(np.int32) - o["Wq"].astype(np.int32)
        assert np.abs(d).max() <= 1 and np.mean(d == 0) >= (0.99 if t == 1 else 0.9999), (t, np.mean(d == 0))
        assert np.allclose(host(dM), o["M"], rtol=0, atol=2e-5 * np.abs(o["M"]).max())
        Wq, Ws, M, V = o["Wq"], o["Ws"], o["M"].astype(np.float32), o["V"].astype(np.float32)
    assert refreshes >= 2
    assert losses[-1] < 0.9 * losses[0], losses
