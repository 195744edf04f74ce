"""The step on seeded random shapes: every edge class (whole tiles; ragged with 16-byte aligned rows; anything), tiny
matrices, r = m, short and wide ones, mixed in grouped plans of one to five matrices and one by one through the
single-matrix call, from a cold (t = 1) or a warm state, against the oracle at the bars of test_gpu_parity."""
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


def random_shape(rng):
    kind = rng.integers(0, 6)
    if kind == 0:     # whole tiles
        r = int(rng.choice([128, 256]))
        return max(int(rng.choice([128, 256, 384, 512, 640])), r), 256 * int(rng.integers(1, 5)), r
    if kind == 1:     # aligned rows, edges
        r = 16 * int(rng.integers(1, 17))
        return int(rng.integers(r, 700)), 8 * int(rng.integers(1, 120)), r
    if kind == 2:     # anything
        r = 8 * int(rng.integers(1, 33))
        return int(rng.integers(r, 700)), int(rng.integers(1, 900)), r
    if kind == 3:     # tiny
        r = 8 * int(rng.integers(1, 4))
        return int(rng.integers(r, 40)), int(rng.integers(1, 40)), r
    if kind == 4:     # r = m
        r = 8 * int(rng.integers(1, 33))
        return r, int(rng.integers(1, 600)), r
    r = 8 * int(rng.integers(1, 9))   # short and wide
    return int(rng.integers(r, 130)), int(rng.integers(256, 3000)), r


def check(s, o, t, what):
    assert rel_fro(host(s.R), o["R"]) <= 2e-5, what
    if t > 1:         # warm state: N is a smooth function of R
        N = Q.bf16_bits_to_f64(host(s.N.view(torch.int16)).view(np.uint16))
        assert rel_fro(N, o["Nb"]) <= 1e-3, what
    assert rel_fro(host(s.M), o["M"]) <= 2e-5 and rel_fro(host(s.V), o["V"]) <= 4e-5, what
    d = host(s.Wq).astype(np.int32) - o["Wq"].astype(np.int32)
    assert np.abs(d).max() <= 1, what
    assert np.mean(d != 0) <= max(1e-4, 2.0 / d.size), what         # a small matrix may hold one differing code
    assert np.all(np.abs(host(s.Ws).astype(np.float64) - o["Ws"]) <= 5e-4 * np.abs(o["Ws"])), what


@pytest.mark.parametrize("sweep", [11, 12, 13])
def test_random_shapes_grouped_and_single(sweep):
    rng = np.random.default_rng(sweep)
    for group in range(12):
        shapes = [random_shape(rng) for _ in range(int(rng.integers(1, 6)))]
        t, seed = int(rng.integers(1, 5)), int(rng.integers(0, 2 ** 62))
        print(f"sweep {sweep} group {group}: t = {t}, shapes {shapes}", flush=True)
        data, warm = [], []
        for li, (m, n, r) in enumerate(shapes):
            Wq, Ws = Q.quant_int8(I.weight_f32(m, n, 0, li, 0))
            Pq, Ps = Q.quant_int4(I.projection_f32(m, r, 0, li, 0))
            data.append(dict(Wq=Wq, Ws=Ws, Pq=Pq, Ps=Ps, Gb=I.gradient_bf16(m, n, t, 0, li, 0)))
            rs = np.random.default_rng([sweep, group, li])
            if t > 1:
                warm.append(((rs.standard_normal((r, n)) * 5e-5).astype(np.float32),
                             ((rs.standard_normal((r, n)) * 5e-5) ** 2 + 1e-12).astype(np.float32)))
            else:
                warm.append((np.zeros((r, n), np.float32), np.zeros((r, n), np.float32)))

        def state():
            return [qg.MatrixState(m, n, r, dev(d["Pq"]), dev(d["Ps"]), dev(d["Gb"]), dev(d["Wq"]), dev(d["Ws"]),
                                   dev(w[0]), dev(w[1]), torch.empty((r, n), dtype=torch.float32, device=DEV),
                                   torch.empty((r, n), dtype=torch.bfloat16, device=DEV))
                    for (m, n, r), d, w in zip(shapes, data, warm)]
        mats = state()
        qg.step_many(qg.StepPlan(mats), qg.hparams(), seed, t)
        singles = state()
        for s in singles:
            qg.step(s.Pq, s.Ps, s.G, s.Wq, s.Ws, s.M, s.V, s.R, s.N, s.m, s.n, s.r, qg.hparams(), seed, t)
        torch.cuda.synchronize()
        for i, (s, one, d, w) in enumerate(zip(mats, singles, data, warm)):
            o = Q.step(d["Wq"], d["Ws"], d["Gb"], d["Pq"], d["Ps"], w[0], w[1], t, HP,
                       seed=(seed + i * 0x9E3779B97F4A7C15) % 2 ** 64, r=s.r)
            check(s, o, t, f"grouped, matrix {i} {shapes[i]}")
            o1 = o if i == 0 else Q.step(d["Wq"], d["Ws"], d["Gb"], d["Pq"], d["Ps"], w[0], w[1], t, HP, seed=seed, r=s.r)
            check(one, o1, t, f"single, matrix {i} {shapes[i]}")
