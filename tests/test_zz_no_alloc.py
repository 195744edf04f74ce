"""The entry point that allocates nothing (qg_subspace_cossim_static, scratch in a device array of the library image)
against the workspace-taking qg_subspace_cossim it is a variant of: same kernels, so the results must be bit-identical;
two calls in a row, the second on a smaller input (the array keeps the first call's contents)."""
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


def test_static_scratch_cossim_two_calls_second_smaller():
    out = torch.full((1,), float("nan"), dtype=torch.float32, device=DEV)   # the caller's output, allocated up front
    for (m, r) in [(11008, 1024), (768, 256), (300, 40)]:
        P = I.projection_f32(m, r)
        pa = Q.quant_int4(P)
        pb = Q.quant_int4(I.perturbed_projection_f32(P, 0.05))
        dA, dB = (dev(pa[0]), dev(pa[1])), (dev(pb[0]), dev(pb[1]))
        want = qg.subspace_cossim(dA[0], dA[1], dB[0], dB[1], m, r)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        qg.subspace_cossim_static(dA[0], dA[1], dB[0], dB[1], m, r, out)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        got = out.cpu().numpy()[0]
        assert got == want.cpu().numpy()[0], (m, r, got, want)
        assert abs(float(got) - Q.subspace_cossim(pa[0], pa[1], pb[0], pb[1], m, r)) <= 1e-5


def test_static_scratch_cossim_rejects_sizes_beyond_the_array():
    m, r = 65536, 2048      # ceil(m/64) * 3 * r floats = 24 MiB > 4 MiB
    z = torch.zeros((m * r // 2,), dtype=torch.uint8, device=DEV)
    s = torch.zeros((m * r // 256,), dtype=torch.float32, device=DEV)
    out = torch.zeros((1,), dtype=torch.float32, device=DEV)
    with pytest.raises(qg.QGError, match="workspace"):
        qg.subspace_cossim_static(z, s, z, s, m, r, out)
