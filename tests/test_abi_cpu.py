"""CPU-only checks of the C-ABI boundary: the library loads, exports every symbol the header
declares, rejects bad arguments before any HIP call, and the host-only policy matches Sec. 3.2."""
import ctypes as C
import os
import re

import pytest

from paper_2407_08296_amd import qgalore as qg
from oracle import qgalore as Q

HEADER = os.path.join(os.path.dirname(os.path.dirname(__file__)), "include", "qgalore.h")
FAKE = 0x10000          # non-null, 16-byte aligned, never dereferenced on the error paths


@pytest.fixture(scope="module")
def L():
    return qg.lib()


def test_header_symbols_are_exported(L):
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"\b(qg_[a-z0-9_]+)\s*\(", text))
    assert names == set(qg.EXPORTS)
    for n in names:
        assert hasattr(L, n), n


def test_status_strings(L):
    assert L.qg_status_string(0) == b"ok"
    for code in range(1, 7):
        assert len(L.qg_status_string(code)) > 0


def test_quant_argument_errors(L):
    assert L.qg_quant_int8(None, 4, 256, 256, FAKE, FAKE, None) == 1
    assert L.qg_quant_int8(FAKE, 0, 256, 256, FAKE, FAKE, None) == 2
    assert L.qg_quant_int8(FAKE, 4, -1, 256, FAKE, FAKE, None) == 2
    assert L.qg_quant_int8(FAKE, 4, 256, 128, FAKE, FAKE, None) == 3
    assert L.qg_quant_int8(FAKE + 4, 4, 256, 256, FAKE, FAKE, None) == 4
    assert L.qg_quant_int4(FAKE, 4, 256, 256, None, FAKE, None) == 1
    assert L.qg_quant_int4(FAKE, 4, 256, 64, FAKE, FAKE, None) == 3
    assert L.qg_dequant_int4(FAKE, FAKE, 4, 256, 256, FAKE + 8, None) == 4
    assert L.qg_dequant_int8(FAKE, None, 4, 256, 256, FAKE, None) == 1


def test_step_piece_argument_errors(L):
    hp = qg.hparams()
    assert L.qg_project(None, FAKE, FAKE, 512, 512, 128, 256, FAKE, None, 0, None) == 1
    assert L.qg_project(FAKE, FAKE, FAKE, 512, 512, 0, 256, FAKE, None, 0, None) == 2
    assert L.qg_project(FAKE, FAKE, FAKE, 512, 512, 127, 256, FAKE, None, 0, None) == 2      # r % 8 != 0
    assert L.qg_project(FAKE, FAKE, FAKE, 64, 512, 128, 256, FAKE, None, 0, None) == 2       # r > m
    assert L.qg_project(FAKE, FAKE, FAKE, 1 << 17, 1 << 17, 128, 256, FAKE, None, 0, None) == 2   # m*n >= 2^32
    assert L.qg_project(FAKE, FAKE, FAKE, 512, 512, 128, 512, FAKE, None, 0, None) == 3
    assert L.qg_project(FAKE, FAKE, FAKE + 2, 512, 512, 128, 256, FAKE, None, 0, None) == 4
    assert L.qg_lowrank_adam(FAKE, FAKE, FAKE, FAKE, 100, 0, C.byref(hp), None) == 2        # t >= 1
    assert L.qg_lowrank_adam(FAKE, FAKE, FAKE, FAKE, 100, 1, None, None) == 1
    assert L.qg_lowrank_adam(FAKE, FAKE, FAKE, FAKE, 0, 1, C.byref(hp), None) == 2
    assert L.qg_backproject_update_sr(FAKE, FAKE, FAKE, FAKE, None, 512, 512, 128, 256, 0.25, 1e-3, 0, 1, None, None) == 1
    assert L.qg_backproject_update_sr(FAKE, FAKE, FAKE, FAKE, FAKE, 512, 512, 128, 256, 0.25, 1e-3, 0, 0, None, None) == 2
    assert L.qg_backproject_update_sr(FAKE, FAKE, FAKE, FAKE, FAKE, 512, 512, 128, 256, 0.25, 1e-3, 0, 1, FAKE + 4, None) == 4
    assert L.qg_subspace_cossim(FAKE, FAKE, FAKE, FAKE, 512, 128, 256, FAKE, None, 0, None) == 5
    assert L.qg_subspace_cossim(FAKE, FAKE, FAKE, FAKE, 512, 128, 256, FAKE, FAKE, 16, None) == 5
    assert L.qg_subspace_cossim(FAKE, FAKE, FAKE, FAKE, 512, 130, 256, FAKE, FAKE, 1 << 20, None) == 2
    assert L.qg_cossim_workspace_bytes(512, 128) == (8 * 3 * 128 + 2 * 2) * 4
    assert L.qg_step(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 512, 512, 128, 256, None, 0, 1, None, 0, None) == 1
    assert L.qg_step(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 512, 512, 128, 256, C.byref(hp), 0, 0, None, 0, None) == 2
    assert L.qg_sr_uniform(0, 1, 0, 0, FAKE, None) == 2
    assert L.qg_sr_uniform(0, 1, 0, 16, None, None) == 1
    assert L.qg_diag_clock_probe(0, FAKE, None) == 2
    assert L.qg_diag_clock_probe(10 ** 9, FAKE, None) == 2      # more than a second of spinning is refused
    assert L.qg_diag_clock_probe(1000, None, None) == 1
    assert L.qg_diag_mfma_loop(0, 0, FAKE, None) == 2
    assert L.qg_diag_mfma_loop(16, 1, None, None) == 1


def test_refresh_argument_errors(L):
    assert L.qg_range_apply(None, FAKE, 512, 512, 128, FAKE, None) == 1
    assert L.qg_range_apply(FAKE, FAKE, 512, 512, 132, FAKE, None) == 2                      # r % 8 != 0
    assert L.qg_range_apply(FAKE, FAKE, 64, 512, 128, FAKE, None) == 2                       # r > m
    assert L.qg_range_apply(FAKE, FAKE, 1 << 17, 1 << 17, 128, FAKE, None) == 2              # m*n >= 2^32
    assert L.qg_range_apply(FAKE, FAKE + 2, 512, 512, 128, FAKE, None) == 4
    ob = L.qg_orthonormalize_workspace_bytes(512, 128)
    assert ob >= 2 * 128 * 128 * 8 + 2 * 64 * 64 * 8 + 512 * 128 * 4 and ob % 256 == 0
    assert L.qg_orthonormalize_workspace_bytes(64, 128) == 0
    assert L.qg_orthonormalize(FAKE, 512, 128, FAKE + 4096, None, FAKE, ob, None) == 1
    assert L.qg_orthonormalize(FAKE, 512, 128, FAKE, FAKE, FAKE, ob, None) == 2              # Y and Q alias
    assert L.qg_orthonormalize(FAKE, 512, 128, FAKE + 4096, FAKE, FAKE, ob - 1, None) == 5
    assert L.qg_orthonormalize(FAKE, 512, 128, FAKE + 4096, FAKE, None, 0, None) == 5
    assert L.qg_orthonormalize(FAKE, 1 << 22, 1024, FAKE + 4096, FAKE, FAKE, 1 << 40, None) == 2   # m*r >= 2^31
    rb = L.qg_refresh_workspace_bytes(1, 512, 512, 128)
    assert rb >= 128 * 512 * 6 + 2 * 512 * 128 * 4 + ob + L.qg_cossim_workspace_bytes(512, 128)
    assert L.qg_refresh_workspace_bytes(1, 512, 0, 128) == 0 and L.qg_refresh_workspace_bytes(0, 512, 512, 128) == 0
    rb4 = L.qg_refresh_workspace_bytes(4, 512, 512, 128)
    assert rb < rb4 <= 4 * rb
    rb64 = L.qg_refresh_workspace_bytes(64, 512, 512, 128)                                   # R and Z: 16 matrices at most
    assert 16 * rb < rb64 <= 64 * rb - 48 * 128 * 512 * 6
    args = (FAKE, FAKE, FAKE, 512, 512, 128, 256, 1, FAKE + 4096, FAKE + 8192, FAKE, FAKE, FAKE, rb, None)

    def call(**kw):
        a = list(args)
        for k, v in kw.items():
            a[int(k[1:])] = v
        return L.qg_subspace_refresh(*a)
    assert call(a0=None) == 1 and call(a10=None) == 1 and call(a11=None) == 1
    assert call(a7=0) == 2 and call(a7=65) == 2                                              # passes
    assert call(a6=128) == 3
    assert call(a8=FAKE) == 2                                                                # new P aliases the old
    assert call(a2=FAKE + 2) == 4
    assert call(a13=rb - 1) == 5 and call(a12=None) == 5
    descs = (qg.RefreshDesc * 2)(qg.RefreshDesc(FAKE, FAKE, FAKE, FAKE + 4096, FAKE + 8192),
                                 qg.RefreshDesc(FAKE, FAKE, FAKE, FAKE + 4096, None))
    assert L.qg_subspace_refresh_many(2, descs, 512, 512, 128, 256, 1, FAKE, FAKE, FAKE, rb4, None) == 1
    assert L.qg_subspace_refresh_many(0, descs, 512, 512, 128, 256, 1, FAKE, FAKE, FAKE, rb4, None) == 2
    assert L.qg_subspace_refresh_many(1, None, 512, 512, 128, 256, 1, FAKE, FAKE, FAKE, rb4, None) == 1
    assert L.qg_subspace_refresh_many(1, descs, 512, 512, 128, 256, 1, FAKE, FAKE + 2, FAKE, rb4, None) == 4


def test_int8_linear_argument_errors(L):
    assert L.qg_int8_linear_forward(None, FAKE, FAKE, None, 16, 512, 512, 256, FAKE, None) == 1
    assert L.qg_int8_linear_forward(FAKE, FAKE, FAKE, None, 0, 512, 512, 256, FAKE, None) == 2
    assert L.qg_int8_linear_forward(FAKE, FAKE, FAKE, None, 1 << 20, 1 << 12, 512, 256, FAKE, None) == 2   # tokens*m >= 2^31
    assert L.qg_int8_linear_forward(FAKE, FAKE, FAKE, None, 16, 512, 512, 128, FAKE, None) == 3
    assert L.qg_int8_linear_forward(FAKE, FAKE, FAKE, FAKE + 2, 16, 512, 512, 256, FAKE, None) == 4
    assert L.qg_int8_linear_backward(FAKE, FAKE, FAKE, FAKE, 16, 512, 512, 256, None, None, None) == 1     # no output asked for
    assert L.qg_int8_linear_backward(FAKE, None, FAKE, FAKE, 16, 512, 512, 256, FAKE, FAKE, None) == 1     # G needs x
    assert L.qg_int8_linear_backward(FAKE, FAKE, None, FAKE, 16, 512, 512, 256, FAKE, None, None) == 1     # dx needs W
    assert L.qg_int8_linear_backward(FAKE, FAKE, FAKE, FAKE, 16, 512, 0, 256, FAKE, FAKE, None) == 2
    assert L.qg_int8_linear_backward(FAKE + 8, FAKE, FAKE, FAKE, 16, 512, 512, 256, FAKE, FAKE, None) == 4
    # the same layer on a weight stored transposed
    assert L.qg_int8_linear_t_forward(FAKE, None, FAKE, None, 16, 512, 512, 256, FAKE, None) == 1
    assert L.qg_int8_linear_t_forward(FAKE, FAKE, FAKE, None, 16, 0, 512, 256, FAKE, None) == 2
    assert L.qg_int8_linear_t_forward(FAKE, FAKE, FAKE, None, 16, 512, 512, 64, FAKE, None) == 3
    assert L.qg_int8_linear_t_forward(FAKE, FAKE + 4, FAKE, None, 16, 512, 512, 256, FAKE, None) == 4
    assert L.qg_int8_linear_t_backward(FAKE, FAKE, FAKE, FAKE, 16, 512, 512, 256, None, None, None) == 1
    assert L.qg_int8_linear_t_backward(FAKE, None, FAKE, FAKE, 16, 512, 512, 256, None, FAKE, None) == 1
    assert L.qg_int8_linear_t_backward(FAKE, FAKE, FAKE, None, 16, 512, 512, 256, FAKE, None, None) == 1
    assert L.qg_int8_linear_t_backward(FAKE, FAKE, FAKE, FAKE, 1 << 20, 512, 1 << 12, 256, FAKE, FAKE, None) == 2
    assert L.qg_int8_linear_t_backward(FAKE, FAKE, FAKE, FAKE, 16, 512, 512, 256, FAKE, FAKE + 2, None) == 4


def test_zero_point_argument_errors(L):
    hp = qg.hparams()
    assert L.qg_quant_int8_zp(FAKE, 4, 256, 256, FAKE, FAKE, None, None) == 1
    assert L.qg_quant_int8_zp(FAKE, 0, 256, 256, FAKE, FAKE, FAKE, None) == 2
    assert L.qg_quant_int8_zp(FAKE, 4, 256, 128, FAKE, FAKE, FAKE, None) == 3
    assert L.qg_quant_int8_zp(FAKE, 4, 256, 256, FAKE, FAKE, FAKE + 4, None) == 4
    assert L.qg_dequant_int8_zp(FAKE, FAKE, None, 4, 256, 256, FAKE, None) == 1
    assert L.qg_backproject_update_sr_zp(FAKE, FAKE, FAKE, FAKE, FAKE, None, 512, 512, 128, 256, 0.25, 1e-3, 0, 1, None) == 1
    assert L.qg_backproject_update_sr_zp(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 512, 512, 12, 256, 0.25, 1e-3, 0, 1, None) == 2
    assert L.qg_backproject_update_sr_zp(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 512, 512, 128, 256, 0.25, 1e-3, 0, 0, None) == 2
    assert L.qg_backproject_update_sr_zp(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE + 8, 512, 512, 128, 256, 0.25, 1e-3, 0, 1, None) == 4
    assert L.qg_step_zp(FAKE, FAKE, FAKE, FAKE, FAKE, None, FAKE, FAKE, None, FAKE, 512, 512, 128, 256, C.byref(hp), 0, 1, None) == 1
    assert L.qg_step_zp(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, FAKE, 512, 512, 128, 64, C.byref(hp), 0, 1, None) == 3
    assert L.qg_int8_linear_zp_forward(FAKE, FAKE, FAKE, None, None, 16, 512, 512, 256, FAKE, None) == 1
    assert L.qg_int8_linear_zp_forward(FAKE, FAKE, FAKE, FAKE, None, 16, 512, 0, 256, FAKE, None) == 2
    assert L.qg_int8_linear_zp_backward(FAKE, FAKE, FAKE, FAKE, None, 16, 512, 512, 256, FAKE, FAKE, None) == 1   # dx needs Wz
    assert L.qg_int8_linear_zp_backward(FAKE, FAKE, None, None, None, 16, 512, 512, 256, None, FAKE + 2, None) == 4
    assert L.qg_int8_linear_t_zp_forward(FAKE, FAKE, FAKE, None, None, 16, 512, 512, 256, FAKE, None) == 1
    assert L.qg_int8_linear_t_zp_forward(FAKE, FAKE, FAKE, FAKE, None, 16, 512, 512, 32, FAKE, None) == 3
    assert L.qg_int8_linear_t_zp_backward(FAKE, FAKE, FAKE, FAKE, None, 16, 512, 512, 256, FAKE, None, None) == 1
    assert L.qg_int8_linear_t_zp_backward(FAKE, FAKE, FAKE, FAKE, FAKE, 0, 512, 512, 256, FAKE, FAKE, None) == 2
    # a plan takes zero points for all matrices or for none
    descs = (qg.MatrixDesc * 2)()
    for d in descs:
        d.m, d.n, d.r = 512, 512, 128
        for f in ("Pq", "Ps", "G", "Wq", "Ws", "M", "V", "R", "N"):
            setattr(d, f, FAKE)
    nbytes = L.qg_plan_bytes(2, descs)
    buf = C.create_string_buffer(nbytes)
    descs[0].Wz = FAKE
    assert L.qg_plan_build(2, descs, buf, nbytes) == 1
    descs[1].Wz = FAKE
    assert L.qg_plan_build(2, descs, buf, nbytes) == 0
    assert (C.c_uint32 * 16).from_buffer(buf)[13] == 1      # header word: zero-point plan


def test_diag_argument_errors(L):
    assert L.qg_diag_mfma_f64_loop(10, 4, None, None) == 1
    assert L.qg_diag_mfma_f64_loop(0, 4, FAKE, None) == 2
    assert L.qg_diag_mfma_f64_loop(10, 0, FAKE, None) == 2
    assert L.qg_diag_mfma_f64_loop(10, 1 << 20, FAKE, None) == 2


def test_adam8_argument_errors(L):
    hp = qg.hparams()
    assert L.qg_state8_quant(None, 256, 1, FAKE, FAKE, None) == 1
    assert L.qg_state8_quant(FAKE, 0, 1, FAKE, FAKE, None) == 2
    assert L.qg_state8_quant(FAKE, 258, 1, FAKE, FAKE, None) == 2                            # not a multiple of 4
    assert L.qg_state8_quant(FAKE, 256, 1, FAKE + 4, FAKE, None) == 4
    assert L.qg_state8_dequant(FAKE, None, 256, 0, FAKE, None) == 1
    assert L.qg_lowrank_adam8(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 256, 1, None, None) == 1
    assert L.qg_lowrank_adam8(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 256, 0, C.byref(hp), None) == 2   # t >= 1
    assert L.qg_lowrank_adam8(FAKE, FAKE, FAKE, FAKE + 8, FAKE, FAKE, 256, 1, C.byref(hp), None) == 4


def test_plan_build_on_host(L):
    descs = (qg.MatrixDesc * 2)()
    for d, (m, n, r) in zip(descs, [(4096, 4096, 1024), (11008, 4096, 1024)]):
        d.m, d.n, d.r = m, n, r
        for f in ("Pq", "Ps", "G", "Wq", "Ws", "M", "V", "R", "N"):
            setattr(d, f, FAKE)
    nbytes = L.qg_plan_bytes(2, descs)
    assert nbytes > 0
    buf = C.create_string_buffer(nbytes)
    assert L.qg_plan_build(2, descs, buf, nbytes - 1) == 5
    assert L.qg_plan_build(2, descs, buf, nbytes) == 0
    # header: magic, count, Adam chunks, no_R, then per class (exact, masked, unaligned): matrices, projection
    # tiles, back-projection tiles
    hdr = (C.c_uint32 * 16).from_buffer(buf)
    assert hdr[1] == 2                                       # count
    assert hdr[2] == 2 * (1024 * 4096) // 4096               # Adam chunks of 4096 elements
    assert hdr[3] == 0                                       # every matrix has an R buffer
    assert list(hdr[4:7]) == [2, 0, 0]                       # both matrices need no edge checks
    assert list(hdr[7:10]) == [2 * 8 * 16, 0, 0]             # projection tiles 128 x 256 over r x n
    assert list(hdr[10:13]) == [32 * 16 + 86 * 16, 0, 0]     # back-projection tiles 128 x 256 over m x n
    descs[1].n = 5461                                        # odd row length: rows not 16-byte aligned
    assert L.qg_plan_build(2, descs, buf, nbytes) == 0
    hdr = (C.c_uint32 * 16).from_buffer(buf)
    assert list(hdr[4:7]) == [1, 0, 1]
    assert list(hdr[7:10]) == [8 * 16, 0, 8 * 22] and list(hdr[10:13]) == [32 * 16, 0, 86 * 22]
    descs[1].n = 2736                                        # ragged but aligned rows; m = 11008 = 86 x 128
    assert L.qg_plan_build(2, descs, buf, nbytes) == 0
    hdr = (C.c_uint32 * 16).from_buffer(buf)
    assert list(hdr[4:7]) == [1, 1, 0]
    assert list(hdr[7:10]) == [8 * 16, 8 * 11, 0] and list(hdr[10:13]) == [32 * 16, 86 * 11, 0]
    descs[1].n, descs[1].ld = 5461, 5472                     # the same odd n with a row pitch: aligned rows, masked class
    assert L.qg_plan_build(2, descs, buf, nbytes) == 0
    hdr = (C.c_uint32 * 16).from_buffer(buf)
    assert list(hdr[4:7]) == [1, 1, 0]
    assert hdr[2] == (1024 * 4096 + 1024 * 5472) // 4096     # the unfused Adam runs over the padding too
    assert list(hdr[7:10]) == [8 * 16, 8 * 22, 0] and list(hdr[10:13]) == [32 * 16, 86 * 22, 0]
    for bad in (5460, 5464, 5461 + 7):                       # below n; not a multiple of 16 (twice)
        descs[1].ld = bad
        assert L.qg_plan_build(2, descs, buf, nbytes) == 2
    descs[1].ld = 5461                                       # ld == n is the dense layout
    assert L.qg_plan_build(2, descs, buf, nbytes) == 0
    descs[1].ld = 0
    descs[1].n = 5461
    descs[1].r = 12
    assert L.qg_plan_build(2, descs, buf, nbytes) == 2
    descs[1].r = 1024
    descs[0].G = None
    assert L.qg_plan_build(2, descs, buf, nbytes) == 1
    hp = qg.hparams()
    assert L.qg_step_many(2, None, FAKE, nbytes, C.byref(hp), 0, 1, None) == 1
    assert L.qg_step_many(3, buf, FAKE, nbytes, C.byref(hp), 0, 1, None) == 5


def test_policy_matches_oracle_tables(L):
    for k, seq in [(1, [0.9, 0.1, 0.4, 0.39]), (2, [0.9, 0.9, 0.9, 0.1, 0.9, 0.9]), (3, [0.5, 0.5, 0.3, 0.5, 0.5, 0.5, 0.5])]:
        p = qg.Policy(200, 0, k, 200, 0.4, 0.0)
        o = Q.Policy(interval=200, k=k, threshold=0.4, next_refresh=200)
        for c in seq:
            assert qg.policy_update(p, c) == o.update(float(C.c_float(c).value))
            assert (p.interval, p.streak, p.next_refresh) == (o.interval, o.streak, o.next_refresh)
    assert L.qg_policy_update(None, 0.5) == -1


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    p = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert p.returncode != 0
    assert "ONE GPU" in (p.stderr + p.stdout)


def test_product_package_does_not_touch_the_oracle():
    """The library and its binding may not import, read or call anything under oracle/ (test infrastructure)."""
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    pkg = os.path.join(root, "paper_2407_08296_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".h", ".hip")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle|oracle[./]|#include.*oracle", text, re.M), \
                    os.path.join(dirpath, f)


def test_sizes_past_the_index_limit_are_refused(L):
    """m * n = 2^32: every call that indexes elements with 32 bits returns the shape error; just below it passes the
    shape check (and fails the next one, here a misaligned pointer)."""
    hp = qg.hparams()
    assert L.qg_step(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 65536, 65536, 128, 256, C.byref(hp), 0, 1,
                     None, 0, None) == 2
    assert L.qg_backproject_update_sr(FAKE, FAKE, FAKE, FAKE, FAKE, 65536, 65536, 128, 256, 0.25, 1e-3, 0, 1, None, None) == 2
    assert L.qg_project(FAKE, FAKE, FAKE, 65536, 65536, 128, 256, FAKE, None, 0, None) == 2
    assert L.qg_backproject_update_sr(FAKE, FAKE, FAKE, FAKE + 4, FAKE, 32768, 130816, 128, 256, 0.25, 1e-3, 0, 1, None,
                                      None) == 4
    descs = (qg.MatrixDesc * 1)()
    d = descs[0]
    d.m, d.n, d.r = 65536, 65536, 128
    for f in ("Pq", "Ps", "G", "Wq", "Ws", "M", "V", "R", "N"):
        setattr(d, f, FAKE)
    nbytes = L.qg_plan_bytes(1, descs)
    buf = C.create_string_buffer(nbytes)
    assert L.qg_plan_build(1, descs, buf, nbytes) == 2

