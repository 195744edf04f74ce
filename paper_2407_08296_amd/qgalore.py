"""ctypes binding of libqgalore.so: argument marshalling only.

Every function has the name and argument order of the C entry point it wraps
(see include/qgalore.h) minus the `qg_` prefix.  Tensors are torch CUDA(HIP)
tensors used purely as device-memory handles; all arithmetic happens in the
library's kernels.  There is no CPU fallback: if the shared library has not
been built, importing a symbol from it raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("QGALORE_LIB") or os.path.join(_HERE, "libqgalore.so")   # QGALORE_LIB: another build of the library
GROUP = 256

EXPORTS = [
    "qg_status_string", "qg_last_hip_error", "qg_quant_int8", "qg_quant_int4", "qg_dequant_int8", "qg_dequant_int4",
    "qg_project", "qg_lowrank_adam", "qg_backproject_update_sr", "qg_cossim_workspace_bytes", "qg_subspace_cossim",
    "qg_policy_update", "qg_workspace_bytes", "qg_step", "qg_plan_bytes", "qg_plan_build", "qg_step_many",
    "qg_sr_uniform", "qg_project_many", "qg_lowrank_adam_many", "qg_backproject_update_sr_many",
    "qg_project_adam", "qg_project_adam_many", "qg_diag_clock_probe", "qg_diag_mfma_loop",
    "qg_diag_mfma_f64_loop",
    "qg_range_apply", "qg_orthonormalize_workspace_bytes", "qg_orthonormalize", "qg_refresh_workspace_bytes",
    "qg_subspace_refresh", "qg_subspace_refresh_many", "qg_int8_linear_forward", "qg_int8_linear_backward",
    "qg_int8_linear_t_forward", "qg_int8_linear_t_backward",
    "qg_quant_int8_zp", "qg_dequant_int8_zp", "qg_backproject_update_sr_zp", "qg_step_zp",
    "qg_int8_linear_zp_forward", "qg_int8_linear_zp_backward",
    "qg_int8_linear_t_zp_forward", "qg_int8_linear_t_zp_backward",
    "qg_state8_quant", "qg_state8_dequant", "qg_lowrank_adam8", "qg_step8",
    "qg_subspace_cossim_static", "qg_subspace_cossim_weighted", "qg_step_ld", "qg_subspace_refresh_many_ld",
    "qg_int8_linear_forward_ld", "qg_int8_linear_backward_ld",
]


class QGError(RuntimeError):
    pass


class HParams(C.Structure):
    _fields_ = [("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float), ("lr", C.c_float),
                ("alpha", C.c_float)]


class Policy(C.Structure):
    _fields_ = [("interval", C.c_int), ("streak", C.c_int), ("k", C.c_int), ("next_refresh", C.c_int),
                ("threshold", C.c_float), ("last_cos", C.c_float)]


class MatrixDesc(C.Structure):
    _fields_ = [("m", C.c_int64), ("n", C.c_int64), ("r", C.c_int64),
                ("Pq", C.c_void_p), ("Ps", C.c_void_p), ("G", C.c_void_p), ("Wq", C.c_void_p), ("Ws", C.c_void_p),
                ("M", C.c_void_p), ("V", C.c_void_p), ("R", C.c_void_p), ("N", C.c_void_p), ("ld", C.c_int64),
                ("Wz", C.c_void_p)]


class RefreshDesc(C.Structure):
    _fields_ = [("Pq", C.c_void_p), ("Ps", C.c_void_p), ("G", C.c_void_p), ("Pq_new", C.c_void_p),
                ("Ps_new", C.c_void_p)]


_lib = None


def lib() -> C.CDLL:
    """Load libqgalore.so (once).  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise QGError(f"{LIB_PATH} is missing: build it with `python -m paper_2407_08296_amd.build` "
                          "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        i64, vp, i32, u64, f32, sz = C.c_int64, C.c_void_p, C.c_int, C.c_uint64, C.c_float, C.c_size_t
        L.qg_status_string.restype = C.c_char_p
        L.qg_status_string.argtypes = [i32]
        L.qg_last_hip_error.restype = i32
        L.qg_quant_int8.argtypes = [vp, i64, i64, i32, vp, vp, vp]
        L.qg_quant_int4.argtypes = [vp, i64, i64, i32, vp, vp, vp]
        L.qg_dequant_int8.argtypes = [vp, vp, i64, i64, i32, vp, vp]
        L.qg_dequant_int4.argtypes = [vp, vp, i64, i64, i32, vp, vp]
        L.qg_project.argtypes = [vp, vp, vp, i64, i64, i64, i32, vp, vp, sz, vp]
        L.qg_lowrank_adam.argtypes = [vp, vp, vp, vp, i64, i64, C.POINTER(HParams), vp]
        L.qg_backproject_update_sr.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i32, f32, f32, u64, i64, vp, vp]
        L.qg_quant_int8_zp.argtypes = [vp, i64, i64, i32, vp, vp, vp, vp]
        L.qg_dequant_int8_zp.argtypes = [vp, vp, vp, i64, i64, i32, vp, vp]
        L.qg_backproject_update_sr_zp.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, i32, f32, f32, u64, i64, vp]
        L.qg_step_zp.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, i32, C.POINTER(HParams), u64,
                                 i64, vp]
        L.qg_int8_linear_zp_forward.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i32, vp, vp]
        L.qg_int8_linear_zp_backward.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i32, vp, vp, vp]
        L.qg_int8_linear_t_zp_forward.argtypes = L.qg_int8_linear_zp_forward.argtypes
        L.qg_int8_linear_t_zp_backward.argtypes = L.qg_int8_linear_zp_backward.argtypes
        L.qg_cossim_workspace_bytes.restype = sz
        L.qg_cossim_workspace_bytes.argtypes = [i64, i64]
        L.qg_subspace_cossim.argtypes = [vp, vp, vp, vp, i64, i64, i32, vp, vp, sz, vp]
        L.qg_subspace_cossim_static.argtypes = [vp, vp, vp, vp, i64, i64, i32, vp, vp]
        L.qg_subspace_cossim_weighted.argtypes = [vp, vp, vp, vp, vp, i64, i64, i32, vp, vp, sz, vp]
        L.qg_step_ld.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, i64, i32, C.POINTER(HParams), u64, i64,
                                 vp]
        L.qg_policy_update.argtypes = [C.POINTER(Policy), f32]
        L.qg_workspace_bytes.restype = sz
        L.qg_workspace_bytes.argtypes = [i64, i64, i64]
        L.qg_step.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, i32, C.POINTER(HParams), u64, i64,
                              vp, sz, vp]
        L.qg_plan_bytes.restype = sz
        L.qg_plan_bytes.argtypes = [i32, C.POINTER(MatrixDesc)]
        L.qg_plan_build.argtypes = [i32, C.POINTER(MatrixDesc), vp, sz]
        L.qg_step_many.argtypes = [i32, vp, vp, sz, C.POINTER(HParams), u64, i64, vp]
        L.qg_sr_uniform.argtypes = [u64, i64, u64, i64, vp, vp]
        L.qg_project_many.argtypes = [i32, vp, vp, sz, vp]
        L.qg_lowrank_adam_many.argtypes = [i32, vp, vp, sz, C.POINTER(HParams), i64, vp]
        L.qg_backproject_update_sr_many.argtypes = [i32, vp, vp, sz, C.POINTER(HParams), u64, i64, vp]
        L.qg_project_adam.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, i32, i64, C.POINTER(HParams), vp]
        L.qg_project_adam_many.argtypes = [i32, vp, vp, sz, C.POINTER(HParams), i64, i32, vp]
        L.qg_diag_clock_probe.argtypes = [i64, vp, vp]
        L.qg_diag_mfma_loop.argtypes = [i64, i32, vp, vp]
        L.qg_diag_mfma_f64_loop.argtypes = [i64, i32, vp, vp]
        L.qg_range_apply.argtypes = [vp, vp, i64, i64, i64, vp, vp]
        L.qg_orthonormalize_workspace_bytes.restype = sz
        L.qg_orthonormalize_workspace_bytes.argtypes = [i64, i64]
        L.qg_orthonormalize.argtypes = [vp, i64, i64, vp, vp, vp, sz, vp]
        L.qg_refresh_workspace_bytes.restype = sz
        L.qg_refresh_workspace_bytes.argtypes = [i32, i64, i64, i64]
        L.qg_subspace_refresh.argtypes = [vp, vp, vp, i64, i64, i64, i32, i32, vp, vp, vp, vp, vp, sz, vp]
        L.qg_state8_quant.argtypes = [vp, i64, i32, vp, vp, vp]
        L.qg_state8_dequant.argtypes = [vp, vp, i64, i32, vp, vp]
        L.qg_lowrank_adam8.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, C.POINTER(HParams), vp]
        L.qg_step8.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, i32, C.POINTER(HParams), u64, i64, vp]
        L.qg_int8_linear_forward.argtypes = [vp, vp, vp, vp, i64, i64, i64, i32, vp, vp]
        L.qg_int8_linear_backward.argtypes = [vp, vp, vp, vp, i64, i64, i64, i32, vp, vp, vp]
        L.qg_int8_linear_forward_ld.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, i64, i32, vp, vp]
        L.qg_int8_linear_backward_ld.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, i64, i32, vp, vp, vp]
        L.qg_int8_linear_t_forward.argtypes = L.qg_int8_linear_forward.argtypes
        L.qg_int8_linear_t_backward.argtypes = L.qg_int8_linear_backward.argtypes
        L.qg_subspace_refresh_many.argtypes = [i32, C.POINTER(RefreshDesc), i64, i64, i64, i32, i32, vp, vp, vp, sz, vp]
        L.qg_subspace_refresh_many_ld.argtypes = [i32, C.POINTER(RefreshDesc), i64, i64, i64, i64, i32, i32, vp, vp, vp, sz,
                                                  vp]
        _lib = L
    return _lib


def _check(status: int) -> None:
    if status != 0:
        L = lib()
        msg = L.qg_status_string(status).decode()
        if status == 6:
            msg += f" (hipError {L.qg_last_hip_error()})"
        raise QGError(f"libqgalore: {msg}")


def _ptr(t: torch.Tensor | None, dtypes=None) -> int | None:
    if t is None:
        return None
    if not t.is_cuda:
        raise QGError("device tensor expected")
    if not t.is_contiguous():
        raise QGError("contiguous tensor expected")
    if dtypes is not None and t.dtype not in dtypes:
        raise QGError(f"dtype {t.dtype} not in {dtypes}")
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


_BF16 = (torch.bfloat16, torch.int16, torch.uint16)


def hparams(beta1=0.9, beta2=0.999, eps=1e-8, lr=1e-3, alpha=0.25) -> HParams:
    return HParams(beta1, beta2, eps, lr, alpha)


# ---------------------------------------------------------------- quantizers
def quant_int8(x: torch.Tensor):
    rows, cols = x.shape
    q = torch.empty((rows, cols), dtype=torch.int8, device=x.device)
    s = torch.empty((rows, (cols + GROUP - 1) // GROUP), dtype=torch.float32, device=x.device)
    _check(lib().qg_quant_int8(_ptr(x, (torch.float32,)), rows, cols, GROUP, _ptr(q), _ptr(s), _stream()))
    return q, s


def quant_int4(x: torch.Tensor):
    rows, cols = x.shape
    total = rows * cols
    q = torch.empty(((total + 1) // 2,), dtype=torch.uint8, device=x.device)
    s = torch.empty(((total + GROUP - 1) // GROUP,), dtype=torch.float32, device=x.device)
    _check(lib().qg_quant_int4(_ptr(x, (torch.float32,)), rows, cols, GROUP, _ptr(q), _ptr(s), _stream()))
    return q, s


def dequant_int8(q: torch.Tensor, s: torch.Tensor) -> torch.Tensor:
    rows, cols = q.shape
    x = torch.empty((rows, cols), dtype=torch.float32, device=q.device)
    _check(lib().qg_dequant_int8(_ptr(q, (torch.int8,)), _ptr(s, (torch.float32,)), rows, cols, GROUP, _ptr(x),
                                 _stream()))
    return x


def dequant_int4(q: torch.Tensor, s: torch.Tensor, rows: int, cols: int) -> torch.Tensor:
    x = torch.empty((rows, cols), dtype=torch.float32, device=q.device)
    _check(lib().qg_dequant_int4(_ptr(q, (torch.uint8,)), _ptr(s, (torch.float32,)), rows, cols, GROUP, _ptr(x),
                                 _stream()))
    return x


# ---------------------------------------------------------------- step pieces
def project(Pq, Ps, G, m: int, n: int, r: int, R: torch.Tensor | None = None) -> torch.Tensor:
    if R is None:
        R = torch.empty((r, n), dtype=torch.float32, device=G.device)
    _check(lib().qg_project(_ptr(Pq, (torch.uint8,)), _ptr(Ps, (torch.float32,)), _ptr(G, _BF16), m, n, r, GROUP,
                            _ptr(R, (torch.float32,)), None, 0, _stream()))
    return R


def lowrank_adam(R, M, V, N, step: int, hp: HParams) -> None:
    _check(lib().qg_lowrank_adam(_ptr(R, (torch.float32,)), _ptr(M, (torch.float32,)), _ptr(V, (torch.float32,)),
                                 _ptr(N, _BF16), R.numel(), step, C.byref(hp), _stream()))


def project_adam(Pq, Ps, G, R, M, V, N, m: int, n: int, r: int, step: int, hp: HParams) -> None:
    _check(lib().qg_project_adam(_ptr(Pq, (torch.uint8,)), _ptr(Ps, (torch.float32,)), _ptr(G, _BF16),
                                 _ptr(R, (torch.float32,)), _ptr(M, (torch.float32,)), _ptr(V, (torch.float32,)),
                                 _ptr(N, _BF16), m, n, r, GROUP, step, C.byref(hp), _stream()))


def backproject_update_sr(Pq, Ps, N, Wq, Ws, m: int, n: int, r: int, alpha: float, lr: float, seed: int, step: int,
                          U_debug: torch.Tensor | None = None) -> None:
    _check(lib().qg_backproject_update_sr(_ptr(Pq, (torch.uint8,)), _ptr(Ps, (torch.float32,)), _ptr(N, _BF16),
                                          _ptr(Wq, (torch.int8,)), _ptr(Ws, (torch.float32,)), m, n, r, GROUP,
                                          alpha, lr, seed, step, _ptr(U_debug, (torch.float32,)), _stream()))


def subspace_cossim(PqA, PsA, PqB, PsB, m: int, r: int, weights: torch.Tensor | None = None) -> torch.Tensor:
    """qg_subspace_cossim, or qg_subspace_cossim_weighted when `weights` (fp32 [r]) is given."""
    nbytes = lib().qg_cossim_workspace_bytes(m, r)
    ws = torch.empty((max(nbytes, 16),), dtype=torch.uint8, device=PqA.device)
    out = torch.empty((1,), dtype=torch.float32, device=PqA.device)
    if weights is None:
        _check(lib().qg_subspace_cossim(_ptr(PqA, (torch.uint8,)), _ptr(PsA, (torch.float32,)), _ptr(PqB, (torch.uint8,)),
                                        _ptr(PsB, (torch.float32,)), m, r, GROUP, _ptr(out), _ptr(ws), nbytes, _stream()))
    else:
        _check(lib().qg_subspace_cossim_weighted(_ptr(PqA, (torch.uint8,)), _ptr(PsA, (torch.float32,)),
                                                 _ptr(PqB, (torch.uint8,)), _ptr(PsB, (torch.float32,)),
                                                 _ptr(weights, (torch.float32,)), m, r, GROUP, _ptr(out), _ptr(ws),
                                                 nbytes, _stream()))
    return out


def subspace_cossim_static(PqA, PsA, PqB, PsB, m: int, r: int, out: torch.Tensor) -> None:
    """qg_subspace_cossim_static: no workspace; `out` is the caller's one-float device tensor."""
    _check(lib().qg_subspace_cossim_static(_ptr(PqA, (torch.uint8,)), _ptr(PsA, (torch.float32,)),
                                           _ptr(PqB, (torch.uint8,)), _ptr(PsB, (torch.float32,)), m, r, GROUP,
                                           _ptr(out, (torch.float32,)), _stream()))


def policy_update(p: Policy, cos: float) -> bool:
    rc = lib().qg_policy_update(C.byref(p), cos)
    if rc < 0:
        raise QGError("libqgalore: null policy")
    return bool(rc)


def step(Pq, Ps, G, Wq, Ws, M, V, R, N, m: int, n: int, r: int, hp: HParams, seed: int, step: int) -> None:
    _check(lib().qg_step(_ptr(Pq, (torch.uint8,)), _ptr(Ps, (torch.float32,)), _ptr(G, _BF16),
                         _ptr(Wq, (torch.int8,)), _ptr(Ws, (torch.float32,)), _ptr(M, (torch.float32,)),
                         _ptr(V, (torch.float32,)), _ptr(R, (torch.float32,)), _ptr(N, _BF16), m, n, r, GROUP,
                         C.byref(hp), seed, step, None, 0, _stream()))


def step_ld(Pq, Ps, G, Wq, Ws, M, V, R, N, m: int, n: int, ld: int, r: int, hp: HParams, seed: int, step: int) -> None:
    """qg_step_ld: every n-wide array is stored with rows ld elements apart."""
    _check(lib().qg_step_ld(_ptr(Pq, (torch.uint8,)), _ptr(Ps, (torch.float32,)), _ptr(G, _BF16),
                            _ptr(Wq, (torch.int8,)), _ptr(Ws, (torch.float32,)), _ptr(M, (torch.float32,)),
                            _ptr(V, (torch.float32,)), _ptr(R, (torch.float32,)), _ptr(N, _BF16), m, n, ld, r, GROUP,
                            C.byref(hp), seed, step, _stream()))


@dataclass
class MatrixState:
    """Device tensors of one weight matrix, as passed to qg_step / qg_step_many."""
    m: int
    n: int
    r: int
    Pq: torch.Tensor
    Ps: torch.Tensor
    G: torch.Tensor
    Wq: torch.Tensor
    Ws: torch.Tensor
    M: torch.Tensor
    V: torch.Tensor
    R: torch.Tensor | None
    N: torch.Tensor
    ld: int = 0   # row pitch in elements of G, Wq, M, V, R, N; 0 = n
    Wz: torch.Tensor | None = None   # zero points of W (all matrices of a plan, or none)


class StepPlan:
    """Host + device copies of the grouped-launch plan of qg_step_many."""

    def __init__(self, mats: list[MatrixState]):
        self.count = len(mats)
        self.mats = mats
        descs = (MatrixDesc * self.count)()
        for d, s in zip(descs, mats):
            d.m, d.n, d.r = s.m, s.n, s.r
            d.Pq, d.Ps, d.G = _ptr(s.Pq, (torch.uint8,)), _ptr(s.Ps, (torch.float32,)), _ptr(s.G, _BF16)
            d.Wq, d.Ws = _ptr(s.Wq, (torch.int8,)), _ptr(s.Ws, (torch.float32,))
            d.M, d.V, d.R = _ptr(s.M, (torch.float32,)), _ptr(s.V, (torch.float32,)), _ptr(s.R, (torch.float32,))
            d.N = _ptr(s.N, _BF16)
            d.ld = s.ld
            d.Wz = _ptr(s.Wz, (torch.float32,))
        self.nbytes = lib().qg_plan_bytes(self.count, descs)
        self.host = torch.empty((self.nbytes,), dtype=torch.uint8).pin_memory()
        _check(lib().qg_plan_build(self.count, descs, self.host.data_ptr(), self.nbytes))
        self.dev = self.host.to(mats[0].Wq.device)


def step_many(plan: StepPlan, hp: HParams, seed: int, step: int) -> None:
    _check(lib().qg_step_many(plan.count, plan.host.data_ptr(), plan.dev.data_ptr(), plan.nbytes, C.byref(hp), seed,
                              step, _stream()))


def project_many(plan: StepPlan) -> None:
    _check(lib().qg_project_many(plan.count, plan.host.data_ptr(), plan.dev.data_ptr(), plan.nbytes, _stream()))


def lowrank_adam_many(plan: StepPlan, hp: HParams, step: int) -> None:
    _check(lib().qg_lowrank_adam_many(plan.count, plan.host.data_ptr(), plan.dev.data_ptr(), plan.nbytes,
                                      C.byref(hp), step, _stream()))


def project_adam_many(plan: StepPlan, hp: HParams, step: int, write_R: bool = False) -> None:
    _check(lib().qg_project_adam_many(plan.count, plan.host.data_ptr(), plan.dev.data_ptr(), plan.nbytes,
                                      C.byref(hp), step, int(write_R), _stream()))


def backproject_update_sr_many(plan: StepPlan, hp: HParams, seed: int, step: int) -> None:
    _check(lib().qg_backproject_update_sr_many(plan.count, plan.host.data_ptr(), plan.dev.data_ptr(), plan.nbytes,
                                               C.byref(hp), seed, step, _stream()))


# ---------------------------------------------------------------- zero-point (asymmetric) INT8 weights
def quant_int8_zp(x: torch.Tensor):
    rows, cols = x.shape
    q = torch.empty((rows, cols), dtype=torch.int8, device=x.device)
    s = torch.empty((rows, (cols + GROUP - 1) // GROUP), dtype=torch.float32, device=x.device)
    z = torch.empty_like(s)
    _check(lib().qg_quant_int8_zp(_ptr(x, (torch.float32,)), rows, cols, GROUP, _ptr(q), _ptr(s), _ptr(z), _stream()))
    return q, s, z


def dequant_int8_zp(q: torch.Tensor, s: torch.Tensor, z: torch.Tensor) -> torch.Tensor:
    rows, cols = q.shape
    x = torch.empty((rows, cols), dtype=torch.float32, device=q.device)
    _check(lib().qg_dequant_int8_zp(_ptr(q, (torch.int8,)), _ptr(s, (torch.float32,)), _ptr(z, (torch.float32,)), rows,
                                    cols, GROUP, _ptr(x), _stream()))
    return x


def backproject_update_sr_zp(Pq, Ps, N, Wq, Ws, Wz, m: int, n: int, r: int, alpha: float, lr: float, seed: int,
                             step: int) -> None:
    _check(lib().qg_backproject_update_sr_zp(_ptr(Pq, (torch.uint8,)), _ptr(Ps, (torch.float32,)), _ptr(N, _BF16),
                                             _ptr(Wq, (torch.int8,)), _ptr(Ws, (torch.float32,)),
                                             _ptr(Wz, (torch.float32,)), m, n, r, GROUP, alpha, lr, seed, step, _stream()))


def step_zp(Pq, Ps, G, Wq, Ws, Wz, M, V, R, N, m: int, n: int, r: int, hp: HParams, seed: int, step: int) -> None:
    _check(lib().qg_step_zp(_ptr(Pq, (torch.uint8,)), _ptr(Ps, (torch.float32,)), _ptr(G, _BF16),
                            _ptr(Wq, (torch.int8,)), _ptr(Ws, (torch.float32,)), _ptr(Wz, (torch.float32,)),
                            _ptr(M, (torch.float32,)), _ptr(V, (torch.float32,)), _ptr(R, (torch.float32,)),
                            _ptr(N, _BF16), m, n, r, GROUP, C.byref(hp), seed, step, _stream()))


def int8_linear_zp_forward(x: torch.Tensor, Wq: torch.Tensor, Ws: torch.Tensor, Wz: torch.Tensor,
                           bias: torch.Tensor | None = None):
    tokens, n = x.shape
    m = Wq.shape[0]
    y = torch.empty((tokens, m), dtype=torch.bfloat16, device=x.device)
    _check(lib().qg_int8_linear_zp_forward(_ptr(x, _BF16), _ptr(Wq, (torch.int8,)), _ptr(Ws, (torch.float32,)),
                                           _ptr(Wz, (torch.float32,)), _ptr(bias, _BF16), tokens, m, n, GROUP,
                                           _ptr(y), _stream()))
    return y


def int8_linear_zp_backward(dy: torch.Tensor, x: torch.Tensor | None, Wq, Ws, Wz, m: int, n: int,
                            want_dx: bool = True, want_G: bool = True):
    tokens = dy.shape[0]
    dx = torch.empty((tokens, n), dtype=torch.bfloat16, device=dy.device) if want_dx else None
    G = torch.empty((m, n), dtype=torch.bfloat16, device=dy.device) if want_G else None
    _check(lib().qg_int8_linear_zp_backward(_ptr(dy, _BF16), _ptr(x, _BF16), _ptr(Wq, (torch.int8,)),
                                            _ptr(Ws, (torch.float32,)), _ptr(Wz, (torch.float32,)), tokens, m, n, GROUP,
                                            _ptr(dx), _ptr(G), _stream()))
    return dx, G


def int8_linear_t_zp_forward(x: torch.Tensor, Sq: torch.Tensor, Ss: torch.Tensor, Sz: torch.Tensor,
                             bias: torch.Tensor | None = None):
    """Zero-point weight stored transposed (Sq: [n][m])."""
    tokens, n = x.shape
    m = Sq.shape[1]
    y = torch.empty((tokens, m), dtype=torch.bfloat16, device=x.device)
    _check(lib().qg_int8_linear_t_zp_forward(_ptr(x, _BF16), _ptr(Sq, (torch.int8,)), _ptr(Ss, (torch.float32,)),
                                             _ptr(Sz, (torch.float32,)), _ptr(bias, _BF16), tokens, m, n, GROUP,
                                             _ptr(y), _stream()))
    return y


def int8_linear_t_zp_backward(dy: torch.Tensor, x: torch.Tensor | None, Sq, Ss, Sz, m: int, n: int,
                              want_dx: bool = True, want_G: bool = True):
    tokens = dy.shape[0]
    dx = torch.empty((tokens, n), dtype=torch.bfloat16, device=dy.device) if want_dx else None
    G = torch.empty((n, m), dtype=torch.bfloat16, device=dy.device) if want_G else None
    _check(lib().qg_int8_linear_t_zp_backward(_ptr(dy, _BF16), _ptr(x, _BF16), _ptr(Sq, (torch.int8,)),
                                              _ptr(Ss, (torch.float32,)), _ptr(Sz, (torch.float32,)), tokens, m, n,
                                              GROUP, _ptr(dx), _ptr(G), _stream()))
    return dx, G


# ---------------------------------------------------------------- 8-bit Adam states
def state8_quant(x: torch.Tensor, signed: bool):
    count = x.numel()
    codes = torch.empty((count,), dtype=torch.uint8, device=x.device)
    scales = torch.empty(((count + GROUP - 1) // GROUP,), dtype=torch.float32, device=x.device)
    _check(lib().qg_state8_quant(_ptr(x, (torch.float32,)), count, int(signed), _ptr(codes), _ptr(scales), _stream()))
    return codes, scales


def state8_dequant(codes: torch.Tensor, scales: torch.Tensor, signed: bool) -> torch.Tensor:
    x = torch.empty((codes.numel(),), dtype=torch.float32, device=codes.device)
    _check(lib().qg_state8_dequant(_ptr(codes, (torch.uint8,)), _ptr(scales, (torch.float32,)), codes.numel(),
                                   int(signed), _ptr(x), _stream()))
    return x


def lowrank_adam8(R, Mq, Ms, Vq, Vs, N, step: int, hp: HParams) -> None:
    _check(lib().qg_lowrank_adam8(_ptr(R, (torch.float32,)), _ptr(Mq, (torch.uint8,)), _ptr(Ms, (torch.float32,)),
                                  _ptr(Vq, (torch.uint8,)), _ptr(Vs, (torch.float32,)), _ptr(N, _BF16), R.numel(), step,
                                  C.byref(hp), _stream()))


def step8(Pq, Ps, G, Wq, Ws, Mq, Ms, Vq, Vs, R, N, m: int, n: int, r: int, hp: HParams, seed: int, step: int) -> None:
    _check(lib().qg_step8(_ptr(Pq, (torch.uint8,)), _ptr(Ps, (torch.float32,)), _ptr(G, _BF16), _ptr(Wq, (torch.int8,)),
                          _ptr(Ws, (torch.float32,)), _ptr(Mq, (torch.uint8,)), _ptr(Ms, (torch.float32,)),
                          _ptr(Vq, (torch.uint8,)), _ptr(Vs, (torch.float32,)), _ptr(R, (torch.float32,)), _ptr(N, _BF16),
                          m, n, r, GROUP, C.byref(hp), seed, step, _stream()))


# ---------------------------------------------------------------- INT8 linear layer
def int8_linear_forward(x: torch.Tensor, Wq: torch.Tensor, Ws: torch.Tensor, bias: torch.Tensor | None = None):
    tokens, n = x.shape
    m = Wq.shape[0]
    y = torch.empty((tokens, m), dtype=torch.bfloat16, device=x.device)
    _check(lib().qg_int8_linear_forward(_ptr(x, _BF16), _ptr(Wq, (torch.int8,)), _ptr(Ws, (torch.float32,)),
                                        _ptr(bias, _BF16), tokens, m, n, GROUP, _ptr(y), _stream()))
    return y


def int8_linear_backward(dy: torch.Tensor, x: torch.Tensor | None, Wq: torch.Tensor | None, Ws: torch.Tensor | None,
                         m: int, n: int, want_dx: bool = True, want_G: bool = True):
    tokens = dy.shape[0]
    dx = torch.empty((tokens, n), dtype=torch.bfloat16, device=dy.device) if want_dx else None
    G = torch.empty((m, n), dtype=torch.bfloat16, device=dy.device) if want_G else None
    _check(lib().qg_int8_linear_backward(_ptr(dy, _BF16), _ptr(x, _BF16), _ptr(Wq, (torch.int8,)),
                                         _ptr(Ws, (torch.float32,)), tokens, m, n, GROUP, _ptr(dx), _ptr(G), _stream()))
    return dx, G


def int8_linear_forward_ld(x, Wq, Ws, bias, tokens: int, m: int, n: int, ld_n: int, ld_m: int, y: torch.Tensor) -> None:
    """qg_int8_linear_forward_ld: x [tokens][ld_n], Wq [m][ld_n], y [tokens][ld_m] (the caller's, padding untouched)."""
    _check(lib().qg_int8_linear_forward_ld(_ptr(x, _BF16), _ptr(Wq, (torch.int8,)), _ptr(Ws, (torch.float32,)),
                                           _ptr(bias, _BF16), tokens, m, n, ld_n, ld_m, GROUP, _ptr(y, _BF16), _stream()))


def int8_linear_backward_ld(dy, x, Wq, Ws, tokens: int, m: int, n: int, ld_n: int, ld_m: int, dx, G) -> None:
    """qg_int8_linear_backward_ld: dy [tokens][ld_m], x and dx [tokens][ld_n], Wq and G [m][ld_n]; dx or G may be None."""
    _check(lib().qg_int8_linear_backward_ld(_ptr(dy, _BF16), _ptr(x, _BF16), _ptr(Wq, (torch.int8,)),
                                            _ptr(Ws, (torch.float32,)), tokens, m, n, ld_n, ld_m, GROUP,
                                            _ptr(dx, _BF16), _ptr(G, _BF16), _stream()))


def int8_linear_t_forward(x: torch.Tensor, Sq: torch.Tensor, Ss: torch.Tensor, bias: torch.Tensor | None = None):
    """The layer on a weight stored transposed (Sq: [n][m])."""
    tokens, n = x.shape
    m = Sq.shape[1]
    y = torch.empty((tokens, m), dtype=torch.bfloat16, device=x.device)
    _check(lib().qg_int8_linear_t_forward(_ptr(x, _BF16), _ptr(Sq, (torch.int8,)), _ptr(Ss, (torch.float32,)),
                                          _ptr(bias, _BF16), tokens, m, n, GROUP, _ptr(y), _stream()))
    return y


def int8_linear_t_backward(dy: torch.Tensor, x: torch.Tensor | None, Sq: torch.Tensor | None, Ss: torch.Tensor | None,
                           m: int, n: int, want_dx: bool = True, want_G: bool = True):
    """Returns (dx [tokens][n], G_S [n][m]) for a weight stored transposed."""
    tokens = dy.shape[0]
    dx = torch.empty((tokens, n), dtype=torch.bfloat16, device=dy.device) if want_dx else None
    G = torch.empty((n, m), dtype=torch.bfloat16, device=dy.device) if want_G else None
    _check(lib().qg_int8_linear_t_backward(_ptr(dy, _BF16), _ptr(x, _BF16), _ptr(Sq, (torch.int8,)),
                                           _ptr(Ss, (torch.float32,)), tokens, m, n, GROUP, _ptr(dx), _ptr(G), _stream()))
    return dx, G


# ---------------------------------------------------------------- subspace refresh
def range_apply(G: torch.Tensor, Z: torch.Tensor, m: int, n: int, r: int) -> torch.Tensor:
    Y = torch.empty((m, r), dtype=torch.float32, device=G.device)
    _check(lib().qg_range_apply(_ptr(G, _BF16), _ptr(Z, _BF16), m, n, r, _ptr(Y), _stream()))
    return Y


def orthonormalize(Y: torch.Tensor):
    """Returns (Q, info): Q fp32 [m][r], info a device int32 (0 = every pivot positive)."""
    m, r = Y.shape
    nbytes = lib().qg_orthonormalize_workspace_bytes(m, r)
    if nbytes == 0:
        raise QGError("libqgalore: shape out of range")
    ws = torch.empty((nbytes,), dtype=torch.uint8, device=Y.device)
    Q = torch.empty_like(Y)
    info = torch.empty((1,), dtype=torch.int32, device=Y.device)
    _check(lib().qg_orthonormalize(_ptr(Y, (torch.float32,)), m, r, _ptr(Q), _ptr(info), _ptr(ws), nbytes, _stream()))
    return Q, info


def subspace_refresh(Pq, Ps, G, m: int, n: int, r: int, passes: int = 1, workspace: torch.Tensor | None = None):
    """Returns (Pq_new, Ps_new, cos, info, workspace); cos and info are device tensors of one element."""
    nbytes = lib().qg_refresh_workspace_bytes(1, m, n, r)
    if nbytes == 0:
        raise QGError("libqgalore: shape out of range")
    if workspace is None:
        workspace = torch.empty((nbytes,), dtype=torch.uint8, device=G.device)
    Pq_new, Ps_new = torch.empty_like(Pq), torch.empty_like(Ps)
    cos = torch.empty((1,), dtype=torch.float32, device=G.device)
    info = torch.empty((1,), dtype=torch.int32, device=G.device)
    _check(lib().qg_subspace_refresh(_ptr(Pq, (torch.uint8,)), _ptr(Ps, (torch.float32,)), _ptr(G, _BF16), m, n, r,
                                     GROUP, passes, _ptr(Pq_new), _ptr(Ps_new), _ptr(cos), _ptr(info),
                                     _ptr(workspace), workspace.numel(), _stream()))
    return Pq_new, Ps_new, cos, info, workspace


def subspace_refresh_many(Pqs, Pss, Gs, m: int, n: int, r: int, passes: int = 1,
                          workspace: torch.Tensor | None = None, out=None, ld: int = 0):
    """Refresh of several matrices of one shape.  Pqs, Pss, Gs: lists of device tensors.  `out`: optional
    (list of Pq_new, list of Ps_new) to write into.  ld: row pitch of the gradients (0: dense).
    Returns (Pq_news, Ps_news, cos[count], info[count], workspace)."""
    count = len(Gs)
    if count == 0 or len(Pqs) != count or len(Pss) != count:
        raise QGError("libqgalore: one Pq and one Ps per gradient expected")
    if workspace is None:
        nbytes = lib().qg_refresh_workspace_bytes(count, m, ld or n, r)
        if nbytes == 0:
            raise QGError("libqgalore: shape out of range")
        workspace = torch.empty((nbytes,), dtype=torch.uint8, device=Gs[0].device)
    if out is None:
        out = ([torch.empty_like(p) for p in Pqs], [torch.empty_like(p) for p in Pss])
    descs = (RefreshDesc * count)()
    for i in range(count):
        descs[i] = RefreshDesc(_ptr(Pqs[i], (torch.uint8,)), _ptr(Pss[i], (torch.float32,)), _ptr(Gs[i], _BF16),
                               _ptr(out[0][i], (torch.uint8,)), _ptr(out[1][i], (torch.float32,)))
    cos = torch.empty((count,), dtype=torch.float32, device=Gs[0].device)
    info = torch.empty((count,), dtype=torch.int32, device=Gs[0].device)
    _check(lib().qg_subspace_refresh_many_ld(count, descs, m, n, ld, r, GROUP, passes, _ptr(cos), _ptr(info),
                                             _ptr(workspace), workspace.numel(), _stream()))
    return out[0], out[1], cos, info, workspace


DIAG_MFMA_WORKGROUPS = 512


def diag_clock_probe(ticks_100mhz: int, out2: torch.Tensor) -> None:
    """Enqueue the clock probe on the current stream; out2 (2 x int64, device) receives {shader cycles, ticks}."""
    _check(lib().qg_diag_clock_probe(ticks_100mhz, _ptr(out2, (torch.int64,)), _stream()))


def diag_mfma_loop(iters: int, random_operands: bool, sink: torch.Tensor) -> float:
    """Enqueue the register-only MFMA loop; returns the flop it performs."""
    assert sink.numel() >= DIAG_MFMA_WORKGROUPS * 512
    _check(lib().qg_diag_mfma_loop(iters, int(random_operands), _ptr(sink, (torch.float32,)), _stream()))
    return DIAG_MFMA_WORKGROUPS * 8 * iters * 16 * 32768.0


def diag_mfma_f64_loop(iters: int, workgroups: int, sink: torch.Tensor) -> float:
    """Enqueue the register-only fp64 MFMA loop; returns the flop it performs."""
    assert sink.numel() >= workgroups * 256
    _check(lib().qg_diag_mfma_f64_loop(iters, workgroups, _ptr(sink, (torch.float32,)), _stream()))
    return workgroups * 4 * iters * 8 * 2048.0


def sr_uniform(seed: int, step: int, idx0: int, count: int, device="cuda") -> torch.Tensor:
    out = torch.empty((count,), dtype=torch.float32, device=device)
    _check(lib().qg_sr_uniform(seed, step, idx0, count, _ptr(out), _stream()))
    return out
