"""fp64 numpy oracle of the Q-GaLore per-matrix optimizer step.

TEST INFRASTRUCTURE ONLY: nothing in the product path may import this module.
It is independent of the HIP library (no shared code, tables or constants
generators) and is pinned by tests/test_oracle_*.py against closed forms,
invariants, library routines and brute force.

Notation follows the paper: W is the m x n weight (INT8 codes Wq plus one fp32
scale per block of 256 elements of a row), G the m x n bf16 gradient, P the
m x r projection matrix (INT4 codes plus one fp32 scale per block of 256
elements of the flattened row-major array), R = P^T G the projected gradient,
M and V the Adam moments (r x n), N the Adam direction, U = alpha * P * N the
back-projected update, t the 1-based step count.

Every function states the passage of the paper it follows.  Where the paper
is silent the reading taken is stated in the function's docstring; all such
readings are "parity unpinned" (no value printed in the paper can confirm
them): the symmetric absmax scale with z = 0, the reciprocal-multiply form of
W/s, the flat/row block rules, the nibble packing, the hash constants of the
stochastic-rounding generator, the textbook Adam form and the column-mean
cosine.  Later sections add the subspace refresh, the INT8 linear layer, 8-bit
Adam states, right-side projection and the zero-point (asymmetric) weight
format, each with its own readings.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

GROUP = 256          # block size of the quantizer (Sec. 3.1, "block size of 256")
QMAX = {4: 7, 8: 127}  # 2^(n-1) - 1


# --------------------------------------------------------------------------
# bf16 helpers (Sec. 3.1: activations and gradients are BFloat16)
# --------------------------------------------------------------------------
def bf16_rne(x) -> np.ndarray:
    """Round fp64 values to the nearest bf16 value (ties to even), ONE rounding.

    Result is returned as fp64 (every bf16 value is exactly representable).
    bf16 keeps 8 significant bits and fp32's exponent range; values below the
    smallest normal (2^-126) are rounded on the subnormal grid 2^-133.
    """
    x = np.asarray(x, dtype=np.float64)
    out = np.empty_like(x)
    bits = x.view(np.uint64) if x.flags["C_CONTIGUOUS"] else np.ascontiguousarray(x).view(np.uint64)
    bits = bits.reshape(x.shape).copy()
    drop = np.uint64(52 - 7)                       # fp64 has 52 fraction bits, bf16 has 7
    lsb = (bits >> drop) & np.uint64(1)
    bits = bits + ((np.uint64(1) << (drop - np.uint64(1))) - np.uint64(1)) + lsb
    bits &= ~((np.uint64(1) << drop) - np.uint64(1))
    out[...] = bits.view(np.float64).reshape(x.shape)
    tiny = np.abs(x) < 2.0 ** -126
    if np.any(tiny):
        q = 2.0 ** -133
        out[tiny] = np.rint(x[tiny] / q) * q
    nonfinite = ~np.isfinite(x)
    if np.any(nonfinite):
        out[nonfinite] = x[nonfinite]
    return out


def bf16_bits_to_f64(bits) -> np.ndarray:
    """Decode bf16 bit patterns (uint16) to their exact values."""
    b = np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return b.view(np.float32).astype(np.float64)


def f64_to_bf16_bits(x) -> np.ndarray:
    """Round to bf16 (one rounding) and return the uint16 bit patterns."""
    r = bf16_rne(x).astype(np.float32)             # exact: bf16 values are fp32 values
    return (r.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


# --------------------------------------------------------------------------
# Block-wise uniform quantization (Sec. 3.1, the Quant_n equation)
# --------------------------------------------------------------------------
def _scale_pair(absmax32: np.ndarray, bits: int):
    """fp32 scale s = a/qmax and fp32 reciprocal scale qmax/a of each block.

    A block whose absmax is 0 gets s = 0 and reciprocal 0 (all codes 0).
    Both quotients are correctly rounded fp32 quotients: an fp64 quotient of two
    fp32 numbers rounded to fp32 equals the fp32 quotient (53 >= 2*24 + 2).
    """
    a = absmax32.astype(np.float64)
    qmax = float(QMAX[bits])
    with np.errstate(divide="ignore", invalid="ignore"):
        s = np.where(a > 0, a / qmax, 0.0).astype(np.float32)
        inv = np.where(a > 0, qmax / a, 0.0).astype(np.float32)
    return s, inv


def _codes_rne(x32: np.ndarray, inv32: np.ndarray, bits: int) -> np.ndarray:
    """clamp(round_half_even(fl32(x * (1/s))), -2^(n-1), 2^(n-1)-1) with z = 0."""
    t = (x32.astype(np.float32) * inv32.astype(np.float32)).astype(np.float32)  # one fp32 product
    q = np.rint(t.astype(np.float64))
    return np.clip(q, -(QMAX[bits] + 1), QMAX[bits]).astype(np.int8)


def quant_int8(x) -> tuple[np.ndarray, np.ndarray]:
    """Quant_8 of an fp32 matrix; a block = 256 consecutive elements of a row.

    The last block of a row is short when cols % 256 != 0.  Returns int8 codes
    [rows][cols] and fp32 scales [rows][ceil(cols/256)].  (Sec. 3.1; symmetric
    absmax scale, zero point 0.)
    """
    x = np.asarray(x, dtype=np.float32)
    rows, cols = x.shape
    ng = (cols + GROUP - 1) // GROUP
    q = np.zeros((rows, cols), dtype=np.int8)
    scales = np.zeros((rows, ng), dtype=np.float32)
    for g in range(ng):
        blk = x[:, g * GROUP:(g + 1) * GROUP]
        a = np.max(np.abs(blk), axis=1).astype(np.float32)
        s, inv = _scale_pair(a, 8)
        scales[:, g] = s
        q[:, g * GROUP:(g + 1) * GROUP] = _codes_rne(blk, inv[:, None], 8)
    return q, scales


def dequant_int8(q, scales) -> np.ndarray:
    """W = W_q * s per block (Appendix A dequantization with zeros = 0), exact in fp64."""
    q = np.asarray(q)
    rows, cols = q.shape
    s = np.repeat(np.asarray(scales, dtype=np.float64), GROUP, axis=1)[:, :cols]
    return q.astype(np.float64) * s


def quant_int4_codes(x) -> tuple[np.ndarray, np.ndarray]:
    """Quant_4 of an fp32 matrix; a block = 256 consecutive elements of the
    flattened row-major array (Sec. 3.3: block size 256 across all layers).

    Returns int8 codes in [-7, 7], shape of x, and fp32 scales [ceil(size/256)].
    """
    x = np.asarray(x, dtype=np.float32)
    flat = x.reshape(-1)
    ng = (flat.size + GROUP - 1) // GROUP
    codes = np.zeros(flat.size, dtype=np.int8)
    scales = np.zeros(ng, dtype=np.float32)
    full = (flat.size // GROUP) * GROUP
    if full:
        blk = flat[:full].reshape(-1, GROUP)
        a = np.max(np.abs(blk), axis=1).astype(np.float32)
        s, inv = _scale_pair(a, 4)
        scales[: full // GROUP] = s
        codes[:full] = _codes_rne(blk, inv[:, None], 4).reshape(-1)
    if full < flat.size:
        blk = flat[full:]
        a = np.max(np.abs(blk)).astype(np.float32).reshape(1)
        s, inv = _scale_pair(a, 4)
        scales[-1] = s[0]
        codes[full:] = _codes_rne(blk, inv, 4)
    return codes.reshape(x.shape), scales


def pack_int4(codes) -> np.ndarray:
    """Two codes per byte: flat element 2b in the low nibble of byte b, 2b+1 in
    the high nibble; stored nibble = code + 8 (offset binary).  An odd count
    leaves the last high nibble at 8 (code 0)."""
    c = np.asarray(codes, dtype=np.int16).reshape(-1) + 8
    if np.any((c < 0) | (c > 15)):
        raise ValueError("INT4 code out of range")
    if c.size % 2:
        c = np.concatenate([c, np.array([8], dtype=np.int16)])
    return (c[0::2] | (c[1::2] << 4)).astype(np.uint8)


def unpack_int4(packed, count: int) -> np.ndarray:
    """Inverse of pack_int4: the first `count` codes as int8."""
    p = np.asarray(packed, dtype=np.uint8).astype(np.int16)
    c = np.empty(p.size * 2, dtype=np.int16)
    c[0::2] = p & 0xF
    c[1::2] = p >> 4
    return (c[:count] - 8).astype(np.int8)


def quant_int4(x) -> tuple[np.ndarray, np.ndarray]:
    """Quant_4 followed by nibble packing: (packed uint8 [ceil(size/2)], scales)."""
    codes, scales = quant_int4_codes(x)
    return pack_int4(codes), scales


def dequant_int4(packed, scales, rows: int, cols: int) -> np.ndarray:
    """P = P_q * s per flat block of 256, exact in fp64, shape [rows][cols]."""
    codes = unpack_int4(packed, rows * cols).astype(np.float64)
    s = np.repeat(np.asarray(scales, dtype=np.float64), GROUP)[: rows * cols]
    return (codes * s).reshape(rows, cols)


# --------------------------------------------------------------------------
# Stochastic rounding (Sec. 3.4, the F_SR equation) and its generator
# --------------------------------------------------------------------------
_M32 = 0xFFFFFFFF
_GOLDEN = 0x9E3779B9


def _mix32(x):
    """32-bit avalanche mixer: xorshift 16, multiply 0x7FEB352D, xorshift 15,
    multiply 0x846CA68B, xorshift 16 (a published public-domain integer hash)."""
    x = np.asarray(x, dtype=np.uint64) & np.uint64(_M32)
    x ^= x >> np.uint64(16)
    x = (x * np.uint64(0x7FEB352D)) & np.uint64(_M32)
    x ^= x >> np.uint64(15)
    x = (x * np.uint64(0x846CA68B)) & np.uint64(_M32)
    x ^= x >> np.uint64(16)
    return x


def sr_key(seed: int, step: int, idx_hi: int = 0) -> int:
    """Fold (seed_lo, seed_hi, step_lo, step_hi, idx_hi) into one 32-bit key:
    key <- mix32((key xor word) + 0x9E3779B9), starting from 0x9E3779B9."""
    seed &= (1 << 64) - 1
    step &= (1 << 64) - 1
    key = _GOLDEN
    for w in (seed & _M32, seed >> 32, step & _M32, step >> 32, idx_hi & _M32):
        key = int(_mix32(((key ^ w) + _GOLDEN) & _M32))
    return key


def sr_hash(seed: int, step: int, idx) -> np.ndarray:
    """32-bit hash of (seed, step, element index): mix32(key xor idx_lo)."""
    idx = np.asarray(idx, dtype=np.uint64)
    hi = idx >> np.uint64(32)
    lo = idx & np.uint64(_M32)
    if hi.size and np.any(hi != hi.reshape(-1)[0]):
        keys = np.array([sr_key(seed, step, int(h)) for h in hi.reshape(-1)], dtype=np.uint64).reshape(hi.shape)
    else:
        keys = np.uint64(sr_key(seed, step, int(hi.reshape(-1)[0]) if hi.size else 0))
    return _mix32(keys ^ lo)


def sr_uniform(seed: int, step: int, idx) -> np.ndarray:
    """u in [0, 1): the top 24 bits of the hash times 2^-24 (exact in fp32)."""
    return (sr_hash(seed, step, idx) >> np.uint64(8)).astype(np.float64) * 2.0 ** -24


def sr_round(v, u) -> np.ndarray:
    """F_SR(v) = floor(v + u), u uniform in [0,1): floor(v) with probability
    ceil(v) - v and ceil(v) with probability v - floor(v).  The sum is taken in
    fp32, the precision in which the library takes this decision."""
    s = (np.asarray(v, dtype=np.float32) + np.asarray(u, dtype=np.float32)).astype(np.float32)
    return np.floor(s.astype(np.float64))


# --------------------------------------------------------------------------
# The optimizer step (Sec. 3.5)
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class HParams:
    """Adam and GaLore hyper-parameters, held as the fp32 values the library
    receives (Sec. 4.1: scale factor alpha = 0.25)."""
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    lr: float = 1e-3
    alpha: float = 0.25

    def f32(self):
        f = lambda v: float(np.float32(v))
        return HParams(f(self.beta1), f(self.beta2), f(self.eps), f(self.lr), f(self.alpha))


def dequant_p_bf16(Pq, Ps, m: int, r: int) -> np.ndarray:
    """P as the GEMMs see it: dequantized by a floating-point multiply, code * scale rounded to fp32 (the form of
    the Appendix A dequantization, a product in a floating type), then stored as a bf16 GEMM operand (Sec. 3.1)."""
    return bf16_rne(dequant_int4(Pq, Ps, m, r).astype(np.float32).astype(np.float64))


def project(Pq, Ps, G_bits, m: int, n: int, r: int) -> np.ndarray:
    """R = P^T G (Sec. 3.5: the full-rank gradient is projected into a low-rank
    format), P dequantized and rounded to bf16, G's bf16 values taken exactly."""
    Pd = dequant_p_bf16(Pq, Ps, m, r)
    G = bf16_bits_to_f64(np.asarray(G_bits).reshape(m, n))
    return Pd.T @ G


def lowrank_adam(R, M, V, t: int, hp: HParams):
    """Adam on the low-rank gradient (Sec. 3.5; Adam as cited in Sec. 4.1):
    M' = b1 M + (1-b1) R;  V' = b2 V + (1-b2) R^2;
    N = (M'/(1-b1^t)) / (sqrt(V'/(1-b2^t)) + eps).  Returns (M', V', N)."""
    hp = hp.f32()
    R = np.asarray(R, dtype=np.float64)
    M1 = hp.beta1 * np.asarray(M, dtype=np.float64) + (1.0 - hp.beta1) * R
    V1 = hp.beta2 * np.asarray(V, dtype=np.float64) + (1.0 - hp.beta2) * R * R
    mhat = M1 / (1.0 - hp.beta1 ** t)
    vhat = V1 / (1.0 - hp.beta2 ** t)
    N = mhat / (np.sqrt(vhat) + hp.eps)
    return M1, V1, N


def backproject(Pq, Ps, Nb, m: int, r: int, alpha: float) -> np.ndarray:
    """U = alpha * P * N (Sec. 3.5: the low-rank update is projected back to full
    rank; Sec. 4.1: scale factor alpha), Nb being N already rounded to bf16."""
    Pd = dequant_p_bf16(Pq, Ps, m, r)
    return float(np.float32(alpha)) * (Pd @ np.asarray(Nb, dtype=np.float64))


def update_sr(Wq, Ws, U, lr: float, seed: int, t: int, n_total: int | None = None, col0: int = 0):
    """INT8 weight update with stochastic rounding (Sec. 3.4, Sec. 3.5).

    x = W_q * s - lr * U; per block of 256 of each row a = max|x|, new scale
    s' = a/127, code = clamp(F_SR(x * (127/a)), -128, 127) with the uniform draw
    u(seed, t, i*n_total + col0 + j).  The decision steps (absmax, the two
    quotients, the product, the sum with u) are taken in fp32.
    Returns (new codes, new scales).
    """
    Wq = np.asarray(Wq)
    m, n = Wq.shape
    n_total = n if n_total is None else n_total
    x = dequant_int8(Wq, Ws) - float(np.float32(lr)) * np.asarray(U, dtype=np.float64)
    x32 = x.astype(np.float32)
    ng = (n + GROUP - 1) // GROUP
    newq = np.zeros((m, n), dtype=np.int8)
    news = np.zeros((m, ng), dtype=np.float32)
    ii = np.arange(m, dtype=np.uint64)[:, None]
    for g in range(ng):
        c0, c1 = g * GROUP, min((g + 1) * GROUP, n)
        blk = x32[:, c0:c1]
        a = np.max(np.abs(blk), axis=1).astype(np.float32)
        s, inv = _scale_pair(a, 8)
        news[:, g] = s
        tq = (blk * inv[:, None]).astype(np.float32)
        idx = ii * np.uint64(n_total) + np.arange(col0 + c0, col0 + c1, dtype=np.uint64)[None, :]
        u = sr_uniform(seed, t, idx)
        newq[:, c0:c1] = np.clip(sr_round(tq, u), -128, 127).astype(np.int8)
    return newq, news


def step(Wq, Ws, G_bits, Pq, Ps, M, V, t: int, hp: HParams, seed: int,
         r: int, n_total: int | None = None, col0: int = 0) -> dict:
    """One Q-GaLore step on one matrix (Sec. 3.5): project, Adam, back-project,
    INT8 stochastic-rounding update.  All operations are column-separable, so a
    slice of columns [col0, col0+n) of a wider matrix (n_total columns, col0 a
    multiple of 256) can be stepped alone and gives that slice of the result.
    """
    Wq = np.asarray(Wq)
    m, n = Wq.shape
    R = project(Pq, Ps, G_bits, m, n, r)
    M1, V1, N = lowrank_adam(R, M, V, t, hp)
    Nb = bf16_rne(N)
    U = backproject(Pq, Ps, Nb, m, r, hp.alpha)
    newq, news = update_sr(Wq, Ws, U, hp.lr, seed, t, n_total, col0)
    return dict(R=R, M=M1, V=V1, N=N, Nb=Nb, U=U, Wq=newq, Ws=news)


# --------------------------------------------------------------------------
# Layer-adaptive subspace check (Sec. 3.2)
# --------------------------------------------------------------------------
def subspace_cossim(PqA, PsA, PqB, PsB, m: int, r: int) -> float:
    """Cosine similarity between two adjacent projection matrices (Fig. 2): the
    mean over the r columns of cos(a_k, b_k) on the dequantized INT4 values."""
    A = dequant_int4(PqA, PsA, m, r)
    B = dequant_int4(PqB, PsB, m, r)
    dots = np.sum(A * B, axis=0)
    den = np.maximum(np.sqrt(np.sum(A * A, axis=0)) * np.sqrt(np.sum(B * B, axis=0)), 1e-8)
    return float(np.mean(dots / den))


def column_energy(Pq, Ps, G_bits, m: int, n: int, r: int) -> np.ndarray:
    """e_k = ||p_k^T G||^2: how much of the gradient's energy (squared Frobenius norm) column k of the projection, as
    the step uses it, captures; the squared row norms of R = P^T G (Sec. 3.5)."""
    R = project(Pq, Ps, G_bits, m, n, r)
    return np.sum(R * R, axis=1)


def subspace_cossim_weighted(PqA, PsA, PqB, PsB, w, m: int, r: int) -> float:
    """sum_k w_k cos(a_k, b_k) / sum_k w_k: the column cosines of `subspace_cossim` under non-negative weights.

    Reading for the subspace refresh that replaces the SVD (Sec. 3.2 compares the columns of two SVD bases): orthogonal
    iteration started from the old projection keeps, among the directions that carry next to no gradient energy,
    whatever the old projection held, so their cosines say nothing about the gradient; weighting each column with
    the energy it captures makes the check follow the part of the subspace that matters to the method.  For a
    projection whose columns all carry comparable energy it is the plain mean."""
    A = dequant_int4(PqA, PsA, m, r)
    B = dequant_int4(PqB, PsB, m, r)
    dots = np.sum(A * B, axis=0)
    den = np.maximum(np.sqrt(np.sum(A * A, axis=0)) * np.sqrt(np.sum(B * B, axis=0)), 1e-8)
    w = np.asarray(w, dtype=np.float64)
    tot = float(np.sum(w))
    return float(np.sum(w * (dots / den)) / tot) if tot > 0 else 0.0


@dataclass
class Policy:
    """Adaptive lazy update of the SVD interval (Sec. 3.2): when the similarity
    stayed at or above the threshold over the previous k checks, the interval
    doubles."""
    interval: int = 200
    k: int = 1
    threshold: float = 0.4
    streak: int = 0
    next_refresh: int = 200
    last_cos: float = 0.0

    def update(self, cos: float) -> bool:
        self.last_cos = float(cos)
        self.streak = self.streak + 1 if cos >= self.threshold else 0
        doubled = False
        if self.streak >= self.k:
            self.interval *= 2
            self.streak = 0
            doubled = True
        self.next_refresh += self.interval
        return doubled


# --------------------------------------------------------------------------
# Subspace refresh (Sec. 3.2, Sec. 3.5: the projection matrix is recomputed
# from the current gradient every `interval` steps and stored as INT4)
# --------------------------------------------------------------------------
def refresh_svd(G_bits, m: int, n: int, r: int):
    """The definition the paper inherits from GaLore (Sec. 1, Sec. 3.2): P is
    made of the first r left singular vectors of the gradient.  Returns
    (P m x r, singular values).  Column signs are the library's (an SVD fixes
    them only up to sign): compare subspaces, not columns."""
    G = bf16_bits_to_f64(np.asarray(G_bits)).reshape(m, n)
    U, s, _ = np.linalg.svd(G, full_matrices=False)
    return U[:, :r], s


def orthonormalize(Y) -> np.ndarray:
    """Q of the QR factorisation Y = Q T with T upper triangular and a
    positive diagonal, i.e. Gram-Schmidt on the columns of Y in order.  For Y
    of full column rank this Q is unique.  The library's Householder QR is the
    step; its sign convention is normalised afterwards."""
    Y = np.asarray(Y, dtype=np.float64)
    Q, T = np.linalg.qr(Y, mode="reduced")
    sgn = np.where(np.diag(T) < 0, -1.0, 1.0)
    return Q * sgn[None, :]


def range_apply(G_bits, Z_bits, m: int, n: int, r: int) -> np.ndarray:
    """Y = G Z^T for the bf16 gradient G (m x n) and a bf16 r x n matrix Z
    (the projected gradient stored in BFloat16 like the gradient itself,
    Sec. 3.1): with Z = P^T G this is (G G^T) P, one step of the power
    method on the left singular subspace."""
    G = bf16_bits_to_f64(np.asarray(G_bits)).reshape(m, n)
    Z = bf16_bits_to_f64(np.asarray(Z_bits)).reshape(r, n)
    return G @ Z.T


def subspace_refresh(Pq, Ps, G_bits, m: int, n: int, r: int, iters: int = 1):
    """Replacement for the SVD of Sec. 3.2 (reading: the paper only asks for
    the dominant left singular subspace; orthogonal iteration started from the
    stored projection converges to the same singular vectors, in the same
    order, at the rate (sigma_{r+1}/sigma_r)^2 per pass).  One pass:
        R = dequant(P)^T G        (the projection of Sec. 3.5)
        Z = bf16(R)
        Y = G Z^T
        Q = orthonormalize(Y)
        P <- quant_int4(fl32(Q))  (Sec. 3.3: the projection is kept in INT4)
    Returns (Pq, Ps, Q of the last pass in fp64)."""
    Q = None
    for _ in range(iters):
        R = project(Pq, Ps, G_bits, m, n, r)
        Z_bits = f64_to_bf16_bits(R)
        Y = range_apply(G_bits, Z_bits, m, n, r)
        Q = orthonormalize(Y)
        Pq, Ps = quant_int4(Q.astype(np.float32))
    return Pq, Ps, Q


def subspace_refresh_check(Pq, Ps, G_bits, m: int, n: int, r: int, iters: int = 1):
    """`subspace_refresh` followed by the convergence check of Sec. 3.2 between the old and the new projection, the
    column cosines weighted with the gradient energy each NEW column captures (`column_energy`).
    Returns (Pq_new, Ps_new, cos)."""
    Pq1, Ps1, _ = subspace_refresh(Pq, Ps, G_bits, m, n, r, iters)
    e = column_energy(Pq1, Ps1, G_bits, m, n, r)
    return Pq1, Ps1, subspace_cossim_weighted(Pq, Ps, Pq1, Ps1, e, m, r)


# --------------------------------------------------------------------------
# INT8 linear layer (Appendix A: forward and backward of a layer whose weight
# is kept in INT8; the backward pass produces the gradient G the optimizer
# step consumes)
# --------------------------------------------------------------------------
def dequant_w_bf16(Wq, Ws) -> np.ndarray:
    """The weight as the layer's GEMMs see it (Appendix A: codes times scales in
    the activation dtype, zeros = 0): code * scale rounded to fp32, then stored
    as a bf16 operand - the same reading as for the projection matrix."""
    return bf16_rne(dequant_int8(Wq, Ws).astype(np.float32).astype(np.float64))


def int8_linear_forward(x_bits, Wq, Ws, bias_bits=None) -> np.ndarray:
    """y = x W^T (+ bias) (Appendix A, forward): x bf16 [tokens][n], W the m x n
    INT8 weight, y [tokens][m].  Returned unrounded in fp64; the layer stores it
    in the activation dtype (bf16)."""
    Wq = np.asarray(Wq)
    m, n = Wq.shape
    x = bf16_bits_to_f64(np.asarray(x_bits)).reshape(-1, n)
    y = x @ dequant_w_bf16(Wq, Ws).T
    if bias_bits is not None:
        y = y + bf16_bits_to_f64(np.asarray(bias_bits)).reshape(1, m)
    return y


def int8_linear_backward(dy_bits, x_bits, Wq, Ws):
    """(grad_input, grad_W) = (dy W, dy^T x) (Appendix A, backward): dy bf16
    [tokens][m], x bf16 [tokens][n].  Returned unrounded in fp64; both are
    stored in bf16 (Sec. 3.1: activations and gradients are BFloat16)."""
    Wq = np.asarray(Wq)
    m, n = Wq.shape
    dy = bf16_bits_to_f64(np.asarray(dy_bits)).reshape(-1, m)
    x = bf16_bits_to_f64(np.asarray(x_bits)).reshape(-1, n)
    return dy @ dequant_w_bf16(Wq, Ws), dy.T @ x


# --------------------------------------------------------------------------
# Right-side projection.  The paper takes its projection from GaLore (Sec. 2,
# Sec. 3.5), which projects a gradient from the left (R = P^T G, the form of
# `step`) or from the right (R = G Q with Q the first r RIGHT singular
# vectors, n x r; moments m x r; update alpha N Q^T).  Neither paper fixes the
# memory layout of a weight.  The reading taken here: a matrix that is
# projected from the right keeps its weight TRANSPOSED, S = W^T (n x m, INT8,
# blocks of 256 along each row of S, i.e. along a column of W), so that its
# blocks, its stochastic-rounding stream (element index j*m + i of S) and its
# kernels are those of a left-projected n x m matrix.  The functions below
# are written in the right-side form on the logical m x n matrix; that they
# agree with `step` on the transposed arrays is a test, not an assumption.
# Parity unpinned against the paper (it prints no right-side formula).
# --------------------------------------------------------------------------
def project_right(Qq, Qs, G_bits, m: int, n: int, r: int) -> np.ndarray:
    """R = G Q (m x r): Q the INT4 n x r projection matrix, dequantized like P."""
    Qd = dequant_p_bf16(Qq, Qs, n, r)
    G = bf16_bits_to_f64(np.asarray(G_bits).reshape(m, n))
    return G @ Qd


def backproject_right(Qq, Qs, Nb, n: int, r: int, alpha: float) -> np.ndarray:
    """U = alpha * N Q^T (m x n), Nb (m x r) being N already rounded to bf16."""
    Qd = dequant_p_bf16(Qq, Qs, n, r)
    return float(np.float32(alpha)) * (np.asarray(Nb, dtype=np.float64) @ Qd.T)


def step_right(Sq, Ss, G_bits, Qq, Qs, M, V, t: int, hp: HParams, seed: int, r: int) -> dict:
    """One step on a matrix projected from the right.  Sq, Ss: the weight as
    stored, S = W^T (n x m codes, n x ceil(m/256) scales); G_bits: the gradient
    of the logical weight W (m x n); M, V: moments m x r.  Returns R, M, V, N
    (m x r), U (m x n) and the new stored codes and scales (of S)."""
    Sq = np.asarray(Sq)
    n, m = Sq.shape
    R = project_right(Qq, Qs, G_bits, m, n, r)
    M1, V1, N = lowrank_adam(R, M, V, t, hp)
    Nb = bf16_rne(N)
    U = backproject_right(Qq, Qs, Nb, n, r, hp.alpha)
    newq, news = update_sr(Sq, Ss, U.T, hp.lr, seed, t)
    return dict(R=R, M=M1, V=V1, N=N, Nb=Nb, U=U, Sq=newq, Ss=news)


def int8_linear_t_forward(x_bits, Sq, Ss, bias_bits=None) -> np.ndarray:
    """y = x W^T (+ bias) with the weight stored transposed, S = W^T (n x m):
    y[t][o] = sum_i x[t][i] S[i][o]  (Appendix A, forward)."""
    Sq = np.asarray(Sq)
    n, m = Sq.shape
    x = bf16_bits_to_f64(np.asarray(x_bits)).reshape(-1, n)
    y = x @ dequant_w_bf16(Sq, Ss)
    if bias_bits is not None:
        y = y + bf16_bits_to_f64(np.asarray(bias_bits)).reshape(1, m)
    return y


def int8_linear_t_backward(dy_bits, x_bits, Sq, Ss):
    """(grad_input, grad_S) for the weight stored transposed (Appendix A,
    backward): grad_input = dy W = dy S^T (tokens x n); grad_S = (dy^T x)^T =
    x^T dy (n x m), the gradient in the layout of S."""
    Sq = np.asarray(Sq)
    n, m = Sq.shape
    dy = bf16_bits_to_f64(np.asarray(dy_bits)).reshape(-1, m)
    x = bf16_bits_to_f64(np.asarray(x_bits)).reshape(-1, n)
    return dy @ dequant_w_bf16(Sq, Ss).T, x.T @ dy


# --------------------------------------------------------------------------
# 8-bit Adam states (Sec. 3.5: the inner optimizer is Adam with its moments
# held in 8 bits).  The paper takes the format from a third-party library
# and does not define it; the format below is designed here after the
# published idea of block-wise dynamic quantization (a data type whose
# resolution is relative: a dynamic exponent plus a linear fraction, scaled by
# the block's absolute maximum).  Parity unpinned against the paper.
#
#   (rule added for the second moment: a positive value takes code 1 at least, see state8_quant)
#   block      256 consecutive elements of the flattened r x n state
#   scale      fp32 absmax of the block (0 for an all-zero block)
#   code       index into a sorted table of 8-bit values in [-1, 1] (first
#              moment) or [0, 1] (second moment), the nearest entry to
#              x / scale; ties go to the lower index
#   table      entry p >= 1 of the unsigned table: level L = floor(log2 p),
#              k = p - 2^L, value = 10^-(7-L) * (0.1 + 0.9 (k+1) / 2^L);
#              entry 0 is 0.  That is 2^L values spaced linearly over each
#              decade (10^-(8-L), 10^-(7-L)], 255 values from 1e-7 to 1.
#              The signed table has 7 magnitude bits (levels 0..6, 1e-6 to 1):
#              indices 0..126 the negatives from -1 up, 127 zero, 128..254 the
#              positives; index 255 is not used.
# --------------------------------------------------------------------------
def state8_table(signed: bool) -> np.ndarray:
    """The sorted table of representable values, as fp32 (255 entries signed, 256 unsigned)."""
    top = 6 if signed else 7
    pos = []
    for p in range(1, 2 ** (top + 1)):
        L = p.bit_length() - 1
        k = p - (1 << L)
        pos.append(10.0 ** -(top - L) * (0.1 + 0.9 * (k + 1) / (1 << L)))
    pos = np.array(pos, dtype=np.float64)
    full = np.concatenate([-pos[::-1], [0.0], pos]) if signed else np.concatenate([[0.0], pos])
    return full.astype(np.float32)


def _state8_mids(table32: np.ndarray) -> np.ndarray:
    t = table32.astype(np.float64)
    return (0.5 * (t[:-1] + t[1:])).astype(np.float32)


def state8_quant(x, signed: bool):
    """Block-wise dynamic 8-bit quantization of a flat state; all decisions in fp32.  Returns (codes uint8, scales fp32)."""
    x32 = np.asarray(x, dtype=np.float32).reshape(-1)
    nb = (x32.size + GROUP - 1) // GROUP
    mids = _state8_mids(state8_table(signed))
    codes = np.zeros(x32.size, dtype=np.uint8)
    scales = np.zeros(nb, dtype=np.float32)
    zero_code = 127 if signed else 0
    for b in range(nb):
        blk = x32[b * GROUP:(b + 1) * GROUP]
        a = np.float32(np.max(np.abs(blk)))
        scales[b] = a
        if a == 0:
            codes[b * GROUP:(b + 1) * GROUP] = zero_code
            continue
        inv = np.float32(1.0) / a                       # correctly rounded fp32 quotient
        xn = (blk * inv).astype(np.float32)
        c = np.searchsorted(mids, xn, side="left").astype(np.uint8)
        if not signed:
            # a positive second moment never rounds to zero: with V flushed to 0 while M survives (the signed table
            # reaches ten times further down), Adam's quotient would be formed from the newest gradient alone
            c = np.where((xn > 0) & (c == 0), np.uint8(1), c)
        codes[b * GROUP:(b + 1) * GROUP] = c
    return codes, scales


def state8_dequant(codes, scales, signed: bool) -> np.ndarray:
    """table[code] * scale as an fp32 product, returned in fp64."""
    t = state8_table(signed)
    c = np.asarray(codes).reshape(-1)
    s = np.repeat(np.asarray(scales, dtype=np.float32), GROUP)[:c.size]
    return (t[np.minimum(c, t.size - 1)] * s).astype(np.float32).astype(np.float64)


def lowrank_adam8(R, Mq, Ms, Vq, Vs, t: int, hp: HParams):
    """Adam on the low-rank gradient with 8-bit states (Sec. 3.5): the states are dequantized, updated exactly
    as in lowrank_adam, and quantized again.  Returns (Mq', Ms', Vq', Vs', N, M', V') with N, M', V' in fp64
    (M', V' before quantization)."""
    R = np.asarray(R, dtype=np.float64)
    M = state8_dequant(Mq, Ms, True).reshape(R.shape)
    V = state8_dequant(Vq, Vs, False).reshape(R.shape)
    M1, V1, N = lowrank_adam(R, M, V, t, hp)
    Mq1, Ms1 = state8_quant(M1, True)
    Vq1, Vs1 = state8_quant(V1, False)
    return Mq1, Ms1, Vq1, Vs1, N, M1, V1


# --------------------------------------------------------------------------
# Asymmetric (zero-point) INT8 weights.  Sec. 3.1 writes the quantizer with a
# zero point, W_q = clamp(round(W/s) + z, -2^(n-1), 2^(n-1)-1), s and z per
# block; Appendix A dequantizes W = (W_q - zeros) * scales.  Neither says how
# s and z follow from the block.  The reading taken here (parity unpinned):
# the usual min/max rule over a range that contains zero,
#     lo = min(0, min x), hi = max(0, max x), s = (hi - lo)/255,
#     z = clamp(-128 - round(lo/s), -128, 127),
# so that lo maps to -128, hi to about 127 and 0 to the code z exactly.  As in
# the symmetric quantizer W/s is the fp32 product with the fp32 reciprocal
# 255/(hi - lo), and every decision step (min, max, difference, the two
# quotients, the products) is taken in fp32.  A block that is all zero gets
# s = 0, z = 0 and codes 0.  Zero points are whole numbers in [-128, 127]
# (kept as fp32 next to the scales).
# --------------------------------------------------------------------------
def _zp_params(lo32: np.ndarray, hi32: np.ndarray):
    """(s, 1/s, z) of each block from its fp32 minimum and maximum (zero already included)."""
    rng = (hi32.astype(np.float32) - lo32.astype(np.float32)).astype(np.float32)
    r64 = rng.astype(np.float64)
    with np.errstate(divide="ignore", invalid="ignore"):
        s = np.where(r64 > 0, r64 / 255.0, 0.0).astype(np.float32)
        inv = np.where(r64 > 0, 255.0 / r64, 0.0).astype(np.float32)
    tz = (lo32.astype(np.float32) * inv).astype(np.float32)
    z = np.where(r64 > 0, np.clip(-128.0 - np.rint(tz.astype(np.float64)), -128, 127), 0.0)
    return s, inv, z.astype(np.float32)


def quant_int8_zp(x):
    """Quant_8 with a zero point (Sec. 3.1 eq.), blocks of 256 along each row.
    Returns int8 codes [rows][cols], fp32 scales and fp32 zero points
    [rows][ceil(cols/256)]."""
    x = np.asarray(x, dtype=np.float32)
    rows, cols = x.shape
    ng = (cols + GROUP - 1) // GROUP
    q = np.zeros((rows, cols), dtype=np.int8)
    scales = np.zeros((rows, ng), dtype=np.float32)
    zeros = np.zeros((rows, ng), dtype=np.float32)
    for g in range(ng):
        blk = x[:, g * GROUP:(g + 1) * GROUP]
        lo = np.minimum(np.min(blk, axis=1), 0).astype(np.float32)
        hi = np.maximum(np.max(blk, axis=1), 0).astype(np.float32)
        s, inv, z = _zp_params(lo, hi)
        scales[:, g], zeros[:, g] = s, z
        t = (blk * inv[:, None]).astype(np.float32)
        q[:, g * GROUP:(g + 1) * GROUP] = np.clip(np.rint(t.astype(np.float64)) + z[:, None], -128, 127).astype(np.int8)
    return q, scales, zeros


def dequant_int8_zp(q, scales, zeros) -> np.ndarray:
    """W = (W_q - zeros) * scales (Appendix A), exact in fp64."""
    q = np.asarray(q)
    rows, cols = q.shape
    s = np.repeat(np.asarray(scales, dtype=np.float64), GROUP, axis=1)[:, :cols]
    z = np.repeat(np.asarray(zeros, dtype=np.float64), GROUP, axis=1)[:, :cols]
    return (q.astype(np.float64) - z) * s


def dequant_w_zp_bf16(Wq, Ws, Wz) -> np.ndarray:
    """The zero-point weight as a GEMM operand: (code - zero) * scale rounded to fp32, then to bf16."""
    return bf16_rne(dequant_int8_zp(Wq, Ws, Wz).astype(np.float32).astype(np.float64))


def update_sr_zp(Wq, Ws, Wz, U, lr: float, seed: int, t: int, n_total: int | None = None, col0: int = 0):
    """The INT8 update of Sec. 3.4/3.5 on a zero-point weight: x = (W_q - z) s -
    lr U; per block new (s', z') from min/max as in quant_int8_zp; code =
    clamp(F_SR(x/s') + z', -128, 127) with the draw u(seed, t, i*n_total + col0 + j)
    (a slice of columns of a wider matrix, as in update_sr).
    Returns (codes, scales, zeros)."""
    Wq = np.asarray(Wq)
    m, n = Wq.shape
    n_total = n if n_total is None else n_total
    x = dequant_int8_zp(Wq, Ws, Wz) - float(np.float32(lr)) * np.asarray(U, dtype=np.float64)
    x32 = x.astype(np.float32)
    ng = (n + GROUP - 1) // GROUP
    newq = np.zeros((m, n), dtype=np.int8)
    news = np.zeros((m, ng), dtype=np.float32)
    newz = np.zeros((m, ng), dtype=np.float32)
    ii = np.arange(m, dtype=np.uint64)[:, None]
    for g in range(ng):
        c0, c1 = g * GROUP, min((g + 1) * GROUP, n)
        blk = x32[:, c0:c1]
        lo = np.minimum(np.min(blk, axis=1), 0).astype(np.float32)
        hi = np.maximum(np.max(blk, axis=1), 0).astype(np.float32)
        s, inv, z = _zp_params(lo, hi)
        news[:, g], newz[:, g] = s, z
        tq = (blk * inv[:, None]).astype(np.float32)
        idx = ii * np.uint64(n_total) + np.arange(col0 + c0, col0 + c1, dtype=np.uint64)[None, :]
        u = sr_uniform(seed, t, idx)
        newq[:, c0:c1] = np.clip(sr_round(tq, u) + z[:, None].astype(np.float64), -128, 127).astype(np.int8)
    return newq, news, newz


def step_zp(Wq, Ws, Wz, G_bits, Pq, Ps, M, V, t: int, hp: HParams, seed: int, r: int,
            n_total: int | None = None, col0: int = 0) -> dict:
    """`step` on a zero-point weight: only the weight's format differs (a slice of
    columns of a wider matrix can be stepped alone, as in `step`)."""
    Wq = np.asarray(Wq)
    m, n = Wq.shape
    R = project(Pq, Ps, G_bits, m, n, r)
    M1, V1, N = lowrank_adam(R, M, V, t, hp)
    Nb = bf16_rne(N)
    U = backproject(Pq, Ps, Nb, m, r, hp.alpha)
    newq, news, newz = update_sr_zp(Wq, Ws, Wz, U, hp.lr, seed, t, n_total, col0)
    return dict(R=R, M=M1, V=V1, N=N, Nb=Nb, U=U, Wq=newq, Ws=news, Wz=newz)


def int8_linear_zp_forward(x_bits, Wq, Ws, Wz, bias_bits=None) -> np.ndarray:
    """Appendix A forward with zeros: y = x ((W_q - zeros) * scales)^T (+ bias)."""
    Wq = np.asarray(Wq)
    m, n = Wq.shape
    x = bf16_bits_to_f64(np.asarray(x_bits)).reshape(-1, n)
    y = x @ dequant_w_zp_bf16(Wq, Ws, Wz).T
    if bias_bits is not None:
        y = y + bf16_bits_to_f64(np.asarray(bias_bits)).reshape(1, m)
    return y


def int8_linear_zp_backward(dy_bits, x_bits, Wq, Ws, Wz):
    """Appendix A backward with zeros: (dy W, dy^T x)."""
    Wq = np.asarray(Wq)
    m, n = Wq.shape
    dy = bf16_bits_to_f64(np.asarray(dy_bits)).reshape(-1, m)
    x = bf16_bits_to_f64(np.asarray(x_bits)).reshape(-1, n)
    return dy @ dequant_w_zp_bf16(Wq, Ws, Wz), dy.T @ x
