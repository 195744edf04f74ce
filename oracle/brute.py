"""Pure-Python brute force of the Q-GaLore step for tiny matrices.

TEST INFRASTRUCTURE ONLY.  Explicit loops over Python floats (fp64) and Python
integers, no numpy: a second, independent statement of the same steps, used to
pin oracle/qgalore.py on sizes of a few hundred elements.  fp32 roundings go
through `struct`, bf16 roundings through `math.frexp` and round-half-even.
"""
from __future__ import annotations

import math
import struct

GROUP = 256


def fl32(x: float) -> float:
    """Nearest fp32 value of a Python float."""
    return struct.unpack("f", struct.pack("f", x))[0]


def bf16(x: float) -> float:
    """Nearest bf16 value (8 significant bits, ties to even) of a normal-range float."""
    if x == 0.0 or not math.isfinite(x):
        return x
    m, e = math.frexp(x)                 # x = m * 2^e, 0.5 <= |m| < 1
    return math.ldexp(round(m * 256.0), e - 8)   # round() is half-to-even


def bf16_from_bits(b: int) -> float:
    return struct.unpack("f", struct.pack("I", (b & 0xFFFF) << 16))[0]


def mix32(x: int) -> int:
    x &= 0xFFFFFFFF
    x ^= x >> 16
    x = (x * 0x7FEB352D) & 0xFFFFFFFF
    x ^= x >> 15
    x = (x * 0x846CA68B) & 0xFFFFFFFF
    x ^= x >> 16
    return x


def uniform(seed: int, step: int, idx: int) -> float:
    key = 0x9E3779B9
    for w in (seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF, step & 0xFFFFFFFF, (step >> 32) & 0xFFFFFFFF,
              (idx >> 32) & 0xFFFFFFFF):
        key = mix32(((key ^ w) + 0x9E3779B9) & 0xFFFFFFFF)
    return (mix32(key ^ (idx & 0xFFFFFFFF)) >> 8) / 16777216.0


def quant_block(xs, qmax: int):
    """One block: (codes, scale) with s = a/qmax, codes = clamp(rne(x * (qmax/a)))."""
    a = max((abs(fl32(v)) for v in xs), default=0.0)
    if a == 0.0:
        return [0] * len(xs), 0.0
    s = fl32(a / qmax)
    inv = fl32(qmax / a)
    codes = []
    for v in xs:
        t = fl32(fl32(v) * inv)
        q = int(round(t))                # half-to-even
        codes.append(max(-qmax - 1, min(qmax, q)))
    return codes, s


def quant_int8_rows(x):
    """x: list of rows -> (codes rows, scales rows), blocks of 256 within a row."""
    qs, ss = [], []
    for row in x:
        qrow, srow = [], []
        for c0 in range(0, len(row), GROUP):
            c, s = quant_block(row[c0:c0 + GROUP], 127)
            qrow += c
            srow.append(s)
        qs.append(qrow)
        ss.append(srow)
    return qs, ss


def quant_int4_flat(x):
    """x: list of rows -> (codes rows, flat scales), blocks of 256 of the flat array."""
    cols = len(x[0])
    flat = [v for row in x for v in row]
    codes, scales = [], []
    for c0 in range(0, len(flat), GROUP):
        c, s = quant_block(flat[c0:c0 + GROUP], 7)
        codes += c
        scales.append(s)
    return [codes[i * cols:(i + 1) * cols] for i in range(len(x))], scales


def step(Wq, Ws, Gbits, Pcodes, Ps, M, V, t, hp, seed):
    """One step with lists of lists.  hp = (beta1, beta2, eps, lr, alpha) already
    fp32-valued.  Returns dict of lists: R, M, V, Nb, U, Wq, Ws."""
    b1, b2, eps, lr, alpha = hp
    m, n, r = len(Wq), len(Wq[0]), len(Pcodes[0])
    Pd = [[bf16(fl32(Pcodes[i][k] * Ps[(i * r + k) // GROUP])) for k in range(r)] for i in range(m)]
    G = [[bf16_from_bits(Gbits[i][j]) for j in range(n)] for i in range(m)]
    R = [[math.fsum(Pd[i][k] * G[i][j] for i in range(m)) for j in range(n)] for k in range(r)]
    M1 = [[b1 * M[k][j] + (1.0 - b1) * R[k][j] for j in range(n)] for k in range(r)]
    V1 = [[b2 * V[k][j] + (1.0 - b2) * R[k][j] * R[k][j] for j in range(n)] for k in range(r)]
    c1, c2 = 1.0 - b1 ** t, 1.0 - b2 ** t
    Nb = [[bf16((M1[k][j] / c1) / (math.sqrt(V1[k][j] / c2) + eps)) for j in range(n)] for k in range(r)]
    U = [[alpha * math.fsum(Pd[i][k] * Nb[k][j] for k in range(r)) for j in range(n)] for i in range(m)]
    newq, news = [], []
    for i in range(m):
        x = [fl32(Wq[i][j] * Ws[i][j // GROUP] - lr * U[i][j]) for j in range(n)]
        qrow, srow = [], []
        for c0 in range(0, n, GROUP):
            blk = x[c0:c0 + GROUP]
            a = max(abs(v) for v in blk)
            if a == 0.0:
                qrow += [0] * len(blk)
                srow.append(0.0)
                continue
            s = fl32(a / 127.0)
            inv = fl32(127.0 / a)
            for jj, v in enumerate(blk):
                tq = fl32(v * inv)
                u = uniform(seed, t, i * n + c0 + jj)
                q = math.floor(fl32(tq + u))
                qrow.append(max(-128, min(127, q)))
            srow.append(s)
        newq.append(qrow)
        news.append(srow)
    return dict(R=R, M=M1, V=V1, Nb=Nb, U=U, Wq=newq, Ws=news)
