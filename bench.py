#!/usr/bin/env python3
"""Benchmark of the Q-GaLore optimizer step on one MI355X.

A "step" is one pass of the whole hot path (project -> Adam -> back-project + INT8 stochastic-rounding
update) over every linear weight of the workload, by the two grouped launches of qg_step_many (projection with
Adam in its epilogue; back-projection with the update in its epilogue).  The unfused projection and Adam launches
are timed too, after the timed region, for their own roofline fractions.  The default workload is the one the
headline metric is quoted on: LLaMA-7B shapes (224 matrices, r = 1024).
Inputs are synthetic, generated on the device before the timed region, and stay resident in HBM.

Prints ONE JSON line: metric, value (ms per step), roofline (the slower of the two launches against the bf16 MFMA
peak, with measured HBM traffic), kernels (every launch with its rate), ceilings (what the machine sustained in the
same run), other_configs (configs 0-3 next to their bounds), rank_sweep and update_pass (config 3's sweep; the update
pass where memory bounds it), cpu_baseline (the oracle on a sample of the workload).  Other modes: --refresh, --linear, --rsweep,
--config N, --pad-rows, --zero-points.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0    # MI355X dense bf16 MFMA, published
PEAK_HBM_GBS = 8000.0        # MI355X HBM3E, published

WORKLOADS = {
    0: "config0: one 512x512 matrix, r=128",
    1: "LLaMA-130M shapes: 84 matrices, r=256",
    2: "LLaMA-350M shapes: 168 matrices, r=256",
    3: "LLaMA-1B shapes: 168 matrices, r=512",
    4: "LLaMA-7B shapes: 224 matrices (32 layers x [4x 4096x4096, 2x 11008x4096, 1x 4096x11008]), r=1024, "
       "INT8 W / bf16 G / INT4 P, group 256",
}


def measured_traffic(kernel: str, config: int):
    """(HBM bytes per launch of `kernel`, what the figure was profiled at) from the committed rocprofv3 --pmc summary
    (FETCH_SIZE + WRITE_SIZE, each scaled by a plain copy of known size), or (None, None) if there is no summary for
    this workload.  The summary names the source revision of the kernels it was taken from (`profiled_at`): a figure
    from an older revision is stale and says so."""
    if config != 4:
        return None, None
    path = os.path.join(ROOT, "profiles", "grouped_step_llama7b_hbm_traffic.txt")
    traffic, stamp = None, None
    try:
        for line in open(path):
            f = line.split()
            if len(f) == 3 and f[0] == "traffic_bytes" and f[1] == kernel:
                traffic = int(f[2])
            if len(f) >= 2 and f[0] == "profiled_at":
                stamp = " ".join(f[1:])
    except OSError:
        pass
    return traffic, stamp


def kernel_source_digest():
    """sha256 (first 12 hex digits) over the GEMM kernel sources: what `profiled_at` in a profile summary refers to."""
    import hashlib
    h = hashlib.sha256()
    for name in ("qg_gemm_kernels.h", "qg_gemm.hip", "qg_common.h"):
        h.update(open(os.path.join(ROOT, "paper_2407_08296_amd", "csrc", name), "rb").read())
    return h.hexdigest()[:12]


def algorithmic_work(shapes):
    """Flops and HBM bytes each kernel must move for these (m, n, r) matrices (no re-reads counted)."""
    flops = sum(2 * m * n * r for m, n, r in shapes)
    p_bytes = lambda m, r: m * r // 2 + 4 * ((m * r + 255) // 256)
    proj = sum(2 * m * n + p_bytes(m, r) + 4 * r * n for m, n, r in shapes)
    adam = sum(22 * r * n for m, n, r in shapes)
    bp = sum(2 * m * n + 8 * m * ((n + 255) // 256) + p_bytes(m, r) + 2 * r * n for m, n, r in shapes)
    return flops, proj, adam, bp


def pitched(t, ld):
    """Copy of the 2-D tensor t with rows ld elements apart (padding zero-filled)."""
    import torch
    out = torch.zeros((t.shape[0], ld), dtype=t.dtype, device=t.device)
    out[:, :t.shape[1]].copy_(t)
    return out


def build_state(config: int, device, pad_rows: bool = False, zero_points: bool = False):
    """Device-resident synthetic state of every matrix of the workload.

    W ~ N(0, 0.02) quantized by qg_quant_int8; G = A B^T + E (rank 16 plus noise) in bf16; one orthonormal P per
    distinct (m, r) (host QR, quantized by qg_quant_int4) shared by the matrices of that shape - values do not
    affect timing.  Generated with torch's device RNG (the host generators of the parity tests would take minutes
    for 6.5e9 elements); distributions and shapes are the same.
    """
    import torch

    from paper_2407_08296_amd import inputs as I
    from paper_2407_08296_amd import qgalore as qg

    gen = torch.Generator(device=device)
    gen.manual_seed(0)
    pcache = {}
    mats = []
    for (layer, kind, m, n, r) in I.config_matrices(config):
        if (m, r) not in pcache:
            P = torch.from_numpy(I.projection_f32(m, r)).to(device)
            pcache[(m, r)] = qg.quant_int4(P)
        Pq, Ps = pcache[(m, r)]
        W = torch.randn((m, n), generator=gen, device=device, dtype=torch.float32) * 0.02
        Wz = None
        if zero_points:
            Wq, Ws, Wz = qg.quant_int8_zp(W)
        else:
            Wq, Ws = qg.quant_int8(W)
        del W
        A = torch.randn((m, 16), generator=gen, device=device) * 0.01
        B = torch.randn((n, 16), generator=gen, device=device) * 0.01
        G = torch.randn((m, n), generator=gen, device=device) * 1e-4
        G.addmm_(A, B.t())
        Gb = G.to(torch.bfloat16)
        del G
        ld = (n + 15) // 16 * 16 if pad_rows and n % 16 else 0   # rows 16-byte aligned in every array
        if ld:
            Gb, Wq = pitched(Gb, ld), pitched(Wq.view(m, n), ld)
        w = ld or n
        mats.append(qg.MatrixState(m, n, r, Pq, Ps, Gb, Wq, Ws,
                                   torch.zeros((r, w), dtype=torch.float32, device=device),
                                   torch.zeros((r, w), dtype=torch.float32, device=device),
                                   torch.empty((r, w), dtype=torch.float32, device=device),
                                   torch.empty((r, w), dtype=torch.bfloat16, device=device), ld=ld, Wz=Wz))
    torch.cuda.synchronize()
    return mats


def cpu_baseline(config: int, shapes):
    """The fp64 oracle, as it stands, timed on this host on a bounded sample of the workload."""
    import numpy as np

    from oracle import qgalore as Q
    from paper_2407_08296_amd import inputs as I

    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = len(os.sched_getaffinity(0))
    if config >= 2:
        layers = 3 if config == 4 else 6          # about 10-30 s of host time
        sample = shapes[:7 * layers]
        note = f"{layers} decoder layers ({7 * layers} matrices), scaled by sum(m*n*r) to the whole step"
    else:
        sample = shapes
        note = "the whole step"
    total = 0.0
    for i, (m, n, r) in enumerate(sample):
        Wq, Ws = Q.quant_int8(I.weight_f32(m, n, kind=i))
        Pq, Ps = Q.quant_int4(I.projection_f32(m, r, kind=i))
        Gb = I.gradient_bf16(m, n, 1, kind=i)
        M = np.zeros((r, n)); V = np.zeros((r, n))
        t0 = time.perf_counter()
        Q.step(Wq, Ws, Gb, Pq, Ps, M, V, 1, Q.HParams(), seed=0, r=r)
        total += time.perf_counter() - t0
    scale = sum(m * n * r for m, n, r in shapes) / sum(m * n * r for m, n, r in sample)
    return {"value": total * scale * 1e3, "unit": "ms", "cores": int(threads), "kind": "oracle",
            "sample": note, "sample_seconds": total, "host_cpus": len(os.sched_getaffinity(0))}


def timed_ms(f, reps):
    import torch
    f(); torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        f()
    b.record(); torch.cuda.synchronize()
    return a.elapsed_time(b) / reps


def step_bounds(shapes):
    """(MFMA-bound ms, HBM-bound ms) of one step over these matrices at the published peaks: both GEMMs' flops, and
    the algorithmic bytes of the two fused launches (no R round trip)."""
    flops, b_proj, b_adam, b_bp = algorithmic_work(shapes)
    b_fused = b_proj + b_adam - sum(8 * r * n for m, n, r in shapes)
    return 2 * flops / PEAK_BF16_TFLOPS / 1e9, (b_fused + b_bp) / PEAK_HBM_GBS / 1e6


def other_configs(device):
    """The step over configs 0-3 (the smaller workloads), each next to its roofline bounds.  Config 3 is run with the
    row pitch its `down` matrices need for aligned rows (n = 5461) and, for comparison, with dense rows."""
    import dataclasses

    import torch

    from paper_2407_08296_amd import inputs as I
    from paper_2407_08296_amd import qgalore as qg

    hp = qg.hparams()
    rows = []
    for config, pad in ((0, False), (1, False), (2, False), (3, True), (3, False)):
        shapes = [(m, n, r) for (_, _, m, n, r) in I.config_matrices(config)]
        mats = build_state(config, device, pad_rows=pad)
        plan = qg.StepPlan([dataclasses.replace(s_, R=None) for s_ in mats])
        tt = [0]

        def one():
            tt[0] += 1
            qg.step_many(plan, hp, 0, tt[0])
        ms = timed_ms(one, 20)
        mfma_ms, hbm_ms = step_bounds(shapes)
        bound = max(mfma_ms, hbm_ms)
        rows.append({"config": config, "workload": WORKLOADS[config], "row_layout": "pitch 16" if pad else "dense",
                     "ms_per_step": ms, "mfma_bound_ms": mfma_ms, "hbm_bound_ms": hbm_ms,
                     "bound": "mfma" if mfma_ms >= hbm_ms else "hbm", "frac_of_bound": bound / ms,
                     "note": ("latency-bound: two dependent launches of four tiles each; a tile's K loop and epilogue set the time "
                              "(replayed from a captured graph the step takes the same 35-39 us)") if config == 0 else None})
        del plan, mats
        torch.cuda.empty_cache()
    return rows


def rank_sweep(device):
    """Config 3's sweep: 2048 x 5461 matrices (24 copies, stored with a row pitch of 5472: 16-byte aligned rows) through
    the grouped launches for r in {128, 256, 512, 1024}, per matrix, next to the two bounds; and the update pass
    where it is bound by memory rather than by the matrix cores (r = 128)."""
    import torch

    from paper_2407_08296_amd import inputs as I
    from paper_2407_08296_amd import qgalore as qg

    m, n, copies = 2048, 5461, 24
    ld = (n + 15) // 16 * 16
    hp = qg.hparams()
    Wq, Ws = qg.quant_int8(torch.randn((m, n), device=device) * 0.02)
    G = (torch.randn((m, n), device=device) * 1e-3).to(torch.bfloat16)
    rows = []
    for r in (128, 256, 512, 1024):
        Pq, Ps = qg.quant_int4(torch.from_numpy(I.projection_f32(m, r)).to(device))
        gm = [qg.MatrixState(m, n, r, Pq, Ps, pitched(G, ld), pitched(Wq.view(m, n), ld), Ws.clone(),
                             torch.zeros((r, ld), device=device), torch.zeros((r, ld), device=device), None,
                             torch.zeros((r, ld), dtype=torch.bfloat16, device=device), ld=ld) for _ in range(copies)]
        plan = qg.StepPlan(gm)
        pa = timed_ms(lambda: qg.project_adam_many(plan, hp, 2, False), 10) / copies
        bp = timed_ms(lambda: qg.backproject_update_sr_many(plan, hp, 0, 2), 10) / copies
        flops, b_proj, b_adam, b_bp = algorithmic_work([(m, n, r)])
        b_fused = b_proj + b_adam - 8 * r * n
        rows.append({"r": r, "project_adam_us": pa * 1e3, "backproject_update_us": bp * 1e3,
                     "mfma_bound_us_per_gemm": flops / PEAK_BF16_TFLOPS / 1e6,
                     "hbm_bound_project_adam_us": b_fused / PEAK_HBM_GBS / 1e3,
                     "hbm_bound_backproject_update_us": b_bp / PEAK_HBM_GBS / 1e3,
                     "project_adam_frac_mfma": flops / pa / 1e9 / PEAK_BF16_TFLOPS,
                     "project_adam_frac_hbm": b_fused / pa / 1e6 / PEAK_HBM_GBS,
                     "backproject_update_frac_mfma": flops / bp / 1e9 / PEAK_BF16_TFLOPS,
                     "backproject_update_frac_hbm": b_bp / bp / 1e6 / PEAK_HBM_GBS})
        del plan, gm
    # the update pass (dequantize, subtract, block absmax, stochastic rounding, requantize) costs UPDATE_VALU_PER_ELEMENT
    # vector instructions per weight element: next to the HBM bound it has a bound of its own from the vector ALUs
    low = rows[0]
    alu_us = m * n * UPDATE_VALU_PER_ELEMENT / PEAK_VALU_LANE_OPS * 1e6
    update = {"where": "r = 128 (HBM-bound side of the crossover), 2048 x 5461, grouped over 24 matrices",
              "us_per_matrix": low["backproject_update_us"], "frac_hbm": low["backproject_update_frac_hbm"],
              "GB/s": low["backproject_update_frac_hbm"] * PEAK_HBM_GBS,
              "alu_bound_us": alu_us, "frac_alu_bound": alu_us / low["backproject_update_us"],
              "note": f"{UPDATE_VALU_PER_ELEMENT} vector instructions per element (8 of them the counter hash) against "
                      "256 CUs x 64 lanes x 2.4 GHz: the update pass alone cannot run faster than this"}
    return {"m": m, "n": n, "ld": ld, "copies": copies, "rows": rows}, update


UPDATE_VALU_PER_ELEMENT = 17             # counted in the compiled epilogue: 3.5 (x = code*s - lr*alpha*U, absmax) + 13.5
PEAK_VALU_LANE_OPS = 256 * 64 * 2.4e9    # vector lanes x clock: one 32-bit operation per lane per cycle


def linear_bench(args, device):
    """Forward and backward of the INT8 linear layer over the seven weights of one decoder layer."""
    import torch

    from paper_2407_08296_amd import inputs as I
    from paper_2407_08296_amd import qgalore as qg

    T = args.tokens
    layer = [(m, n) for (l, _, m, n, _) in I.config_matrices(args.config) if l == 0]
    g = torch.Generator(device=device).manual_seed(0)
    ops = []
    for (m, n) in layer:
        Wq, Ws = qg.quant_int8(torch.randn((m, n), generator=g, device=device) * 0.02)
        x = torch.randn((T, n), generator=g, device=device).to(torch.bfloat16)
        dy = (torch.randn((T, m), generator=g, device=device) * 0.05).to(torch.bfloat16)
        ops.append((m, n, Wq, Ws, x, dy))

    def timed(f, reps):
        f()
        torch.cuda.synchronize()
        a = torch.cuda.Event(enable_timing=True); b = torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            f()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    reps = max(1, args.steps)
    flop = sum(2.0 * T * m * n for m, n in layer)
    legs = {
        "forward": lambda: [qg.int8_linear_forward(x, Wq, Ws) for (m, n, Wq, Ws, x, dy) in ops],
        "grad_input": lambda: [qg.int8_linear_backward(dy, None, Wq, Ws, m, n, want_G=False) for (m, n, Wq, Ws, x, dy) in ops],
        "grad_W": lambda: [qg.int8_linear_backward(dy, x, None, None, m, n, want_dx=False) for (m, n, Wq, Ws, x, dy) in ops],
    }
    out = {"metric": "INT8 linear layer ms per decoder layer (forward + backward)", "unit": "ms", "n_gpus": 1,
           "higher_is_better": False, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": WORKLOADS[args.config], "tokens": T, "weights": [f"{m}x{n}" for m, n in layer]},
           "kernels": {}}
    total = 0.0
    for name, f in legs.items():
        ms = timed(f, reps)
        total += ms
        out["kernels"][name] = {"ms": ms, "TFLOP/s": flop / ms / 1e9, "frac_mfma": flop / ms / 1e9 / PEAK_BF16_TFLOPS}
    out["value"] = total
    out["mfma_bound_ms"] = 3 * flop / PEAK_BF16_TFLOPS / 1e9
    # the same layer with every weight stored transposed (the storage of right-projected matrices): same flops, the
    # forward pass then has the operand layout of grad_input and vice versa
    tops = [(m, n, *qg.quant_int8(torch.randn((n, m), generator=g, device=device) * 0.02), x, dy)
            for (m, n, _, _, x, dy) in ops]
    tlegs = {
        "forward": lambda: [qg.int8_linear_t_forward(x, Sq, Ss) for (m, n, Sq, Ss, x, dy) in tops],
        "grad_input": lambda: [qg.int8_linear_t_backward(dy, None, Sq, Ss, m, n, want_G=False) for (m, n, Sq, Ss, x, dy) in tops],
        "grad_W": lambda: [qg.int8_linear_t_backward(dy, x, None, None, m, n, want_dx=False) for (m, n, Sq, Ss, x, dy) in tops],
    }
    out["transposed_storage_ms"] = {name: timed(f, reps) for name, f in tlegs.items()}
    del tops
    # the vendor GEMM (torch.mm -> hipBLASLt) on the same shapes with a bf16 weight, no dequantization: for scale
    if not args.no_cpu_baseline:                # the oracle as it stands on one small layer, next to the library on the same
        import numpy as np

        from oracle import qgalore as Q
        tk, mk, nk = 256, 768, 768
        Wq_h, Ws_h = Q.quant_int8(I.weight_f32(mk, nk))
        rs = np.random.default_rng(0)
        xb = Q.f64_to_bf16_bits(rs.standard_normal((tk, nk)))
        dyb = Q.f64_to_bf16_bits(rs.standard_normal((tk, mk)) * 0.05)
        t0 = time.perf_counter()
        Q.int8_linear_forward(xb, Wq_h, Ws_h)
        Q.int8_linear_backward(dyb, xb, Wq_h, Ws_h)
        t_or = time.perf_counter() - t0
        xd = torch.from_numpy(xb.view(np.int16).reshape(tk, nk)).to(device)
        dyd = torch.from_numpy(dyb.view(np.int16).reshape(tk, mk)).to(device)
        Wqd, Wsd = torch.from_numpy(Wq_h).to(device), torch.from_numpy(Ws_h).to(device)
        t_gpu = timed(lambda: (qg.int8_linear_forward(xd, Wqd, Wsd), qg.int8_linear_backward(dyd, xd, Wqd, Wsd, mk, nk)), 10)
        out["cpu_baseline"] = {"kind": "oracle", "sample": "forward + backward of one 768x768 weight at 256 tokens",
                               "oracle_ms": t_or * 1e3, "gpu_ms_same_sample": t_gpu, "host_cpus": len(os.sched_getaffinity(0))}
    Wb = [(x, (torch.randn((m, n), generator=g, device=device) * 0.02).to(torch.bfloat16), dy) for (m, n, _, _, x, dy) in ops]
    out["vendor_bf16_gemm_ms"] = {
        "forward": timed(lambda: [torch.mm(x, W.t()) for (x, W, dy) in Wb], reps),
        "grad_input": timed(lambda: [torch.mm(dy, W) for (x, W, dy) in Wb], reps),
        "grad_W": timed(lambda: [torch.mm(dy.t(), x) for (x, W, dy) in Wb], reps)}
    return out


PEAK_FP64_TFLOPS = 78.6      # MI355X fp64 matrix (and vector) peak, published


def refresh_bench(args, shapes, mats):
    """One subspace refresh (one pass of orthogonal iteration, Cholesky QR twice, INT4 requantization, cosine check)
    of every matrix of the workload, one qg_subspace_refresh call per matrix on one shared workspace."""
    import torch

    from paper_2407_08296_amd import qgalore as qg

    L = qg.lib()
    dev = mats[0].G.device
    groups = {}
    for s in mats:
        groups.setdefault((s.m, s.n, s.r), []).append(s)
    ws = torch.empty((max(L.qg_refresh_workspace_bytes(len(g), m, n, r) for (m, n, r), g in groups.items()),),
                     dtype=torch.uint8, device=dev)
    outs = {k: ([torch.empty_like(s.Pq) for s in g], [torch.empty_like(s.Ps) for s in g]) for k, g in groups.items()}

    def one_round(read_info=False):
        """Every matrix of the workload once: one batched call per distinct shape."""
        bad = 0
        for (m, n, r), g in groups.items():
            _, _, _, info, _ = qg.subspace_refresh_many([s.Pq for s in g], [s.Ps for s in g], [s.G for s in g], m, n, r,
                                                        1, workspace=ws, out=outs[(m, n, r)])
            if read_info:
                bad += int((info != 0).sum().item())
        return bad

    def timed(f, reps):
        f()
        torch.cuda.synchronize()
        a = torch.cuda.Event(enable_timing=True); b = torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            f()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    bad = one_round(read_info=True)                     # warm-up, and the only round that reads `info` back
    torch.cuda.synchronize()
    rounds = max(1, min(args.steps, 3))
    t0 = time.perf_counter()
    ms = timed(one_round, rounds)
    wall = (time.perf_counter() - t0) / (rounds + 1) * 1e3
    per_shape = {}
    for (m, n, r), g in groups.items():
        s = g[0]
        one = timed(lambda: qg.subspace_refresh(s.Pq, s.Ps, s.G, m, n, r, 1, workspace=ws), 3)
        many = timed(lambda: qg.subspace_refresh_many([x.Pq for x in g], [x.Ps for x in g], [x.G for x in g], m, n, r, 1,
                                                      workspace=ws, out=outs[(m, n, r)]), 1)
        per_shape[f"{m}x{n} r{r}"] = {"count": len(g), "single_call_ms": one, "batched_ms_per_matrix": many / len(g)}
    # what the fp64 matrix pipe sustains with nothing else to do: register-only loop, three 256-thread workgroups per
    # CU (the residency of k_gram and k_apply) and eight (a full CU)
    sink = torch.empty((256 * 8 * 256,), dtype=torch.float32, device=dev)
    ceilings = {"note": "register-only v_mfma_f64_16x16x4 loop, 8 independent accumulators per wave, TFLOP/s"}
    for per_cu in (3, 8):
        it = 2000
        fl = qg.diag_mfma_f64_loop(it, 256 * per_cu, sink)
        t = timed(lambda: qg.diag_mfma_f64_loop(it, 256 * per_cu, sink), 3)
        ceilings[f"mfma_f64_loop_{per_cu}_workgroups_per_cu"] = fl / t / 1e9
    del sink
    bf16_flop = sum(6.0 * m * n * r for m, n, r in shapes)     # P^T G, Y = G Z^T, and P_new^T G for the check's weights
    fp64_flop = sum(2 * (m * r * r + r ** 3 / 3 + r ** 3 / 3 + m * r * r) for m, n, r in shapes)   # two rounds
    out = {"metric": "Q-GaLore subspace refresh ms over all linear weights", "value": ms, "unit": "ms",
           "n_gpus": 1, "rounds": rounds, "higher_is_better": False, "dtype": "bf16 GEMMs + fp64 orthonormalisation",
           "data": "synthetic", "config": {"workload": WORKLOADS[args.config], "matrices": len(shapes), "passes": 1,
                                           "calls": "one qg_subspace_refresh_many per distinct shape"},
           "workspace_GB": ws.numel() / 1e9,
           "wall_ms": wall, "per_shape": per_shape, "info_nonzero": bad,
           "work": {"bf16_TFLOP": bf16_flop / 1e12, "fp64_TFLOP": fp64_flop / 1e12,
                    "bf16_bound_ms": bf16_flop / PEAK_BF16_TFLOPS / 1e9, "fp64_bound_ms": fp64_flop / PEAK_FP64_TFLOPS / 1e9},
           "amortized_ms_per_step_at_interval_200": ms / 200.0,
           "ceilings": ceilings,
           "context": "the paper reports about 10 minutes per SVD refresh of LLaMA-7B on one RTX A6000 (Sec. 4.3)"}
    if not args.no_cpu_baseline:
        import numpy as np

        from oracle import qgalore as Q
        from paper_2407_08296_amd import inputs as I
        m, n, r = 768, 768, 256
        Pq, Ps = Q.quant_int4(I.projection_f32(m, r))
        Gb = I.gradient_bf16(m, n, 1)
        t0 = time.perf_counter()
        Q.subspace_refresh(Pq, Ps, Gb, m, n, r, iters=1)
        t_or = time.perf_counter() - t0
        t1 = time.perf_counter()
        Q.refresh_svd(Gb, m, n, r)
        t_svd = time.perf_counter() - t1
        Pqd, Psd = torch.from_numpy(Pq).to(dev), torch.from_numpy(Ps).to(dev)
        Gd = torch.from_numpy(Gb.view(np.int16)).to(dev)
        qg.subspace_refresh(Pqd, Psd, Gd, m, n, r, 1); torch.cuda.synchronize()
        a = torch.cuda.Event(enable_timing=True); b = torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(5):
            qg.subspace_refresh(Pqd, Psd, Gd, m, n, r, 1)
        b.record(); torch.cuda.synchronize()
        out["cpu_baseline"] = {"kind": "oracle", "sample": "one 768x768 matrix, r=256 (LLaMA-130M attention shape)",
                               "oracle_pass_ms": t_or * 1e3, "oracle_svd_ms": t_svd * 1e3,
                               "gpu_ms_same_matrix": a.elapsed_time(b) / 5, "host_cpus": len(os.sched_getaffinity(0))}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=4, choices=sorted(WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip the smaller workloads (configs 0-3), the rank sweep and the update-pass figure that the "
                         "default run reports after the timed region")
    ap.add_argument("--rsweep", action="store_true",
                    help="time qg_project / qg_lowrank_adam / qg_backproject_update_sr on one 2048x5461 matrix for "
                         "r in {128, 256, 512, 1024} (the roofline crossover of the LLaMA-1B shape) and exit")
    ap.add_argument("--pad-rows", action="store_true",
                    help="store matrices whose n is not a multiple of 16 with a row pitch of n rounded up to 16 "
                         "(the descriptor's ld): aligned rows for the direct loads")
    ap.add_argument("--zero-points", action="store_true",
                    help="weights in the zero-point (asymmetric) INT8 format instead of the symmetric one")
    ap.add_argument("--refresh", action="store_true",
                    help="time the subspace refresh (qg_subspace_refresh, one pass) over every matrix of the workload "
                         "instead of the optimizer step, print its own JSON line and exit")
    ap.add_argument("--linear", action="store_true",
                    help="time the INT8 linear layer (forward, grad_input, grad_W) over the seven weights of one decoder "
                         "layer of the workload at --tokens tokens, print its own JSON line and exit")
    ap.add_argument("--tokens", type=int, default=4096, help="tokens per micro-batch for --linear (16 sequences of 256)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 1 GiB device-to-device copy three times (reference for scaling the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (the step has no cross-GPU part); use --gpus 1")

    import torch

    from paper_2407_08296_amd import inputs as I
    from paper_2407_08296_amd import qgalore as qg

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    qg.lib()                                   # fail loudly if the HIP library is not built
    device = torch.device("cuda:0")
    torch.cuda.set_device(device)

    if args.copy_calibration:
        src = torch.ones((1 << 28,), dtype=torch.float32, device=device)      # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_read": src.numel() * 4, "bytes_written": src.numel() * 4}))
        return

    if args.rsweep:
        m, n = 2048, 5461
        rows = []
        for r in (128, 256, 512, 1024):
            P = torch.from_numpy(I.projection_f32(m, r)).to(device)
            Pq, Ps = qg.quant_int4(P)
            Wq, Ws = qg.quant_int8(torch.randn((m, n), device=device) * 0.02)
            G = (torch.randn((m, n), device=device) * 1e-3).to(torch.bfloat16)
            M = torch.zeros((r, n), device=device); V = torch.zeros((r, n), device=device)
            R = torch.empty((r, n), device=device); N = torch.empty((r, n), dtype=torch.bfloat16, device=device)
            hp = qg.hparams()
            def run(f, reps=20):
                f(); torch.cuda.synchronize()
                e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(reps):
                    f()
                e1.record(); torch.cuda.synchronize()
                return e0.elapsed_time(e1) / reps
            flops, b_proj, b_adam, b_bp = algorithmic_work([(m, n, r)])
            tp = run(lambda: qg.project(Pq, Ps, G, m, n, r, R))
            ta = run(lambda: qg.lowrank_adam(R, M, V, N, 2, hp))
            tb = run(lambda: qg.backproject_update_sr(Pq, Ps, N, Wq, Ws, m, n, r, 0.25, 1e-3, 0, 2))
            # steady state: the same matrix 24 times (the 24 `down` weights of the 1B model) through the grouped
            # launches - what a training step sees; the single launches above are bound by launch and load latency
            copies = 24
            gm = []
            for _ in range(copies):
                gm.append(qg.MatrixState(m, n, r, Pq, Ps, G.clone(), Wq.clone(), Ws.clone(), torch.zeros_like(M),
                                         torch.zeros_like(V), torch.empty_like(R), torch.empty_like(N)))
            gplan = qg.StepPlan(gm)
            gp = run(lambda: qg.project_many(gplan), 10) / copies
            ga = run(lambda: qg.lowrank_adam_many(gplan, hp, 2), 10) / copies
            gb = run(lambda: qg.backproject_update_sr_many(gplan, hp, 0, 2), 10) / copies
            del gm, gplan
            # the same 24 matrices stored with a row pitch of 5472: 16-byte aligned rows, the direct-load kernels
            ld = (n + 15) // 16 * 16
            gm = []
            for _ in range(copies):
                gm.append(qg.MatrixState(m, n, r, Pq, Ps, pitched(G, ld), pitched(Wq.view(m, n), ld), Ws.clone(),
                                         torch.zeros((r, ld), device=device), torch.zeros((r, ld), device=device),
                                         torch.empty((r, ld), device=device),
                                         torch.empty((r, ld), dtype=torch.bfloat16, device=device), ld=ld))
            gplan = qg.StepPlan(gm)
            pp = run(lambda: qg.project_many(gplan), 10) / copies
            pa = run(lambda: qg.lowrank_adam_many(gplan, hp, 2), 10) / copies
            pb = run(lambda: qg.backproject_update_sr_many(gplan, hp, 0, 2), 10) / copies
            pf = run(lambda: qg.project_adam_many(gplan, hp, 2, False), 10) / copies
            del gm, gplan
            rows.append({"r": r, "pitched_project_us": pp * 1e3, "pitched_project_TFLOP/s": flops / pp / 1e9,
                         "pitched_adam_us": pa * 1e3, "pitched_backproject_us": pb * 1e3,
                         "pitched_backproject_TFLOP/s": flops / pb / 1e9, "pitched_project_adam_us": pf * 1e3,
                         "grouped_project_us": gp * 1e3, "grouped_project_TFLOP/s": flops / gp / 1e9,
                         "grouped_project_GB/s": b_proj / gp / 1e6, "grouped_adam_us": ga * 1e3,
                         "grouped_adam_GB/s": b_adam / ga / 1e6, "grouped_backproject_us": gb * 1e3,
                         "grouped_backproject_TFLOP/s": flops / gb / 1e9, "grouped_backproject_GB/s": b_bp / gb / 1e6,
                         "project_us": tp * 1e3, "project_TFLOP/s": flops / tp / 1e9,
                         "project_GB/s": b_proj / tp / 1e6, "adam_us": ta * 1e3, "adam_GB/s": b_adam / ta / 1e6,
                         "backproject_us": tb * 1e3, "backproject_TFLOP/s": flops / tb / 1e9,
                         "backproject_GB/s": b_bp / tb / 1e6,
                         "mfma_bound_us": flops / PEAK_BF16_TFLOPS / 1e6, "hbm_bound_project_us": b_proj / PEAK_HBM_GBS / 1e3,
                         "hbm_bound_backproject_us": b_bp / PEAK_HBM_GBS / 1e3})
        print(json.dumps({"rsweep": {"m": m, "n": n, "rows": rows}}))
        return

    if args.linear:
        print(json.dumps(linear_bench(args, device)))
        return

    shapes = [(m, n, r) for (_, _, m, n, r) in I.config_matrices(args.config)]
    mats = build_state(args.config, device, args.pad_rows, args.zero_points)

    if args.refresh:
        if args.pad_rows:
            sys.exit("bench.py: the subspace refresh takes dense gradients only (--pad-rows is for the step)")
        print(json.dumps(refresh_bench(args, shapes, mats)))
        return
    import dataclasses
    # The step needs no R buffers (the projected gradient stays in registers between the projection and Adam); the
    # unfused pair of launches, timed after the step for its own roofline figures, does.
    plan = qg.StepPlan([dataclasses.replace(s, R=None) for s in mats])
    plan_unfused = qg.StepPlan(mats)
    hp = qg.hparams()
    K, W = args.steps, args.warmup

    t = 0
    for _ in range(W):
        t += 1
        qg.step_many(plan, hp, 0, t)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(K)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(K):                 # qg_step_many = these two grouped launches; events between them
        t += 1
        ev[k][0].record()
        qg.project_adam_many(plan, hp, t, False)
        ev[k][1].record()
        qg.backproject_update_sr_many(plan, hp, 0, t)
        ev[k][2].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / K
    dur2 = [sum(ev[k][i].elapsed_time(ev[k][i + 1]) for k in range(K)) / K for i in range(2)]   # ms per launch

    # Outside the timed region.  (1) The unfused projection and Adam launches, for their own roofline fractions.
    def timed(f, reps):
        f(); torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            f()
        b.record(); torch.cuda.synchronize()
        return a.elapsed_time(b) / reps
    t += 1
    d_proj = timed(lambda: qg.project_many(plan_unfused), 3)
    d_adam = timed(lambda: qg.lowrank_adam_many(plan_unfused, hp, t), 3)
    dur = [d_proj, d_adam, dur2[1]]

    # (2) The shader clock each kernel runs at (a one-wave probe on a second stream counts shader cycles against the
    # constant 100 MHz counter for about half of the kernel), and (3) the two ceilings the fractions can be read
    # against (a register-only MFMA loop, a plain device copy).
    side = torch.cuda.Stream()
    probe_out = torch.zeros((4, 2), dtype=torch.int64, device=device)
    phases = [(d_proj, lambda: qg.project_many(plan_unfused)), (d_adam, lambda: qg.lowrank_adam_many(plan_unfused, hp, t)),
              (dur2[1], lambda: qg.backproject_update_sr_many(plan, hp, 0, t)),
              (dur2[0], lambda: qg.project_adam_many(plan, hp, t + 1, False))]
    main = torch.cuda.current_stream()
    for i, (d, launch) in enumerate(phases):
        ticks = max(int(d * 0.5 * 1e5), 1000)          # 1e5 ticks per ms
        if d * 1e5 < 4000:                               # too short to sample
            launch()
            continue
        start = torch.cuda.Event()
        start.record(main)
        launch()
        with torch.cuda.stream(side):
            side.wait_event(start)
            qg.diag_clock_probe(ticks, probe_out[i])
    torch.cuda.synchronize()
    po = probe_out.cpu().tolist()
    sclk = [(c / (w / 100.0)) if w > 0 else None for c, w in po]   # MHz
    t += 1

    sink = torch.empty((qg.DIAG_MFMA_WORKGROUPS * 512,), dtype=torch.float32, device=device)
    mfma_iters = 256
    mfma_flop = qg.DIAG_MFMA_WORKGROUPS * 8 * mfma_iters * 16 * 32768.0
    ceil_const = mfma_flop / timed(lambda: qg.diag_mfma_loop(mfma_iters, False, sink), 5) / 1e9
    ceil_random = mfma_flop / timed(lambda: qg.diag_mfma_loop(mfma_iters, True, sink), 5) / 1e9
    csrc = torch.ones((1 << 27,), dtype=torch.float32, device=device)      # 512 MiB
    cdst = torch.empty_like(csrc)
    copy_gbs = 2 * csrc.numel() * 4 / timed(lambda: cdst.copy_(csrc), 5) / 1e6
    del csrc, cdst
    ceilings = {"mfma_loop_constant_operands_TFLOP/s": ceil_const, "mfma_loop_random_operands_TFLOP/s": ceil_random,
                "device_copy_GB/s": copy_gbs,
                "note": "register-only bf16 32x32x16 MFMA loop, two waves per SIMD; plain 512 MiB device copy "
                        "(read + written bytes)"}
    # The paper's default configuration, Adam with 8-bit states, after the timed region: R and N of all matrices are
    # carved out of two flat buffers, so that one flat call (the block format ignores matrix boundaries when every
    # matrix holds a whole number of blocks) serves the whole model between the two grouped GEMM launches.
    adam8 = step8 = None
    count8 = sum(r * n for m, n, r in shapes)
    if all((r * n) % 256 == 0 for m, n, r in shapes) and not args.pad_rows:
        R8 = torch.empty((count8,), dtype=torch.float32, device=device)
        N8 = torch.empty((count8,), dtype=torch.bfloat16, device=device)
        Mq8, Ms8 = qg.state8_quant(torch.zeros((count8,), dtype=torch.float32, device=device), True)
        Vq8, Vs8 = qg.state8_quant(torch.zeros((count8,), dtype=torch.float32, device=device), False)
        views, off = [], 0
        for s_ in mats:
            cnt = s_.r * s_.n
            views.append(dataclasses.replace(s_, R=R8[off:off + cnt].view(s_.r, s_.n), N=N8[off:off + cnt].view(s_.r, s_.n)))
            off += cnt
        plan8 = qg.StepPlan(views)

        def step8_launches(tt):
            qg.project_many(plan8)
            qg.lowrank_adam8(R8, Mq8, Ms8, Vq8, Vs8, N8, tt, hp)
            qg.backproject_update_sr_many(plan8, hp, 0, tt)
        step8_launches(1)                                               # leaves non-trivial states behind
        t8 = timed(lambda: qg.lowrank_adam8(R8, Mq8, Ms8, Vq8, Vs8, N8, 2, hp), 5)
        b8 = count8 * 10 + (count8 // 256) * 16
        adam8 = {"ms": t8, "GB/s": b8 / t8 / 1e6, "frac_hbm": b8 / t8 / 1e6 / PEAK_HBM_GBS, "in_timed_region": False,
                 "bytes_per_element": 10}
        step8 = {"ms": timed(lambda: step8_launches(3), 3), "launches_per_step": 3,
                 "note": "projection, Adam with 8-bit states, back-projection + update over the whole workload"}
        del plan8, views, R8, N8, Mq8, Ms8, Vq8, Vs8
    per_step = sorted(ev[k][0].elapsed_time(ev[k][2]) for k in range(K))      # GPU time of each step, ms
    step_stats = {"gpu_ms_min": per_step[0], "gpu_ms_median": per_step[len(per_step) // 2], "gpu_ms_max": per_step[-1]}
    flops, b_proj, b_adam, b_bp = algorithmic_work(shapes)
    b_fused = b_proj + b_adam - sum(8 * r * n for m, n, r in shapes)      # no R written, no R read back
    mfma = lambda ms: {"TFLOP/s": flops / ms / 1e9, "frac_mfma": flops / ms / 1e9 / PEAK_BF16_TFLOPS}
    kernels = {
        # the two launches of the step, timed inside the timed region
        "project_adam": {"ms": dur2[0], **mfma(dur2[0]), "GB/s": b_fused / dur2[0] / 1e6, "sclk_mhz": sclk[3],
                         "in_timed_region": True},
        "backproject_update_sr": {"ms": dur2[1], **mfma(dur2[1]), "GB/s": b_bp / dur2[1] / 1e6, "sclk_mhz": sclk[2],
                                  "in_timed_region": True},
        # the unfused projection and Adam launches (same results), timed after the step
        "project": {"ms": dur[0], **mfma(dur[0]), "GB/s": b_proj / dur[0] / 1e6, "sclk_mhz": sclk[0],
                    "in_timed_region": False},
        "lowrank_adam": {"ms": dur[1], "GB/s": b_adam / dur[1] / 1e6, "frac_hbm": b_adam / dur[1] / 1e6 / PEAK_HBM_GBS,
                         "sclk_mhz": sclk[1], "in_timed_region": False},
    }
    if adam8 is not None:
        kernels["lowrank_adam8"] = adam8
    dom_name, dom_kernel, dom_bytes = (("project_adam", "k_project_adam_many", b_fused) if dur2[0] >= dur2[1] else
                                       ("backproject_update_sr", "k_backproject_many", b_bp))
    roofline = {"kernel": dom_kernel, "bound": "mfma", "achieved": kernels[dom_name]["TFLOP/s"],
                "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": kernels[dom_name]["frac_mfma"], "traffic": None}
    if kernels[dom_name]["sclk_mhz"]:
        roofline["sclk_mhz"] = kernels[dom_name]["sclk_mhz"]
        # the published peak assumes 2400 MHz
        roofline["frac_of_peak_at_measured_clock"] = roofline["frac"] * 2400.0 / roofline["sclk_mhz"]
    roofline["traffic"], stamp = measured_traffic(roofline["kernel"], args.config)
    roofline["traffic_unit"] = "bytes per launch (rocprofv3 --pmc FETCH_SIZE + WRITE_SIZE, see profiles/)"
    roofline["traffic_profiled_at"] = stamp
    roofline["kernel_sources_now"] = kernel_source_digest()
    roofline["traffic_is_current"] = bool(stamp) and stamp.split()[0] == roofline["kernel_sources_now"]
    roofline["algorithmic_bytes"] = dom_bytes
    out = {
        "metric": "qgalore_step_ms_all_linear_weights", "value": ms_per_step, "unit": "ms", "n_gpus": 1,
        "steps": K, "warmup": W, "ms_per_step": ms_per_step, "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": WORKLOADS[args.config], "matrices": len(shapes), "launches_per_step": 2,
                   "row_layout": "pitch of n rounded up to 16" if args.pad_rows else "dense",
                   "weight_format": "INT8 with zero points" if args.zero_points else "INT8 symmetric"},
        "roofline": roofline, "kernels": kernels, "ceilings": ceilings, "step_stats": step_stats,
    }
    if step8 is not None:
        out["step_with_8bit_adam_states"] = step8
    del plan, plan_unfused, mats
    torch.cuda.empty_cache()
    if args.config == 4 and not args.pad_rows and not args.zero_points and not args.no_other_configs:
        out["other_configs"] = other_configs(device)
        out["rank_sweep"], out["update_pass"] = rank_sweep(device)
        out["update_pass_hbm_frac"] = out["update_pass"]["frac_hbm"]
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.config, shapes)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
