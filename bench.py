#!/usr/bin/env python3
"""Benchmark of the TSVD forward path y = U (diag(S) (V x)) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workloads a,b,...]

A step is one pass of the whole hot path (all kernels of tsvd_forward) over one batch of the
seeded synthetic workload; inputs are resident in HBM before the timed region.  The headline
line is for the largest configuration of the benchmark spec that fits one GPU, the OPT-66B fc1 prefill
shape (opt66b_fc1_prefill); the other workloads are reported in "per_config" of the same JSON line.
The roofline of a batched workload prices the algorithmic flops of its dominant kernel (stage U:
2 M K B) against the dense MFMA peak of the operand types that kernel multiplies (fp4 x fp6:
10.1 PFLOP/s; bf16 / fp16: 2.5 PFLOP/s, given beside it); B = 1 prices algorithmic bytes
K (M+N)/4 + 4K + N sizeof(x) + 4M against 8 TB/s.  "traffic" is read from the tracked counter summary
profiles/hbm_traffic_fetch_write_size.md and only reported when that summary was taken on the kernel
the library selects now (else null).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import workloads  # noqa: E402

PEAK_HBM_GBS = 8000.0
PEAK_MFMA_TFLOPS = 2500.0
PEAK_MFMA_FP6_TFLOPS = 10100.0      # dense fp6 / fp4 MFMA
PRIMARY = "opt66b_fc1_prefill"
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "hbm_traffic_fetch_write_size.md")


def _traffic_from_profile(workload, kernel_key):
    """HBM bytes per launch of the dominant kernel (scaled FETCH_SIZE + WRITE_SIZE) from the tracked counter
    summary, or None when the summary has no record for this workload or was taken on another kernel / tile
    shape than the library selects now (kernel_key).  The record is the fenced block "json bench-traffic"."""
    try:
        text = open(TRAFFIC_PROFILE).read()
        start = text.index("```json bench-traffic") + len("```json bench-traffic")
        table = json.loads(text[start:text.index("```", start)])
    except (OSError, ValueError):
        return None
    rec = table.get(workload)
    if not rec or rec.get("kernel") != kernel_key:
        return None
    return float(rec["fetch_bytes"]) + float(rec["write_bytes"])


def _device_x(inputs, dev):
    import torch
    if inputs.x_dtype == "bf16":
        return torch.from_numpy(inputs.X_bits.view(np.int16)).to(dev).view(torch.bfloat16)
    return torch.from_numpy(inputs.X).to(dev)


def _timed(fn, steps, warmup):
    """Runs fn() warmup + steps times; returns (wall ms per step, event ms per step)."""
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    return (t1 - t0) * 1e3 / steps, e0.elapsed_time(e1) / steps


def _stage_u_kernel_name(tsvd, handle, B):
    """Name of the batched stage-U kernel the library picks (its tile-shape rule, asked through the
    diagnostic interface include/tsvd_tuning.h)."""
    try:
        _, su = tsvd.tsvd_tuning_tile_shapes(handle, B)
    except ValueError:
        return "batched stage-U kernel", -1
    if su < 0:
        return "batched stage-U kernel", su
    if su == 32:
        return "tsvd_panel_kernel", su
    if su == 33:
        return "tsvd_panel_fp6_kernel", su
    if su == 40:
        return "tsvd_gemm_fp6_kernel", su
    return ("tsvd_gemm_ring_kernel" if su >= 14 else "tsvd_gemm_pipe_kernel"), su


def cpu_baseline(w, inputs, budget_s):
    """The oracle as it stands, timed on this host: tokens/s over about budget_s seconds of work.

    Returns (record, columns, reference): the oracle's output for `columns` doubles as the
    parity reference of the GPU result."""
    import oracle
    per_token = float(w.K) * (w.M + w.N)                       # multiply-adds per token
    rate_guess = 1.5e9 * oracle.threads()                      # multiply-adds per second, rough
    ncols = int(min(w.B, max(1, budget_s * rate_guess / per_token)))
    cols = np.unique(np.linspace(0, w.B - 1, ncols).astype(np.int64))
    X = np.ascontiguousarray(inputs.X[:, cols])
    reps, t0, ref = 0, time.perf_counter(), None
    while True:
        ref = oracle.forward(inputs.U, inputs.S, inputs.V, X)
        reps += 1
        dt = time.perf_counter() - t0
        if dt >= budget_s or reps >= 200:
            break
    rec = {"value": reps * len(cols) / dt, "unit": "tokens/s", "cores": oracle.threads(), "kind": "oracle",
           "sample": f"{reps} pass(es) over {len(cols)} of {w.B} tokens (evenly spaced columns), all {w.M} rows, {dt:.1f} s"}
    return rec, cols, ref


def bench_workload(name, steps, warmup, with_cpu=True, cpu_budget_s=4.0):
    import torch
    import paper_2308_07641_amd as tsvd

    w = workloads.WORKLOADS[name]
    dev = torch.device("cuda:0")
    t_gen = time.perf_counter()
    inputs = workloads.make_workload(name)
    print(f"[bench] {name}: inputs drawn in {time.perf_counter() - t_gen:.1f} s", file=sys.stderr, flush=True)
    batched = w.B >= 64
    x = _device_x(inputs, dev)
    y = torch.empty((w.M, w.B), dtype=torch.float32, device=dev)

    # B = 1 streams the weights once per token: rotate over enough copies of the packed
    # weights that the 256 MB memory-side cache cannot serve them (the HBM figure), and also
    # report the cache-warm time on a single copy.
    blob_bytes = tsvd.tsvd_packed_bytes(w.M, w.K, w.N)
    ncopies = 1 if batched else max(2, int(np.ceil(640e6 / blob_bytes)))
    ncopies = min(ncopies, 64)
    handles = [tsvd.tsvd_pack(inputs.U, inputs.S, inputs.V) for _ in range(ncopies)]
    ws = torch.empty(tsvd.tsvd_workspace_bytes(handles[0], w.B, tsvd.TSVD_BF16 if w.x_dtype == "bf16" else tsvd.TSVD_F32),
                     dtype=torch.uint8, device=dev)
    info = tsvd.tsvd_info(handles[0])
    print(f"[bench] {name}: packed {blob_bytes / 1e6:.1f} MB x {ncopies}", file=sys.stderr, flush=True)

    state = {"i": 0, "mask": 7}

    def step_rot():
        h = handles[state["i"] % ncopies]
        state["i"] += 1
        if state["mask"] == 7:
            tsvd.tsvd_forward(h, x, y, workspace=ws)
        else:       # one stage alone, on the z an earlier full call left in the workspace (diagnostic entry point)
            tsvd.tsvd_tuning_forward_stages(h, x, y, state["mask"], workspace=ws)

    def step_one():
        tsvd.tsvd_forward(handles[0], x, y, workspace=ws)

    wall_ms, ev_ms = _timed(step_rot, steps, warmup)
    res = {"workload": name, "M": w.M, "N": w.N, "K": w.K, "B": w.B, "x_dtype": w.x_dtype,
           "ms_per_step": wall_ms, "event_ms_per_step": ev_ms, "tokens_per_s": w.B / (wall_ms * 1e-3),
           "weight_copies_rotated": ncopies,
           "paper_counts_per_token": {"mults": w.K, "adds": info["nnzU"] + info["nnzV"]}}
    flops_exec = 2.0 * w.K * (w.M + w.N) * w.B
    flops_dense = 2.0 * w.M * w.N * w.B
    res["executed_tflops"] = flops_exec / (ev_ms * 1e-3) / 1e12
    res["dense_equiv_tflops"] = flops_dense / (ev_ms * 1e-3) / 1e12

    # dominant kernel: stage U (M/(M+N) of the work), timed alone on the z left in the workspace
    # by the full passes above (tsvd_tuning_forward_stages)
    state["mask"] = 4
    _, u_ms = _timed(step_rot, steps, max(2, warmup // 2))
    state["mask"] = 2
    _, v_ms = _timed(step_rot, steps, max(2, warmup // 2))
    state["mask"] = 7
    step_rot()                      # a full pass again: y is compared with the oracle below
    torch.cuda.synchronize()
    res["stage_ms"] = {"V": v_ms, "U": u_ms}
    if batched:
        # the layer form beside it (bf16 y instead of fp32, same arithmetic until the last rounding): half the output bytes
        yb = torch.empty((w.M, w.B), dtype=torch.bfloat16, device=dev)
        _, lb_ms = _timed(lambda: tsvd.tsvd_forward_ex(handles[0], x, y=yb, y_dtype=tsvd.TSVD_BF16, workspace=ws), steps, max(2, warmup // 2))
        res["bf16_output"] = {"event_ms_per_step": lb_ms, "executed_tflops": flops_exec / (lb_ms * 1e-3) / 1e12,
                              "frac_of_bf16_peak": flops_exec / (lb_ms * 1e-3) / 1e12 / PEAK_MFMA_TFLOPS}
        del yb
    kernel_name, shape_u = _stage_u_kernel_name(tsvd, handles[0], w.B) if batched else (None, -1)
    kernel_key = f"{kernel_name}:{shape_u}" if batched else ("tsvd_mid_kernel" if w.B > 1 else "tsvd_gemv_kernel")
    traffic = _traffic_from_profile(name, kernel_key)
    res["dominant_kernel_key"] = kernel_key
    if batched and kernel_name == "tsvd_panel_kernel":
        # one launch does both stages (z stays in LDS): the call IS the dominant kernel; the stage
        # times above belong to the two-launch path that the stage mask falls back to
        res["two_launch_stage_ms"] = res.pop("stage_ms")
        res["roofline"] = {"bound": "mfma", "kernel": "tsvd_panel_kernel (both stages, bf16 + fp16 MFMA)",
                           "achieved": res["executed_tflops"], "peak": PEAK_MFMA_TFLOPS, "unit": "TFLOP/s",
                           "frac": res["executed_tflops"] / PEAK_MFMA_TFLOPS,
                           "traffic": traffic,
                           "whole_path_frac": res["executed_tflops"] / PEAK_MFMA_TFLOPS}
    elif batched and kernel_name == "tsvd_panel_fp6_kernel":
        # one launch does both stages on fp4 codes x three fp6 planes (x and z as planes in LDS): the call IS the
        # dominant kernel.  Achieved = ALGORITHMIC flops 2 K (M + N) B per second against the 10.1 PFLOP/s fp4 / fp6
        # peak; three times as many are executed; the fraction of the 2.5 PFLOP/s bf16 / fp16 peak is given beside it
        # because that is what the benchmark spec prices the batched path against.
        res["two_launch_stage_ms"] = res.pop("stage_ms")
        ach = res["executed_tflops"]
        res["roofline"] = {"bound": "mfma", "kernel": "tsvd_panel_fp6_kernel (both stages, fp4 x fp6 MFMA, 3 planes)",
                           "achieved": ach, "peak": PEAK_MFMA_FP6_TFLOPS, "unit": "TFLOP/s", "frac": ach / PEAK_MFMA_FP6_TFLOPS,
                           "executed_tflops": 3.0 * ach, "executed_frac": 3.0 * ach / PEAK_MFMA_FP6_TFLOPS,
                           "frac_of_bf16_peak": ach / PEAK_MFMA_TFLOPS,
                           "traffic": traffic,
                           "whole_path_frac_of_bf16_peak": ach / PEAK_MFMA_TFLOPS}
    elif batched and kernel_name == "tsvd_gemm_fp6_kernel":
        # stage U = fp4 x fp6 kernel (+ the planes pass where stage V leaves fp16 z).  Achieved = ALGORITHMIC flops (2 M K B) per second; the
        # kernel executes three times as many (three planes) on the fp4 / fp6 MFMA path, whose dense
        # peak is 10.1 PFLOP/s; the fraction of the 2.5 PFLOP/s fp16 peak is given beside it because that
        # is what every other batched kernel here is priced against.
        fl_u = 2.0 * w.K * w.M * w.B
        ach = fl_u / (u_ms * 1e-3) / 1e12
        res["roofline"] = {"bound": "mfma", "kernel": "tsvd_gemm_fp6_kernel (stage U, fp4 x fp6 MFMA, 3 planes; where stage V does not write the planes of z "
                                                     "itself, timed together with the operand pass tsvd_z_planes_kernel, about 2 % of it)",
                           "achieved": ach, "peak": PEAK_MFMA_FP6_TFLOPS, "unit": "TFLOP/s", "frac": ach / PEAK_MFMA_FP6_TFLOPS,
                           "algorithmic_flops": fl_u, "launch_ms": u_ms,
                           "executed_tflops": 3.0 * ach, "executed_frac": 3.0 * ach / PEAK_MFMA_FP6_TFLOPS,
                           "frac_of_bf16_peak": ach / PEAK_MFMA_TFLOPS,
                           "traffic": traffic,
                           "whole_path_frac_of_bf16_peak": res["executed_tflops"] / PEAK_MFMA_TFLOPS}
    elif batched:
        fl_u = 2.0 * w.K * w.M * w.B
        res["roofline"] = {"bound": "mfma", "kernel": kernel_name + " (stage U, fp16 MFMA)",
                           "achieved": fl_u / (u_ms * 1e-3) / 1e12, "peak": PEAK_MFMA_TFLOPS, "unit": "TFLOP/s",
                           "frac": fl_u / (u_ms * 1e-3) / 1e12 / PEAK_MFMA_TFLOPS,
                           "traffic": traffic,
                           "whole_path_frac": res["executed_tflops"] / PEAK_MFMA_TFLOPS}
    else:
        xb = 2 if w.x_dtype == "bf16" else 4
        kp = -(-w.K // 256) * 256
        bytes_alg = w.K * (w.M + w.N) / 4.0 + 4.0 * w.K + w.N * xb * w.B + 4.0 * w.M * w.B
        few = w.B > 1                                             # few-token kernel: z is fp16 [Kp][16]
        # codes of U + z (B = 1: 8 digit planes of Kp bytes; few tokens: fp16 [Kp][16]) + y
        bytes_u = w.K * w.M / 4.0 + (32.0 * kp if few else 8.0 * kp) + 4.0 * w.M * w.B
        _, warm_ev = _timed(step_one, steps, warmup)
        res["cache_warm_event_ms"] = warm_ev
        gbs = bytes_u / (u_ms * 1e-3) / 1e9
        res["roofline"] = {"bound": "hbm", "kernel": "tsvd_mid_kernel (stage U)" if few else "tsvd_gemv_kernel (stage U)",
                           "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS,
                           "traffic": traffic, "algorithmic_bytes": bytes_u,
                           "whole_path_gbs": bytes_alg / (ev_ms * 1e-3) / 1e9,
                           "whole_path_frac": bytes_alg / (ev_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                           "whole_path_bytes": bytes_alg,
                           "cache_warm_whole_path_gbs": bytes_alg / (warm_ev * 1e-3) / 1e9}

    if with_cpu:
        res["cpu_baseline"], cols, ref = cpu_baseline(w, inputs, cpu_budget_s)
        got = y[:, torch.from_numpy(cols).to(dev)].cpu().numpy().astype(np.float64)
        res["parity_rel_err"] = float(np.max(np.abs(got - ref)) / np.max(np.abs(ref)))
    for h in handles:
        tsvd.tsvd_free(h)
    return res


def bench_dense_codes(steps=200, warmup=20):
    """NEXT row of the scope table (the paper's remark that 2 bits per ternary element are redundant): stage U of
    the single-token decode workload on the five-elements-per-byte code of U (1.6 bits per element) against the
    2-bit tiles, weights rotating through HBM.  The dense code is a diagnostic switch, never a default."""
    import torch
    import paper_2308_07641_amd as tsvd
    name = "opt6b7_fc1_decode"
    w = workloads.WORKLOADS[name]
    inputs = workloads.make_workload(name)
    dev = torch.device("cuda:0")
    x = _device_x(inputs, dev)
    y = torch.empty((w.M, 1), dtype=torch.float32, device=dev)
    out = {"workload": f"{name}: stage U on 2-bit tiles vs five elements per byte", "bytes_of_U": {"two_bit": w.M * w.K / 4.0,
           "dense": float(tsvd.tsvd_dense_bytes(w.M, w.K))}}
    import oracle
    ref = oracle.forward(inputs.U, inputs.S, inputs.V, inputs.X)
    for label, flag in (("two_bit", 0), ("dense", 1)):
        tsvd.tsvd_tuning_set("TSVD_DENSE_U", flag)
        handles = [tsvd.tsvd_pack(inputs.U, inputs.S, inputs.V) for _ in range(16)]
        tsvd.tsvd_tuning_reset()
        ws = torch.empty(tsvd.tsvd_workspace_bytes(handles[0], 1, tsvd.TSVD_BF16), dtype=torch.uint8, device=dev)
        state = {"i": 0}

        def full():
            state["i"] += 1
            tsvd.tsvd_forward(handles[state["i"] % 16], x, y, workspace=ws)

        def stage_u():
            state["i"] += 1
            tsvd.tsvd_tuning_forward_stages(handles[state["i"] % 16], x, y, 4, workspace=ws)

        _, call_ms = _timed(full, steps, warmup)
        _, u_ms = _timed(stage_u, steps, warmup)
        full()
        torch.cuda.synchronize()
        err = float(np.max(np.abs(y.cpu().numpy().astype(np.float64) - ref)) / np.max(np.abs(ref)))
        out[label] = {"call_us": call_ms * 1e3, "stage_u_us": u_ms * 1e3, "parity_rel_err": err}
        for h in handles:
            tsvd.tsvd_free(h)
    return out


def bench_transition(max_rank_gpu=64, max_rank_cpu=24):
    """NEXT row of the scope table: the direct transition W -> (U, S, V) (Algorithm 2) on the
    paper's random-matrix setting, a [512, 256] Laplace matrix at theta = 0.576.  A bounded number
    of iterations is timed on the GPU and, beside it, in the numpy oracle (whose cost per
    iteration grows with the rank: a full SVD of the residual plus a pseudo-inverse of order K)."""
    import torch
    import paper_2308_07641_amd as tsvd
    from oracle import transition as tr
    W = np.random.default_rng(4).laplace(size=(512, 256))
    Wd = torch.from_numpy(W).to("cuda:0")
    tsvd.tsvd_transition(Wd, 0.576, 0.0, 4)                       # warm-up (allocations, code load)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    U, S, V, errs, status = tsvd.tsvd_transition(Wd, 0.576, 0.0, max_rank_gpu)
    torch.cuda.synchronize()
    gpu_s = time.perf_counter() - t0
    t0 = time.perf_counter()
    Uo, So, Vo, eo = tr.transition(W, 0.576, max_rank=max_rank_cpu)
    cpu_s = time.perf_counter() - t0
    k = min(max_rank_gpu, max_rank_cpu)
    same = all(np.array_equal(U[:, j].cpu().numpy(), Uo[:, j]) or np.array_equal(-U[:, j].cpu().numpy(), Uo[:, j]) for j in range(k))
    return {"workload": "transition_laplace_512x256: W fp64 [512,256] Laplace, theta=0.576, q=1",
            "gpu_ms_per_iteration": gpu_s / max_rank_gpu * 1e3, "gpu_iterations": max_rank_gpu,
            "relative_error_after": errs[-1], "status": status,
            "nonzero_rate": float((torch.count_nonzero(U) + torch.count_nonzero(V)).item() / (U.numel() + V.numel())),
            "cpu_baseline": {"value": cpu_s / max_rank_cpu * 1e3, "unit": "ms/iteration", "kind": "oracle",
                             "sample": f"first {max_rank_cpu} iterations (numpy SVD + pseudo-inverse)"},
            "first_components_equal_oracle": bool(same), "oracle_error_after": eo[k - 1], "gpu_error_at_same_rank": errs[k - 1]}


def bench_conv(steps=50):
    """NEXT row of the scope table: a convolution in ternary-SVD form (section "TSVD in Convolution
    Layer"), a 3 x 3, 256 -> 256 channel layer on 32 images of 14 x 14 (a ResNet-50 stage-4 shape), in
    form 0 (V is the 3 x 3 convolution: gather, then the linear map) and form 1 (U is: map, then
    tap sum), rank 768, P(0) = 0.7; the oracle (dense kernel, fp64) is timed on one image."""
    import torch
    import paper_2308_07641_amd as tsvd
    from oracle import conv as oc
    co = ci = 256
    k, K, images, H = 3, 768, 32, 14
    rng = np.random.default_rng(23080764 + 7000)
    out = {"workload": f"conv3x3 {ci}->{co}, {images} images {H}x{H}, pad 1, rank {K}, bf16 x, fp32 y"}
    for form in (0, 1):
        rows, cols = (co, ci * k * k) if form == 0 else (co * k * k, ci)
        U = rng.choice([-1, 0, 1], size=(rows, K), p=[0.15, 0.7, 0.15]).astype(np.int8)
        V = rng.choice([-1, 0, 1], size=(K, cols), p=[0.15, 0.7, 0.15]).astype(np.int8)
        S = (np.abs(rng.standard_normal(K)) * 0.02).astype(np.float32)
        xb = workloads.f32_to_bf16_bits(rng.standard_normal((ci, images, H, H)).astype(np.float32))
        x = torch.from_numpy(xb.view(np.int16)).to("cuda:0").view(torch.bfloat16)
        h = tsvd.tsvd_pack(U, S, V)
        fn = lambda: tsvd.tsvd_conv2d_forward(h, form, ci, co, k, k, x, (1, 1), (1, 1), (1, 1))
        _, ev_ms = _timed(fn, steps, 5)
        y = fn()
        torch.cuda.synchronize()
        xr = workloads.bf16_bits_to_f32(xb[:, :1]).transpose(1, 0, 2, 3)
        t0 = time.perf_counter()
        ref = oc.tsvd_conv2d(xr, U, S, V, form, co, ci, k, k, (1, 1), (1, 1), (1, 1))
        cpu_s = time.perf_counter() - t0
        err = float(np.max(np.abs(y[:, 0].float().cpu().numpy() - ref[0])) / np.max(np.abs(ref)))
        flops = 2.0 * K * (rows + cols) * images * H * H
        out[f"form{form}"] = {"ms_per_call": ev_ms, "images_per_s": images / (ev_ms * 1e-3), "executed_tflops": flops / (ev_ms * 1e-3) / 1e12,
                              "parity_rel_err": err,
                              "cpu_baseline": {"value": 1.0 / cpu_s, "unit": "images/s", "kind": "oracle", "sample": "1 image"}}
        tsvd.tsvd_free(h)
    # depth-wise 7 x 7 with rank 5 per channel (how the paper's converted ConvNeXt lists its dwconv
    # layers; first-stage shape: 96 channels, 56 x 56), 32 images, non-zero rate 0.235
    C, k, kg, H = 96, 7, 5, 56
    U = np.zeros((C, C * kg), dtype=np.int8)
    for c in range(C):
        U[c, c * kg:(c + 1) * kg] = rng.choice([-1, 1], size=kg)
    V = rng.choice([-1, 0, 1], size=(C * kg, k * k), p=[0.1175, 0.765, 0.1175]).astype(np.int8)
    S = (np.abs(rng.standard_normal(C * kg)) * 0.05).astype(np.float32)
    xb = workloads.f32_to_bf16_bits(rng.standard_normal((C, images, H, H)).astype(np.float32))
    x = torch.from_numpy(xb.view(np.int16)).to("cuda:0").view(torch.bfloat16)
    h = tsvd.tsvd_pack(U, S, V)
    fn = lambda: tsvd.tsvd_conv2d_forward(h, 0, C, C, k, k, x, (1, 1), (3, 3), (1, 1), groups=C)
    _, ev_ms = _timed(fn, steps, 5)
    y = fn()
    torch.cuda.synchronize()
    xr = workloads.bf16_bits_to_f32(xb[:, :1]).transpose(1, 0, 2, 3)
    t0 = time.perf_counter()
    ref = oc.tsvd_conv2d(xr, U, S, V, 0, C, C, k, k, (1, 1), (3, 3), (1, 1), None, C)
    cpu_s = time.perf_counter() - t0
    err = float(np.max(np.abs(y[:, 0].float().cpu().numpy() - ref[0])) / np.max(np.abs(ref)))
    moved = C * images * H * H * (2 + 4)            # x bf16 read once, y fp32 written once
    adds = (np.count_nonzero(V) + np.count_nonzero(U)) * images * H * H
    out["depthwise7x7"] = {"workload": f"depth-wise 7x7, {C} channels, rank {kg} per channel, {images} images {H}x{H}, pad 3",
                           "ms_per_call": ev_ms, "images_per_s": images / (ev_ms * 1e-3),
                           "hbm_gbs": moved / (ev_ms * 1e-3) / 1e9, "hbm_frac": moved / (ev_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                           "additions_per_s": adds / (ev_ms * 1e-3), "parity_rel_err": err,
                           "cpu_baseline": {"value": 1.0 / cpu_s, "unit": "images/s", "kind": "oracle", "sample": "1 image"}}
    tsvd.tsvd_free(h)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workloads",
                    default="opt66b_fc1_prefill,tiny,bert_ffn_in,convnext_mlp,opt6b7_fc1_decode,opt6b7_fc1_decode_b16,opt6b7_fc1_prefill_b256,ffn_768x3072_rank1545")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing / parity leg")
    ap.add_argument("--no-transition", action="store_true", help="skip the transition (Algorithm 2) measurement")
    ap.add_argument("--dense-codes-only", action="store_true", help="run only the dense-code measurement (for profiling)")
    ap.add_argument("--conv-only", action="store_true", help="run only the convolution-form measurement (for profiling)")
    ap.add_argument("--transition-only", action="store_true",
                    help="run only the transition measurement and print its record (for profiling)")
    ap.add_argument("--tune", action="append", default=[], metavar="NAME=VALUE",
                    help="set a diagnostic switch of include/tsvd_tuning.h for this run (A/B measurements; repeatable)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 256 MiB device copy (reference for FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; --gpus above 1 is not supported "
              "(the path would shard over tokens or over rank slices with one all-reduce of y)", file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    import paper_2308_07641_amd as tsvd
    tsvd.load_library()
    for item in args.tune:
        k, v = item.split("=", 1)
        tsvd.tsvd_tuning_set(k, int(v))

    if args.transition_only:
        print(json.dumps(bench_transition()), flush=True)
        return
    if args.conv_only:
        print(json.dumps(bench_conv()), flush=True)
        return
    if args.dense_codes_only:
        print(json.dumps(bench_dense_codes()), flush=True)
        return

    if args.copy_calibration:
        src = torch.ones(256 << 20, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    names = [n for n in args.workloads.split(",") if n]
    if PRIMARY not in names:
        names.insert(0, PRIMARY)
    per = {}
    for n in names:
        steps = args.steps if workloads.WORKLOADS[n].B * workloads.WORKLOADS[n].K < 1 << 24 else max(5, args.steps // 10)
        per[n] = bench_workload(n, steps, args.warmup, with_cpu=not args.no_cpu,
                                cpu_budget_s=12.0 if n == PRIMARY else 3.0)
        per[n]["steps"] = steps
        print(f"[bench] {n}: {json.dumps(per[n])}", file=sys.stderr, flush=True)

    if not args.no_transition and not args.no_cpu:
        per["transition_laplace_512x256"] = bench_transition()
        print(f"[bench] transition: {json.dumps(per['transition_laplace_512x256'])}", file=sys.stderr, flush=True)
        per["conv3x3_c256"] = bench_conv()
        print(f"[bench] conv: {json.dumps(per['conv3x3_c256'])}", file=sys.stderr, flush=True)
        per["dense_codes_decode"] = bench_dense_codes()
        print(f"[bench] dense codes: {json.dumps(per['dense_codes_decode'])}", file=sys.stderr, flush=True)

    p = per[PRIMARY]
    w = workloads.WORKLOADS[PRIMARY]
    line = {
        "metric": "TSVD linear fwd: tokens/s + HBM GB/s (B=1) / MFMA util (batched) vs roofline",
        "value": p["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": p["steps"], "warmup": args.warmup,
        "ms_per_step": p["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "fp4 codes x fp6 (E2M3) planes of bf16 x and of fp32 z, fp32 accumulation",
        "data": "synthetic",
        "config": {"workload": f"{PRIMARY}: M={w.M} N={w.N} K={w.K} B={w.B}, ternary U,V P(0)={w.p0}, bf16 X",
                   "executed_tflops": p["executed_tflops"], "dense_equiv_tflops": p["dense_equiv_tflops"]},
        "roofline": {k: p["roofline"][k] for k in ("bound", "achieved", "peak", "unit", "frac", "traffic", "kernel",
                                                    "frac_of_bf16_peak", "whole_path_frac_of_bf16_peak") if k in p["roofline"]},
        "cpu_baseline": p.get("cpu_baseline"),
        "per_config": per,
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
