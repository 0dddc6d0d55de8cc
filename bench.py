#!/usr/bin/env python3
"""Benchmark of the QwT-v2 hot path on one MI355X.

One "step" is one pass of the whole path over one synthetic batch, for every
linear layer of the workload:
    calibration forward (int8 GEMM -> fp32 Y_quant)      qlinear_cwac_forward, fp32 out
    per-channel statistics of (Y_full, Y_quant)          cwac_calibrate_stats_first (a run's first batch: no reset)
    closed-form fit                                      cwac_solve
    fold into the engine parameters                      cwac_fold
    inference forward (int8 GEMM + CWAC epilogue -> int8) qlinear_cwac_forward, int8 out
All inputs are resident in HBM before the timed region.  Prints ONE JSON line.
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

METRIC = "W8A8 GEMM+CWAC epilogue TOPS (% int8 MFMA peak); calib stats GB/s (% HBM)"
INT8_MFMA_PEAK_TOPS = 5000.0   # MI355X dense int8, published
FP16_MFMA_PEAK_TFLOPS = 2500.0  # MI355X dense fp16, published
HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
# HBM-side bytes per launch.  NOT measured by this run: constants copied from the committed rocprofv3
# --pmc FETCH_SIZE / WRITE_SIZE summaries of `bench.py --probe` (the file named in "traffic_source"),
# scaled by what the same counters read for a plain 1 GiB copy (x1.997, x1.000); mean over the
# workload's launches.
PMC_TRAFFIC_BYTES = {5: {"forward_int8": 982e6 + 139e6, "statistics": 1113e6 + 8e6,
                         "forward_w4a16": 1044e6 + 292e6}}
PMC_TRAFFIC_SOURCE = {5: "profiles/bench_config5_pmc_traffic.md (constant from that profile, not measured in this run)"}


class LayerState:
    pass


def setup_layers(P, synth, torch, cfg: int, dev: str, cal_rows: int):
    """Synthetic fp32 tensors of the workload -> device-resident quantized inputs.
    Quantization and parameter preparation run in the library's own kernels; the
    full-precision layer output Y_full is upstream of the path (torch fp32 matmul)."""
    wl = synth.WORKLOADS[cfg]
    layers = []
    for li, ly in enumerate(wl.layers):
        L = LayerState()
        L.name, L.n, L.k, L.m, L.cal_rows = ly.name, ly.n, ly.k, wl.m, cal_rows
        w, b = synth.weights(wl, li, device=dev)
        x = synth.activations(wl, li, wl.m, device=dev)
        xcal = synth.activations(wl, li, cal_rows, calibration=True, device=dev)
        L.bias = b
        L.wq = torch.empty(ly.n, ly.k, dtype=torch.int8, device=dev)
        L.sw = torch.empty(ly.n, dtype=torch.float32, device=dev)
        P.cwac_quantize_rows_sym(w, L.sw, L.wq)
        L.colsum = torch.empty(ly.n, dtype=torch.int32, device=dev)
        P.cwac_colsum(L.wq, L.colsum)
        L.xq = torch.empty(wl.m, ly.k, dtype=torch.int8, device=dev)
        L.xq_cal = torch.empty(cal_rows, ly.k, dtype=torch.int8, device=dev)
        if wl.per_token:
            L.sx_row = torch.empty(wl.m, dtype=torch.float32, device=dev)
            L.sx_row_cal = torch.empty(cal_rows, dtype=torch.float32, device=dev)
            P.cwac_quantize_rows_sym(x, L.sx_row, L.xq)
            P.cwac_quantize_rows_sym(xcal, L.sx_row_cal, L.xq_cal)
            L.sx, L.zx = 1.0, 0
        else:
            mm = torch.empty(2, dtype=torch.float32, device=dev)
            ws = torch.empty(P.cwac_range_workspace(xcal.numel()), dtype=torch.uint8, device=dev)
            P.cwac_range_f32(xcal, mm, ws)
            mn, mx = (float(v) for v in mm.cpu())
            L.sx, z_u = P.cwac_qparams_from_range(mn, mx, 8)
            L.zx = z_u - 128
            P.cwac_quantize_act(x, L.sx, L.zx, L.xq)
            P.cwac_quantize_act(xcal, L.sx, L.zx, L.xq_cal)
            L.sx_row = L.sx_row_cal = None
        L.y_full = xcal @ w.t()
        if b is not None:
            L.y_full += b
        # output quantization parameters: Eq. 2 on the full-precision output range (stand-in for
        # the compensated output's range, which it approximates by construction of the fit)
        mm = torch.empty(2, dtype=torch.float32, device=dev)
        ws = torch.empty(P.cwac_range_workspace(L.y_full.numel()), dtype=torch.uint8, device=dev)
        P.cwac_range_f32(L.y_full, mm, ws)
        mn, mx = (float(v) for v in mm.cpu())
        L.sr, zr_u = P.cwac_qparams_from_range(mn, mx, 8)
        L.zr = zr_u - 128
        L.per_token = wl.per_token
        mode = P.CWAC_EPI_FP_BIAS if wl.per_token else P.CWAC_EPI_INT_OFFSET
        L.qp = P.make_qparams(mode, wl.per_token, L.sx, L.zx, L.sr, L.zr)
        L.qp_deq = P.make_qparams(P.CWAC_EPI_FP_BIAS, wl.per_token, L.sx, L.zx, 1.0, 0)
        f32 = dict(dtype=torch.float32, device=dev)
        L.deq_mult, L.deq_fb = torch.empty(ly.n, **f32), torch.empty(ly.n, **f32)
        L.deq_off = torch.empty(ly.n, dtype=torch.int32, device=dev)
        P.cwac_fold(None, None, L.sw, L.bias, L.colsum, L.qp_deq, L.deq_mult, L.deq_off, L.deq_fb)
        L.mult, L.fbias = torch.empty(ly.n, **f32), torch.empty(ly.n, **f32)
        L.offset = torch.empty(ly.n, dtype=torch.int32, device=dev)
        L.alpha, L.beta = torch.empty(ly.n, **f32), torch.empty(ly.n, **f32)
        L.stats = torch.empty(P.cwac_stats_bytes(ly.n) // 8 + 2, dtype=torch.float64, device=dev)
        L.ws = torch.empty(P.cwac_calibrate_stats_workspace(cal_rows, ly.n), dtype=torch.uint8,
                           device=dev)
        del w, x, xcal
        layers.append(L)
    n_max = max(L.n for L in layers)
    yq_buf = torch.empty(cal_rows * n_max, dtype=torch.float32, device=dev)
    out_buf = torch.empty(wl.m * n_max, dtype=torch.int8, device=dev)
    for L in layers:
        L.yq = yq_buf[:cal_rows * L.n].view(cal_rows, L.n)
        L.out = out_buf[:wl.m * L.n].view(wl.m, L.n)
    torch.cuda.synchronize()
    return wl, layers


def run_step(P, layers, ev=None):
    """One pass of the hot path.  ev (optional): list that receives per-layer event tuples."""
    import torch
    for L in layers:
        if ev is not None:
            e = [torch.cuda.Event(enable_timing=True) for _ in range(5)]
            e[0].record()
        P.qlinear_cwac_forward(L.xq_cal, L.wq, None, L.deq_mult, L.deq_off,
                               L.deq_fb if L.bias is not None else None, L.sx_row_cal,
                               P.CWAC_OUT_FP32, L.yq)
        if ev is not None:
            e[1].record()
        P.cwac_calibrate_stats_first(L.y_full, L.yq, L.stats, L.ws)
        if ev is not None:
            e[2].record()
        P.cwac_solve(L.stats, L.n, L.alpha, L.beta)
        P.cwac_fold(L.alpha, L.beta, L.sw, L.bias, L.colsum, L.qp, L.mult, L.offset, L.fbias)
        if ev is not None:
            e[3].record()
        if L.per_token:
            P.qlinear_cwac_forward(L.xq, L.wq, L.qp, L.mult, L.offset, L.fbias, L.sx_row,
                                   P.CWAC_OUT_INT8, L.out)
        else:
            P.qlinear_cwac_forward(L.xq, L.wq, L.qp, L.mult, L.offset, None, None,
                                   P.CWAC_OUT_INT8, L.out)
        if ev is not None:
            e[4].record()
            ev.append(e)


def _forward_int8(P, L, mult, offset, fbias):
    if L.per_token:
        P.qlinear_cwac_forward(L.xq, L.wq, L.qp, mult, offset, fbias, L.sx_row, P.CWAC_OUT_INT8, L.out)
    else:
        P.qlinear_cwac_forward(L.xq, L.wq, L.qp, mult, offset, None, None, P.CWAC_OUT_INT8, L.out)


def comparators(P, torch, layers, reps: int = 3):
    """What the fold buys (Sec. 3.4): the fused CWAC forward against (B0) the same kernel with
    plain PTQ parameters (alpha = 1, beta = 0) and against (B1 + EPI) a raw int32 GEMM followed
    by the epilogue as a separate pass over the stored accumulators.  ms per pass over all layers."""
    dev = layers[0].xq.device
    n_max, m = max(L.n for L in layers), layers[0].m
    acc_buf = torch.empty(m * n_max, dtype=torch.int32, device=dev)
    ptq = []
    for L in layers:
        f32 = dict(dtype=torch.float32, device=dev)
        pm, pf = torch.empty(L.n, **f32), torch.empty(L.n, **f32)
        po = torch.empty(L.n, dtype=torch.int32, device=dev)
        P.cwac_fold(None, None, L.sw, L.bias, L.colsum, L.qp, pm, po, pf)
        ptq.append((pm, po, pf))

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    def fused():
        for L in layers:
            _forward_int8(P, L, L.mult, L.offset, L.fbias)

    def plain():
        for L, (pm, po, pf) in zip(layers, ptq):
            _forward_int8(P, L, pm, po, pf)

    def unfused():
        for L in layers:
            acc = acc_buf[:L.m * L.n].view(L.m, L.n)
            P.qlinear_cwac_forward(L.xq, L.wq, None, None, None, None, None, P.CWAC_OUT_INT32, acc)
            P.cwac_epilogue_int32(acc, L.qp, L.mult, L.offset, L.fbias if L.per_token else None,
                                  L.sx_row, P.CWAC_OUT_INT8, L.out)

    # integer-only engine form (fixed-point multiplier) on the same shapes; a per-tensor activation
    # scale is assumed for it, since per-token scales have no per-channel integer form
    fixed = []
    for L in layers:
        qpi = P.make_qparams(P.CWAC_EPI_INT_OFFSET, False,
                             float(L.sx_row.mean()) if L.per_token else L.sx, L.zx, L.sr, L.zr)
        m0 = torch.empty(L.n, dtype=torch.int32, device=dev)
        sh = torch.empty(L.n, dtype=torch.int32, device=dev)
        fo = torch.empty(L.n, dtype=torch.int32, device=dev)
        P.cwac_fold_fixed_point(L.alpha, L.beta, L.sw, L.bias, L.colsum, qpi, m0, sh, fo)
        fixed.append((qpi, m0, sh, fo))

    def integer_only():
        for L, (qpi, m0, sh, fo) in zip(layers, fixed):
            P.qlinear_cwac_forward_fixed_point(L.xq, L.wq, qpi, m0, sh, fo, L.out)

    # the two fused variants run the same kernel on different parameter values, so what is measured
    # is drift: alternate them and take the median of the paired ratios
    pairs = []
    for i in range(6):
        if i % 2 == 0:
            tf = timed(fused)
            tp = timed(plain)
        else:  # alternate who goes first: the second of a pair runs on a warmer chip
            tp = timed(plain)
            tf = timed(fused)
        pairs.append((tf, tp))
    ratios = sorted(tf / tp for tf, tp in pairs)
    t_fused = sum(tf for tf, _ in pairs) / len(pairs)
    t_plain = sum(tp for _, tp in pairs) / len(pairs)
    overhead = (ratios[2] + ratios[3]) / 2 - 1.0
    t_unf = timed(unfused)
    # the integer-only epilogue against the fused one, alternated in the same way (the device's clock drifts
    # with what ran just before)
    ipairs = []
    for i in range(4):
        if i % 2 == 0:
            ti = timed(integer_only)
            tf = timed(fused)
        else:
            tf = timed(fused)
            ti = timed(integer_only)
        ipairs.append((ti, tf))
    iratios = sorted(ti / tf for ti, tf in ipairs)
    t_int = sum(ti for ti, _ in ipairs) / len(ipairs)
    return {"integer_only_epilogue_ms": round(t_int, 4),
            "integer_only_over_fp32_epilogue": round((iratios[1] + iratios[2]) / 2, 3),
            "fused_cwac_ms": round(t_fused, 4), "plain_ptq_same_kernel_ms": round(t_plain, 4),
            "cwac_overhead_vs_plain_ptq": round(overhead, 4),
            "unfused_gemm_int32_plus_epilogue_pass_ms": round(t_unf, 4),
            "unfused_over_fused": round(t_unf / t_fused, 3)}


def run_step_fused(P, layers):
    """The same step with the calibration side as ONE call (statistics in the GEMM's epilogue)."""
    for L in layers:
        P.cwac_stats_reset(L.stats, L.n)
        P.qlinear_cwac_calibrate_fused(L.xq_cal, L.wq, L.deq_mult, L.deq_off,
                                       L.deq_fb if L.bias is not None else None, L.sx_row_cal,
                                       L.y_full, L.stats, L.ws_fused)
        P.cwac_solve(L.stats, L.n, L.alpha, L.beta)
        P.cwac_fold(L.alpha, L.beta, L.sw, L.bias, L.colsum, L.qp, L.mult, L.offset, L.fbias)
        _forward_int8(P, L, L.mult, L.offset, L.fbias)


def fused_calibration(P, torch, layers, steps: int, reps: int = 5):
    """The calibration side of the step (Sec. 3.3) as one call: the statistics taken in the
    epilogue of the calibration GEMM, so that Y_quant never reaches memory, against the two calls
    the timed step uses (fp32 forward, then the statistics pass).  ms per pass over all layers;
    None where a layer's shape is outside the fused kernel's range."""
    dev = layers[0].xq.device
    if any(L.cal_rows < 256 or L.n < 256 or L.k % 128 or L.n % 4 for L in layers):
        return None
    ws = [torch.empty(P.cwac_calibrate_fused_workspace(L.cal_rows, L.n), dtype=torch.uint8,
                      device=dev) for L in layers]

    def two_calls():
        for L in layers:
            P.qlinear_cwac_forward(L.xq_cal, L.wq, None, L.deq_mult, L.deq_off,
                                   L.deq_fb if L.bias is not None else None, L.sx_row_cal,
                                   P.CWAC_OUT_FP32, L.yq)
            P.cwac_calibrate_stats_first(L.y_full, L.yq, L.stats, L.ws)

    def fused():
        for L, w in zip(layers, ws):
            P.cwac_stats_reset(L.stats, L.n)
            P.qlinear_cwac_calibrate_fused(L.xq_cal, L.wq, L.deq_mult, L.deq_off,
                                           L.deq_fb if L.bias is not None else None,
                                           L.sx_row_cal, L.y_full, L.stats, w)

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    t_a1, t_b1, t_a2, t_b2 = timed(two_calls), timed(fused), timed(two_calls), timed(fused)
    t_two, t_fused = (t_a1 + t_a2) / 2, (t_b1 + t_b2) / 2
    # the whole step with the fused calibration side, timed like the headline step
    for L, w in zip(layers, ws):
        L.ws_fused = w
    run_step_fused(P, layers)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        run_step_fused(P, layers)
    torch.cuda.synchronize()
    t_step = (time.perf_counter() - t0) / steps
    gemm_ops = sum(2.0 * (L.m + L.cal_rows) * L.n * L.k for L in layers)
    return {"forward_fp32_then_statistics_ms": round(t_two, 4), "fused_ms": round(t_fused, 4),
            "speedup": round(t_two / t_fused, 3),
            "whole_step_ms": round(t_step * 1e3, 4),
            "whole_step_tops": round(gemm_ops / t_step / 1e12, 2)}


def hbm_read_ceiling(P, torch, layers, reps: int = 3):
    """Context for roofline_stats.frac: the rate of a plain read-only stream (cwac_hbm_read_probe: 16-byte
    non-temporal loads at a grid stride) over the statistics pass's own inputs - every layer's Y_full, then the
    shared Y_quant buffer - so that, as in the step, each launch reads what the caches no longer hold."""
    dev = layers[0].y_full.device
    cus = torch.cuda.get_device_properties(dev).multi_processor_count
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    bufs = [L.y_full for L in layers] + [max((L.yq for L in layers), key=lambda t: t.numel())]
    out = {}
    for wgs_per_cu in (8, 16, 32):
        for b in bufs:
            P.cwac_hbm_read_probe(b, cus * wgs_per_cu, sink)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        nbytes = 0.0
        for _ in range(reps):
            for b in bufs:
                nbytes += P.cwac_hbm_read_probe(b, cus * wgs_per_cu, sink)
        e1.record()
        torch.cuda.synchronize()
        out[f"{wgs_per_cu}_workgroups_per_cu"] = round(nbytes / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1)
    best = max(out.values())
    return {"gbs": out, "best_gbs": best, "best_of_peak": round(best / HBM_PEAK_GBS, 4),
            "bytes_per_pass": sum(b.numel() * b.element_size() for b in bufs)}


def mfma_ceiling(P, torch, layers, iters: int = 20000, reps: int = 4):
    """Context for roofline.frac: the rate the int8 matrix cores sustain on THIS device with
    register-resident operands and no memory traffic (the forward kernel's 4 x 4 MFMA pattern),
    for constant operands, uniformly random bytes, and operand words sampled from the workload's
    own quantized weights and activations.  POP/s."""
    dev = layers[0].xq.device
    cus = torch.cuda.get_device_properties(dev).multi_processor_count
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    g = torch.Generator(device="cpu").manual_seed(1234)

    def sample(t):
        words = t.contiguous().view(-1).view(torch.int32).view(-1, 4)      # 16-byte operand chunks
        idx = torch.randint(0, words.shape[0], (512,), generator=g).to(dev)
        return words[idx]

    L = layers[0]
    variants = {
        "constant_operands": torch.full((1024, 4), 0x01010101, dtype=torch.int32, device=dev),
        "uniform_random_bytes": torch.randint(-2**31, 2**31 - 1, (1024, 4), generator=g,
                                              dtype=torch.int64).to(torch.int32).to(dev),
        "workload_operands": torch.cat([sample(L.wq), sample(L.xq)]).contiguous(),
    }
    out = {}
    for name, ops_buf in variants.items():
        P.cwac_mfma_probe(ops_buf, iters // 4, cus, sink)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        ops = 0.0
        for _ in range(reps):
            ops += P.cwac_mfma_probe(ops_buf, iters, cus, sink)
        e1.record()
        torch.cuda.synchronize()
        out[name] = round(ops / (e0.elapsed_time(e1) * 1e-3) / 1e15, 3)
    out["unit"] = "POP/s"
    out["workgroups"] = cus
    # the K loop of the forward's 256 x 256 tile, one ingredient at a time (workload operands everywhere)
    ops_buf = variants["workload_operands"]
    panels = torch.cat([sample(L.wq) for _ in range(4)] + [sample(L.xq) for _ in range(4)]).contiguous()   # 64 KiB
    names = ("mfma_only", "plus_lds_fragment_reads", "plus_stage_barrier", "plus_panel_stream",
             "panel_stream_issued_by_four_wavefronts")
    loop = {}
    for mode, name in enumerate(names):
        P.cwac_kloop_probe(ops_buf, panels, mode, iters // 8, cus, sink)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        ops = 0.0
        for _ in range(reps):
            ops += P.cwac_kloop_probe(ops_buf, panels, mode, iters // 2, cus, sink)
        e1.record()
        torch.cuda.synchronize()
        loop[name] = round(ops / (e0.elapsed_time(e1) * 1e-3) / 1e15, 3)
    out["k_loop_of_the_256_tile"] = loop
    return out


def setup_weight_only(P, synth, torch, cfg: int, dev: str):
    """Device-resident inputs of the weight-only step: INT4 group-128 weights in the kernel's
    streaming layout, fp16 activations, the upstream fp32 layer output."""
    wl = synth.WORKLOADS[cfg]
    m = wl.m
    layers = []
    for li, ly in enumerate(wl.layers):
        L = LayerState()
        L.n, L.k = ly.n, ly.k
        w = synth.weights(wl, li, device=dev)[0]
        L.x = synth.activations(wl, li, m, device=dev).to(torch.float16)
        L.xcal = synth.activations(wl, li, m, calibration=True, device=dev).to(torch.float16)
        L.y_full = L.xcal.float() @ w.t()                      # upstream full-precision layer
        L.wh = w.to(torch.float16)                             # comparator only: dense fp16 weights
        codes = torch.empty(ly.n, ly.k, dtype=torch.uint8, device=dev)
        sc = torch.empty(ly.n, ly.k // 128, dtype=torch.float16, device=dev)
        ze = torch.empty(ly.n, ly.k // 128, dtype=torch.uint8, device=dev)
        P.cwac_w4_quantize_groupwise(w, codes, sc, ze)
        L.pw = torch.empty(P.cwac_w4_packed_w_bytes(ly.n, ly.k), dtype=torch.uint8, device=dev)
        L.psz = torch.empty((ly.k // 128) * ly.n, dtype=torch.int32, device=dev)
        P.cwac_w4_pack(codes, sc, ze, L.pw, L.psz)
        f32 = dict(dtype=torch.float32, device=dev)
        L.alpha, L.beta = torch.empty(ly.n, **f32), torch.empty(ly.n, **f32)
        L.mult, L.fbias = torch.empty(ly.n, **f32), torch.empty(ly.n, **f32)
        L.stats = torch.empty(P.cwac_stats_bytes(ly.n) // 8 + 2, dtype=torch.float64, device=dev)
        L.ws = torch.empty(P.cwac_calibrate_stats_workspace(m, ly.n), dtype=torch.uint8, device=dev)
        del w, codes, sc, ze
        layers.append(L)
    n_max = max(L.n for L in layers)
    yq_buf = torch.empty(m * n_max, dtype=torch.float32, device=dev)
    out_buf = torch.empty(m * n_max, dtype=torch.float16, device=dev)
    for L in layers:
        L.yq = yq_buf[:m * L.n].view(m, L.n)
        L.out = out_buf[:m * L.n].view(m, L.n)
    torch.cuda.synchronize()
    return layers


def run_step_weight_only(P, layers, ev=None):
    """fp32 calibration forward -> statistics -> fit -> fold -> compensated fp16 forward, per layer."""
    import torch
    for L in layers:
        e = [torch.cuda.Event(enable_timing=True) for _ in range(4)] if ev is not None else None
        if e:
            e[0].record()
        P.qlinear_w4a16_cwac_forward(L.xcal, L.pw, L.psz, L.n, None, None, L.yq)
        if e:
            e[1].record()
        P.cwac_calibrate_stats_first(L.y_full, L.yq, L.stats, L.ws)
        P.cwac_solve(L.stats, L.n, L.alpha, L.beta)
        P.cwac_fold_weight_only(L.alpha, L.beta, None, L.mult, L.fbias)
        if e:
            e[2].record()
        P.qlinear_w4a16_cwac_forward(L.x, L.pw, L.psz, L.n, L.mult, L.fbias, L.out)
        if e:
            e[3].record()
            ev.append(e)


def weight_only_int4(P, synth, torch, cfg: int, dev: str, steps: int, cpu_rows: int):
    """The paper's LLM setting on the same layer shapes: INT4 group-128 weights, fp16 activations,
    CWAC in the epilogue.  A step = calibration forward (fp32 out) -> statistics -> fit -> fold ->
    compensated fp16 forward, for every layer; the fp16 forward is the kernel the roofline is for."""
    import numpy as np
    wl = synth.WORKLOADS[cfg]
    m = wl.m
    layers = setup_weight_only(P, synth, torch, cfg, dev)

    def step(ev=None):
        run_step_weight_only(P, layers, ev)

    for _ in range(2):
        step()
    torch.cuda.synchronize()
    ev = []
    t0 = time.perf_counter()
    for _ in range(steps):
        step(ev)
    torch.cuda.synchronize()
    t_step = (time.perf_counter() - t0) / steps
    fwd_flops = sum(2.0 * m * L.n * L.k for L in layers)
    t_cal = sum(e[0].elapsed_time(e[1]) for e in ev) / steps
    t_fit = sum(e[1].elapsed_time(e[2]) for e in ev) / steps
    t_fwd = sum(e[2].elapsed_time(e[3]) for e in ev) / steps
    # comparator: the vendor library's dense fp16 GEMM on the same activations and un-quantized
    # fp16 weights (no 4-bit expansion, no epilogue vectors, 4x the weight bytes)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for L in layers:
        torch.matmul(L.x, L.wh.t(), out=L.out)
    e0.record()
    for _ in range(steps):
        for L in layers:
            torch.matmul(L.x, L.wh.t(), out=L.out)
    e1.record()
    torch.cuda.synchronize()
    t_dense = e0.elapsed_time(e1) / steps
    tf = fwd_flops / (t_fwd * 1e-3) / 1e12
    res = {
        "workload": f"config {wl.cfg} layer shapes, INT4 group-128 asymmetric weights, fp16 "
                    f"activations, M={m} tokens, {m} calibration rows per step",
        "dtype": "f16", "ms_per_step": round(t_step * 1e3, 4),
        "value": round(2.0 * fwd_flops / t_step / 1e12, 2), "unit": "TFLOP/s",
        "roofline": {"bound": "mfma", "achieved": round(tf / 1e3, 4),
                     "peak": FP16_MFMA_PEAK_TFLOPS / 1e3, "unit": "PFLOP/s",
                     "frac": round(tf / FP16_MFMA_PEAK_TFLOPS, 4),
                     "traffic": PMC_TRAFFIC_BYTES.get(wl.cfg, {}).get("forward_w4a16"),
                     "traffic_source": "profiles/bench_config5_w4a16_pmc.md (constant from that profile, not measured "
                                       "in this run)",
                     "kernel": "w4a16_kernel (fp16 out, fused CWAC epilogue)",
                     "launches_per_step": len(layers), "avg_launch_ms": round(t_fwd / len(layers), 4),
                     "flops_per_step": fwd_flops},
        "phases_ms": {"calibration_forward_fp32": round(t_cal, 4),
                      "statistics_solve_fold": round(t_fit, 4), "forward_fp16": round(t_fwd, 4)},
        "calibration_forward_tflops": round(fwd_flops / (t_cal * 1e-3) / 1e12, 2),
        "dense_fp16_library_gemm_tflops": round(fwd_flops / (t_dense * 1e-3) / 1e12, 2),
    }
    # the same forward with the earlier 256 x 256 tile, and both (and the library GEMM) on zero activations, which
    # draw the least power in the matrix cores: what the kernels' own pipelines allow
    def fwd_pass(xs, tun):
        for L, x in zip(layers, xs):
            P.qlinear_w4a16_cwac_forward(x, L.pw, L.psz, L.n, L.mult, L.fbias, L.out, tuning=tun)

    def dense_pass(xs, tun):
        for L, x in zip(layers, xs):
            torch.matmul(x, L.wh.t(), out=L.out)

    def timed(fn, xs, tun=None):
        fn(xs, tun)
        e0.record()
        for _ in range(steps):
            fn(xs, tun)
        e1.record()
        torch.cuda.synchronize()
        return round(fwd_flops / (e0.elapsed_time(e1) / steps * 1e-3) / 1e12, 2)

    xs_w = [L.x for L in layers]
    zero = torch.zeros(m, max(L.k for L in layers), dtype=torch.float16, device=dev)
    xs_0 = [zero[:, :L.k] for L in layers]
    t256 = P.make_tuning(w4_tile=256)
    res["tile_and_operand_comparison_tflops"] = {
        "forward_fp16": timed(fwd_pass, xs_w), "forward_fp16_256x256_tile": timed(fwd_pass, xs_w, t256),
        "forward_fp16_zero_activations": timed(fwd_pass, xs_0),
        "forward_fp16_256x256_tile_zero_activations": timed(fwd_pass, xs_0, t256),
        "dense_fp16_library_gemm": timed(dense_pass, xs_w),
        "dense_fp16_library_gemm_zero_activations": timed(dense_pass, xs_0)}
    del zero, xs_0
    # context for roofline.frac: what the binary16 matrix cores sustain on this device with register-resident
    # operands sampled from this workload (weight values of layer 0 in fp16, its activations), no memory traffic
    cus = torch.cuda.get_device_properties(dev).multi_processor_count
    g = torch.Generator(device="cpu").manual_seed(4321)
    sink = torch.zeros(1, dtype=torch.int32, device=dev)

    def sample16(t):
        v = t.contiguous().view(-1)[:(t.numel() // 8) * 8].view(-1, 8)        # 16-byte operand chunks
        return v[torch.randint(0, v.shape[0], (512,), generator=g).to(dev)]

    probes = {"zero_operands": torch.zeros(1024, 8, dtype=torch.float16, device=dev),
              "workload_operands": torch.cat([sample16(layers[0].wh), sample16(layers[0].x)]).contiguous()}
    ceiling = {}
    for name, ops_buf in probes.items():
        P.cwac_mfma_probe_f16(ops_buf, 5000, cus, sink)
        torch.cuda.synchronize()
        e0.record()
        fl = 0.0
        for _ in range(4):
            fl += P.cwac_mfma_probe_f16(ops_buf, 20000, cus, sink)
        e1.record()
        torch.cuda.synchronize()
        ceiling[name] = round(fl / (e0.elapsed_time(e1) * 1e-3) / 1e15, 3)
    ceiling["unit"] = "PFLOP/s"
    res["mfma_ceiling_probe_f16"] = ceiling
    # decode-sized batches (8 tokens): the layer is a stream of 4-bit weights; 20 passes over the
    # five layers replayed from a HIP graph (a launch from Python costs as much as the kernel)
    sm = 8
    outs = [torch.empty(sm, L.n, dtype=torch.float16, device=dev) for L in layers]
    # Every pass streams its own copy of the packed weights: four copies of the five layers (4 x 101 MB) cycle,
    # more than the 256 MB last-level cache holds, so that the bytes of a pass really come from HBM (a decoder
    # has tens of such layers; one copy replayed would sit in that cache)
    copies = 4
    reps = [[(L.pw, L.psz) if c == 0 else (L.pw.clone(), L.psz.clone()) for L in layers] for c in range(copies)]

    def small_pass(c):
        for (pw, psz), L, o in zip(reps[c], layers, outs):
            P.qlinear_w4a16_cwac_forward(L.x[:sm], pw, psz, L.n, L.mult, L.fbias, o)

    for c in range(copies):
        small_pass(c)
    torch.cuda.synchronize()
    passes = 5 * copies
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            for i in range(passes):
                small_pass(i % copies)
    g.replay()
    torch.cuda.synchronize()
    e0.record()
    g.replay()
    e1.record()
    torch.cuda.synchronize()
    t_small = e0.elapsed_time(e1) / passes                  # ms per pass over the layers
    small_bytes = sum(L.n * L.k / 2 + L.n * (L.k // 128) * 4 + sm * L.k * 2 + sm * L.n * 2 for L in layers)
    gbs = small_bytes / (t_small * 1e-3) / 1e9
    res["small_batch"] = {
        "tokens": sm, "us_per_layer": round(t_small * 1e3 / len(layers), 2),
        "weights": f"{copies} copies of the packed layers cycle ({copies * small_bytes / 1e6:.0f} MB), so every pass reads "
                   "its weights from HBM",
        "roofline": {"bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": None,
                     "kernel": "w4a16_small_m_kernel (fp16 out, fused CWAC epilogue)",
                     "bytes_per_pass": small_bytes}}
    del reps
    if cpu_rows > 0:
        from oracle import cwac_oracle as orc
        from oracle import w4a16_oracle as w4
        flops, secs = 0.0, 0.0
        for li, ly in enumerate(wl.layers):
            w = synth.weights(wl, li)[0].numpy()
            x16 = synth.activations(wl, li, cpu_rows).numpy().astype(np.float16)
            xc16 = synth.activations(wl, li, cpu_rows, calibration=True).numpy().astype(np.float16)
            y_full = (xc16.astype(np.float32) @ w.T).astype(np.float32)        # upstream
            codes, sc, ze = w4.quantize_groupwise(w)                             # setup
            t0 = time.perf_counter()                                             # the step
            wd = w4.dequant(codes, sc, ze)
            acc_c, _ = w4.product(xc16, wd)
            alpha, beta = orc.fit(y_full, acc_c.astype(np.float32))
            mult, fb = w4.fold(alpha, beta, None, ly.n)
            acc, _ = w4.product(x16, wd)
            w4.folded_real(acc, mult, fb)
            secs += time.perf_counter() - t0
            flops += 2.0 * 2.0 * cpu_rows * ly.n * ly.k
        res["cpu_baseline"] = {"value": round(flops / secs / 1e12, 5), "unit": "TFLOP/s",
                               "cores": orc.get_threads(), "kind": "oracle",
                               "sample": f"the same step on {cpu_rows} inference rows and {cpu_rows} "
                                         f"calibration rows of every layer ({secs:.1f} s of oracle time)"}
    return res


# ResNet-50 bottleneck convolutions (stages 2-5; H = W of the layer's input at 224 x 224 images):
# name, H, C_in, C_out, filter, stride, padding
RESNET50_CONVS = (
    ("s2 1x1 256->64", 56, 256, 64, 1, 1, 0), ("s2 3x3 64->64", 56, 64, 64, 3, 1, 1),
    ("s2 1x1 64->256", 56, 64, 256, 1, 1, 0),
    ("s3 1x1 512->128", 28, 512, 128, 1, 1, 0), ("s3 3x3 128->128", 28, 128, 128, 3, 1, 1),
    ("s3 1x1 128->512", 28, 128, 512, 1, 1, 0),
    ("s4 1x1 1024->256", 14, 1024, 256, 1, 1, 0), ("s4 3x3 256->256", 14, 256, 256, 3, 1, 1),
    ("s4 1x1 256->1024", 14, 256, 1024, 1, 1, 0),
    ("s5 1x1 2048->512", 7, 2048, 512, 1, 1, 0), ("s5 3x3 512->512", 7, 512, 512, 3, 1, 1),
    ("s5 1x1 512->2048", 7, 512, 2048, 1, 1, 0),
    ("s3 3x3/2 128->128", 56, 128, 128, 3, 2, 1), ("s4 3x3/2 256->256", 28, 256, 256, 3, 2, 1),
    ("s5 3x3/2 512->512", 14, 512, 512, 3, 2, 1),
)


def conv_section(P, synth, torch, dev: str, batch: int, steps: int, cpu_batch: int):
    """Quantized convolutional layers with the CWAC epilogue (Sec. 3.3-3.4 applied to a CNN): the 15
    distinct bottleneck convolutions of ResNet-50 on synthetic post-ReLU images.  A step = for every
    layer: calibration forward (fp32 out) -> statistics -> fit -> fold -> compensated int8 forward;
    the int8 forward is the kernel the roofline is for.  Y_full comes from torch's fp32 convolution
    (upstream of the path, set-up)."""
    import numpy as np
    import torch.nn.functional as F
    f32 = dict(dtype=torch.float32, device=dev)
    layers = []
    for li, (name, h, c, n, k, stride, pad) in enumerate(RESNET50_CONVS):
        L = LayerState()
        L.name, L.h, L.c, L.n, L.kf, L.stride, L.pad = name, h, c, n, k, stride, pad
        L.oh = (h + 2 * pad - k) // stride + 1
        L.m, L.k = batch * L.oh * L.oh, k * k * c
        seed = 7000 + li
        xf = torch.relu(synth.normal(seed, 0, batch * h * h * c, device=dev)).view(batch, h, h, c)
        xf[..., 3::37] *= 6.0                                     # a few strong channels
        wf = (synth.normal(seed, 1, n * k * k * c, device=dev) * (2.0 / L.k) ** 0.5).view(n, L.k)
        L.bias = synth.normal(seed, 2, n, device=dev) * 0.05
        L.wq = torch.empty(n, L.k, dtype=torch.int8, device=dev)
        L.sw = torch.empty(n, **f32)
        P.cwac_quantize_rows_sym(wf, L.sw, L.wq)
        L.colsum = torch.empty(n, dtype=torch.int32, device=dev)
        P.cwac_colsum(L.wq, L.colsum)
        mm = torch.empty(2, **f32)
        ws = torch.empty(P.cwac_range_workspace(xf.numel()), dtype=torch.uint8, device=dev)
        P.cwac_range_f32(xf, mm, ws)
        mn, mx = (float(v) for v in mm.cpu())
        L.sx, z_u = P.cwac_qparams_from_range(mn, mx, 8)
        L.zx = z_u - 128
        L.xq = torch.empty(batch, h, h, c, dtype=torch.int8, device=dev)
        P.cwac_quantize_act(xf.view(-1, c), L.sx, L.zx, L.xq.view(-1, c))
        w4 = wf.view(n, k, k, c).permute(0, 3, 1, 2).contiguous()
        L.y_full = (F.conv2d(xf.permute(0, 3, 1, 2), w4, L.bias, stride=stride, padding=pad)
                    .permute(0, 2, 3, 1).reshape(L.m, n).contiguous())
        ws = torch.empty(P.cwac_range_workspace(L.y_full.numel()), dtype=torch.uint8, device=dev)
        P.cwac_range_f32(L.y_full, mm, ws)
        mn, mx = (float(v) for v in mm.cpu())
        L.sr, zr_u = P.cwac_qparams_from_range(mn, mx, 8)
        L.zr = zr_u - 128
        L.qp = P.make_qparams(P.CWAC_EPI_INT_OFFSET, False, L.sx, L.zx, L.sr, L.zr)
        L.qp_deq = P.make_qparams(P.CWAC_EPI_FP_BIAS, False, L.sx, L.zx, 1.0, 0)
        L.deq_mult, L.deq_fb = torch.empty(n, **f32), torch.empty(n, **f32)
        L.deq_off = torch.empty(n, dtype=torch.int32, device=dev)
        P.cwac_fold(None, None, L.sw, L.bias, L.colsum, L.qp_deq, L.deq_mult, L.deq_off, L.deq_fb)
        L.mult, L.offset = torch.empty(n, **f32), torch.empty(n, dtype=torch.int32, device=dev)
        L.alpha, L.beta = torch.empty(n, **f32), torch.empty(n, **f32)
        L.stats = torch.empty(P.cwac_stats_bytes(n) // 8 + 2, dtype=torch.float64, device=dev)
        L.ws = torch.empty(P.cwac_calibrate_stats_workspace(L.m, n), dtype=torch.uint8, device=dev)
        L.wq4 = L.wq.view(n, k, k, c)
        L.xf_cpu = xf[:cpu_batch].cpu().numpy() if cpu_batch else None
        L.wf_cpu = wf.cpu().numpy() if cpu_batch else None
        del xf, wf, w4
        layers.append(L)
    mn_max = max(L.m * L.n for L in layers)
    yq_buf = torch.empty(mn_max, **f32)
    out_buf = torch.empty(mn_max, dtype=torch.int8, device=dev)
    for L in layers:
        L.yq, L.out = yq_buf[:L.m * L.n].view(L.m, L.n), out_buf[:L.m * L.n].view(L.m, L.n)
    torch.cuda.synchronize()

    def step(ev=None):
        for L in layers:
            if ev is not None:
                e = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
                e[0].record()
            P.qconv2d_cwac_forward(L.xq, L.wq4, L.stride, L.pad, L.qp_deq, L.deq_mult, L.deq_off, L.deq_fb,
                                   P.CWAC_OUT_FP32, L.yq)
            if ev is not None:
                e[1].record()
            P.cwac_calibrate_stats_first(L.y_full, L.yq, L.stats, L.ws)
            P.cwac_solve(L.stats, L.n, L.alpha, L.beta)
            P.cwac_fold(L.alpha, L.beta, L.sw, L.bias, L.colsum, L.qp, L.mult, L.offset)
            if ev is not None:
                e[2].record()
            P.qconv2d_cwac_forward(L.xq, L.wq4, L.stride, L.pad, L.qp, L.mult, L.offset, None,
                                   P.CWAC_OUT_INT8, L.out)
            if ev is not None:
                e[3].record()
                ev.append(e)

    for _ in range(2):
        step()
    torch.cuda.synchronize()
    ev = []
    t0 = time.perf_counter()
    for _ in range(steps):
        step(ev)
    torch.cuda.synchronize()
    t_step = (time.perf_counter() - t0) / steps
    nl = len(layers)
    fwd_ops = sum(2.0 * L.m * L.n * L.k for L in layers)
    t_cal = sum(e[0].elapsed_time(e[1]) for e in ev) / steps
    t_fit = sum(e[1].elapsed_time(e[2]) for e in ev) / steps
    t_fwd = sum(e[2].elapsed_time(e[3]) for e in ev) / steps
    per_layer = []
    for i, L in enumerate(layers):
        us = sum(ev[s * nl + i][2].elapsed_time(ev[s * nl + i][3]) for s in range(steps)) / steps * 1e3
        nbytes = L.xq.numel() + L.wq.numel() + L.m * L.n        # image + filter + int8 output, each once
        per_layer.append({"layer": L.name, "m": L.m, "n": L.n, "k": L.k, "us": round(us, 1),
                          "tops": round(2.0 * L.m * L.n * L.k / us / 1e6, 1),
                          "algorithmic_gbs": round(nbytes / us / 1e3, 1)})
    tops = fwd_ops / (t_fwd * 1e-3) / 1e12
    res = {
        "metric": "int8 convolution + CWAC epilogue TOPS (% int8 MFMA peak)",
        "value": round(2.0 * fwd_ops / t_step / 1e12, 2), "unit": "TOPS", "n_gpus": 1, "steps": steps,
        "warmup": 2, "ms_per_step": round(t_step * 1e3, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": f"ResNet-50 bottleneck convolutions (15 distinct layers of stages 2-5), "
                               f"batch {batch}, channels-last int8 images, per-tensor activations"},
        "roofline": {"bound": "mfma", "achieved": round(tops / 1e3, 4), "peak": INT8_MFMA_PEAK_TOPS / 1e3,
                     "unit": "POP/s", "frac": round(tops / INT8_MFMA_PEAK_TOPS, 4), "traffic": None,
                     "kernel": "qlinear_fast_kernel / qlinear_persist_kernel / qlinear_kernel as the dispatcher picks per layer "
                               "(int8 out, fused CWAC epilogue)",
                     "launches_per_step": nl, "avg_launch_ms": round(t_fwd / nl, 4),
                     "ops_per_step": fwd_ops},
        "phases_ms": {"calibration_forward_fp32": round(t_cal, 4),
                      "statistics_solve_fold": round(t_fit, 4), "forward_int8": round(t_fwd, 4)},
        "layers": per_layer,
    }
    if cpu_batch > 0:
        from oracle import cwac_oracle as orc
        ops, secs = 0.0, 0.0
        for L in layers:
            xf, wf = L.xf_cpu, L.wf_cpu
            bias = L.bias.cpu().numpy()
            wq, sw = orc.quantize_rows_sym(wf)                       # set-up
            colsum = orc.colsum_i8(wq)
            xq = orc.quantize_act_i8(xf, L.sx, L.zx)
            y_full = L.y_full[:cpu_batch * L.oh * L.oh].cpu().numpy()
            wq4 = wq.reshape(L.n, L.kf, L.kf, L.c)
            t0 = time.perf_counter()                                 # the step
            acc = orc.conv2d_i8(xq, wq4, L.stride, L.pad, L.zx)
            y_quant = orc.dequant_output(acc, colsum, L.zx, orc.deq_scale(sw, L.sx), bias)
            alpha, beta = orc.fit(y_full, y_quant)[:2]
            mult, offset, _ = orc.fold_int_offset(alpha, beta, sw, bias, colsum, L.sx, L.zx, L.sr)
            acc = orc.conv2d_i8(xq, wq4, L.stride, L.pad, L.zx)
            orc.folded_forward(acc, offset, mult, L.zr)
            secs += time.perf_counter() - t0
            ops += 2.0 * 2.0 * cpu_batch * L.oh * L.oh * L.n * L.k
        res["cpu_baseline"] = {"value": round(ops / secs / 1e12, 5), "unit": "TOPS",
                               "cores": orc.get_threads(), "kind": "oracle",
                               "sample": f"the same step on {cpu_batch} images of every layer "
                                         f"({secs:.1f} s of oracle time)"}
    return res



def block_section(P, torch, dev: str, batch: int, steps: int, warmup: int, cpu_images: int, n_blocks: int = 12,
                  shape=(197, 12, 64, 3072)):
    """One W8A8 Vision Transformer block (ViT-B/16: 197 tokens, 12 heads, MLP 3072) from residual
    stream to residual stream: the four compensated linear layers (Sec. 3.4) chained with the
    non-linear glue that per-layer compensation steps around (Sec. 3.2).  A step = one call of
    vit_block_w8a8_forward (eight launches); every stage is also timed alone."""
    import numpy as np
    sys.path.insert(0, os.path.join(ROOT, "tests"))   # the block's set-up (an upstream fp32 model in torch) is a fixture
    import vit_block_fixture as vit_block
    tokens, heads, head_dim, hidden = shape
    blk = vit_block.build_block(2, batch, tokens, heads, hidden, device=dev, head_dim=head_dim)
    m, c = blk.m, blk.c
    h = vit_block.residual_stream(2, m, c, dev)
    h_out = torch.empty_like(h)
    ws = torch.empty(P.vit_block_workspace(batch, tokens, heads, hidden), dtype=torch.int8, device=dev)
    for _ in range(warmup):
        P.vit_block_w8a8_forward(blk.params, h, h_out, ws)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        P.vit_block_w8a8_forward(blk.params, h, h_out, ws)
    e1.record()
    torch.cuda.synchronize()
    t_step = (time.perf_counter() - t0) / steps
    ms_block = e0.elapsed_time(e1) / steps

    # the same call replayed from a HIP graph (eight kernel nodes)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            P.vit_block_w8a8_forward(blk.params, h, h_out, ws)
    torch.cuda.current_stream().wait_stream(side)
    graph.replay()
    torch.cuda.synchronize()
    e0.record()
    for _ in range(steps):
        graph.replay()
    e1.record()
    torch.cuda.synchronize()
    ms_graph = e0.elapsed_time(e1) / steps

    # a stack of n_blocks such blocks in one call (ViT-B/16's encoder is 12): between two blocks the last
    # residual of one and the LN1 + quantizer of the next are one pass; the stream is updated in place
    stack = [blk] + [vit_block.build_block(100 + i, batch, tokens, heads, hidden, device=dev, head_dim=head_dim)
                     for i in range(1, n_blocks)]
    stack_params = [b.params for b in stack]
    hs = h.clone()
    for _ in range(2):
        P.vit_encoder_w8a8_forward(stack_params, h, hs, ws)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(steps):
        P.vit_encoder_w8a8_forward(stack_params, h, hs, ws)
    e1.record()
    torch.cuda.synchronize()
    ms_stack = e0.elapsed_time(e1) / steps

    t = vit_block.staged_forward(blk, h)
    L = blk.layers
    B = P.binding

    def timed(fn, reps=20):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps * 1e3  # us

    def linear(i, x, out):
        qp = B.make_qparams(mode=B.CWAC_EPI_INT_OFFSET, s_x=L[i]["s_x"], z_x=L[i]["z_x"], s_r=L[i]["s_r"],
                            z_r=L[i]["z_r"])
        return lambda: B.qlinear_cwac_forward(x, L[i]["w_q"], qp, L[i]["mult"], L[i]["offset"], None, None,
                                              B.CWAC_OUT_INT8, out)

    stages = [
        ("ln1_quant", lambda: B.vit_residual_ln_quant(h, None, 0.0, 0, None, blk.ln[0], blk.ln[1], blk.eps,
                                                      L[0]["s_x"], L[0]["z_x"], t["x1"]), "hbm", 3.0 * m * c),
        ("qkv", linear(0, t["x1"], t["r1"]), "mfma", 2.0 * m * 3 * c * c),
        ("attention", lambda: B.vit_attention_int8(t["r1"], L[0]["s_r"], L[0]["z_r"], batch, tokens, heads,
                                                   L[1]["s_x"], L[1]["z_x"], t["a"], head_dim=head_dim), "mfma_f16",
         4.0 * batch * heads * tokens * tokens * head_dim),
        ("proj", linear(1, t["a"], t["r2"]), "mfma", 2.0 * m * c * c),
        ("residual_ln2_quant", lambda: B.vit_residual_ln_quant(h, t["r2"], L[1]["s_r"], L[1]["z_r"], t["h1"], blk.ln[2],
                                                               blk.ln[3], blk.eps, L[2]["s_x"], L[2]["z_x"], t["x2"]),
         "hbm", 6.0 * m * c),
        ("fc1_with_gelu_table", lambda: B.qlinear_cwac_forward_table(
            t["x2"], L[2]["w_q"], B.make_qparams(mode=B.CWAC_EPI_INT_OFFSET, s_x=L[2]["s_x"], z_x=L[2]["z_x"],
                                                 s_r=L[2]["s_r"], z_r=L[2]["z_r"]),
            L[2]["mult"], L[2]["offset"], blk.gelu_table, t["g"]), "mfma", 2.0 * m * hidden * c),
        ("fc2", linear(3, t["g"], t["r4"]), "mfma", 2.0 * m * c * hidden),
        ("residual", lambda: B.vit_residual_ln_quant(t["h1"], t["r4"], L[3]["s_r"], L[3]["z_r"], t["h2"], None, None,
                                                     0.0, 1.0, 0, None), "hbm", 5.0 * m * c),
    ]
    per_stage, lin_us, glue_us = [], 0.0, 0.0
    for name, fn, bound, work in stages:
        us = timed(fn)
        ent = {"stage": name, "us": round(us, 1), "bound": bound}
        if bound == "hbm":
            ent["algorithmic_gbs"] = round(work / us / 1e3, 1)
            ent["frac"] = round(work / us / 1e3 / HBM_PEAK_GBS, 4)
            glue_us += us
        elif bound == "mfma":
            ent["tops"] = round(work / us / 1e6, 1)
            ent["frac"] = round(work / us / 1e6 / INT8_MFMA_PEAK_TOPS, 4)
            lin_us += us
        else:
            ent["tflops"] = round(work / us / 1e6, 1)
            ent["frac"] = round(work / us / 1e6 / 2500.0, 4)
            glue_us += us
        per_stage.append(ent)
    # what the table in fc1's epilogue replaces: the plain forward and a lookup pass over its output
    unfused_us = timed(linear(2, t["x2"], t["r3"])) + timed(lambda: B.vit_table_lookup(t["r3"], blk.gelu_table, t["g"]))
    lin_ops = 2.0 * m * c * (3 * c + c + 2 * hidden)
    att = next(e for e in per_stage if e["stage"] == "attention")
    res = {
        "metric": "W8A8 Transformer block forward, linear-layer TOPS over the whole block's time",
        "value": round(lin_ops / (ms_block * 1e-3) / 1e12, 2), "unit": "TOPS", "n_gpus": 1, "steps": steps,
        "warmup": warmup, "ms_per_step": round(t_step * 1e3, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": f"{'ViT-B/16' if shape == (197, 12, 64, 3072) else 'Transformer'} block, {batch} images "
                               f"(attending units) x {tokens} tokens, {heads} heads x {head_dim}, MLP {hidden}, "
                               f"per-tensor int8 activations, binary16 residual stream"},
        "block_ms": round(ms_block, 4), "images_per_s": round(batch / (ms_block * 1e-3), 1),
        "graph_replay_ms": round(ms_graph, 4),
        "encoder_stack": {"blocks": n_blocks, "ms": round(ms_stack, 4), "ms_per_block": round(ms_stack / n_blocks, 4),
                          "images_per_s": round(batch / (ms_stack * 1e-3), 1),
                          "linear_layer_tops": round(n_blocks * 2.0 * m * c * (3 * c + c + 2 * hidden)
                                                     / (ms_stack * 1e-3) / 1e12, 1)},
        "linear_layers_us": round(lin_us, 1), "glue_us": round(glue_us, 1),
        "glue_share_of_stage_sum": round(glue_us / (glue_us + lin_us), 4),
        "fc1_then_table_lookup_pass_us": round(unfused_us, 1),
        # the dominant kernel of the block: the int8 forward (four launches, one with the GELU table)
        "roofline": {"bound": "mfma", "achieved": round(lin_ops / lin_us / 1e9, 4), "peak": INT8_MFMA_PEAK_TOPS / 1e3,
                     "unit": "POP/s", "frac": round(lin_ops / lin_us / 1e6 / INT8_MFMA_PEAK_TOPS, 4), "traffic": None,
                     "kernel": "qlinear_persist_kernel (int8 out, fused CWAC epilogue, fc1 with the GELU code table; K = 768 / 3072)",
                     "launches_per_step": 4, "avg_launch_ms": round(lin_us / 4e3, 4), "ops_per_step": lin_ops},
        "roofline_attention": {"bound": "mfma", "achieved": round(att["tflops"] / 1e3, 4), "peak": 2.5,
                               "unit": "PFLOP/s", "frac": att["frac"], "traffic": None,
                               "kernel": ("attention_int8_kernel" if tokens <= 224 else "attention_long_kernel")
                                         + " (the longest glue stage; fp16 MFMA, 4 T^2 d flops "
                                         "per head; bound by its vector work, not by the matrix cores)"},
        "stages": per_stage,
    }
    if cpu_images > 0:
        from oracle import block_oracle as blk_o
        from oracle import cwac_oracle as orc
        rows = cpu_images * tokens
        cpu = {k: v[:rows].cpu().numpy() for k, v in t.items()}
        hh = h[:rows].cpu().numpy()
        ln = [x.cpu().numpy() for x in blk.ln]
        t0 = time.perf_counter()
        x1, _ = blk_o.quantize(blk_o.layernorm(hh, ln[0], ln[1], blk.eps), L[0]["s_x"], L[0]["z_x"])
        fwd = lambda i, x: orc.folded_forward(orc.gemm_i8(x, L[i]["w_q"].cpu().numpy()),  # noqa: E731
                                              L[i]["offset"].cpu().numpy(), L[i]["mult"].cpu().numpy(), L[i]["z_r"])
        r1 = fwd(0, x1)
        o, _ = blk_o.attention_codes(r1, L[0]["s_r"], L[0]["z_r"], cpu_images, tokens, heads)
        a, _ = blk_o.quantize(o, L[1]["s_x"], L[1]["z_x"])
        r2 = fwd(1, a)
        h1, _ = blk_o.residual(hh, r2, L[1]["s_r"], L[1]["z_r"])
        x2, _ = blk_o.quantize(blk_o.layernorm(h1, ln[2], ln[3], blk.eps), L[2]["s_x"], L[2]["z_x"])
        r3 = fwd(2, x2)
        tab, _ = blk_o.gelu_table(L[2]["s_r"], L[2]["z_r"], L[3]["s_x"], L[3]["z_x"])
        g = tab[r3.astype(int) + 128]
        r4 = fwd(3, g)
        blk_o.residual(h1, r4, L[3]["s_r"], L[3]["z_r"])
        secs = time.perf_counter() - t0
        agree = float((r4 == cpu["r4"]).mean())
        worst = int(np.abs(r4.astype(int) - cpu["r4"].astype(int)).max())
        res["cpu_baseline"] = {"value": round(2.0 * rows * c * (3 * c + c + 2 * hidden) / secs / 1e12, 5), "unit": "TOPS",
                               "cores": orc.get_threads(), "kind": "oracle",
                               "sample": f"the same block on {cpu_images} images ({secs:.1f} s of oracle time; its "
                                         f"fc2 output codes equal the GPU's on {agree:.4f} of the elements, largest "
                                         f"difference {worst} - the glue's rounding (binary16 attention weights, fp32 "
                                         f"ties) carried through the chain; parity is tested stage by stage)"}
    return res


def cpu_baseline(synth, cfg: int, sample_rows: int):
    """The oracle, as it stands, timed on this host on a bounded row sample of the same step."""
    import numpy as np
    from oracle import cwac_oracle as orc
    wl = synth.WORKLOADS[cfg]
    ops = 0.0
    t_total = 0.0
    for li, ly in enumerate(wl.layers):
        w, b = synth.weights(wl, li)
        w = w.numpy()
        b = None if b is None else b.numpy()
        x = synth.activations(wl, li, sample_rows).numpy()
        xcal = synth.activations(wl, li, sample_rows, calibration=True).numpy()
        y_full = (xcal @ w.T + (0 if b is None else b[None, :])).astype(np.float32)  # upstream
        wq, sw = orc.quantize_rows_sym(w)                                            # setup
        colsum = orc.colsum_i8(wq)
        if wl.per_token:
            xq, sxr = orc.quantize_rows_sym(x)
            xqc, sxrc = orc.quantize_rows_sym(xcal)
            sx, zx, deq = np.float32(1.0), 0, sw
        else:
            mn, mx = orc.range_f32(xcal)
            sx, z_u = orc.qparams_asym(mn, mx, 8)
            zx = z_u - 128
            xq, xqc = orc.quantize_act_i8(x, sx, zx), orc.quantize_act_i8(xcal, sx, zx)
            sxr = sxrc = None
            deq = orc.deq_scale(sw, sx)
        mn, mx = orc.range_f32(y_full)
        sr, zr_u = orc.qparams_asym(mn, mx, 8)
        t0 = time.perf_counter()                                                      # the step
        acc_c = orc.gemm_i8(xqc, wq)
        yq = orc.dequant_output(acc_c, colsum, zx, deq, b, sxrc)
        mom = orc.channel_moments(y_full, yq)
        alpha, beta, _ = orc.solve(mom)
        if wl.per_token:
            mult, fb, off = orc.fold_fp_bias(alpha, beta, sw, b, colsum, True, sx, zx, sr)
        else:
            mult, off, _ = orc.fold_int_offset(alpha, beta, sw, b, colsum, sx, zx, sr)
            fb = None
        acc = orc.gemm_i8(xq, wq)
        orc.folded_forward(acc, off, mult, zr_u - 128, fb, sxr)
        t_total += time.perf_counter() - t0
        ops += 2.0 * 2.0 * sample_rows * ly.n * ly.k
    return ops / t_total / 1e12, orc.get_threads(), t_total


def power_trace(P, synth, torch, dev: str, cfg: int, seconds: float = 5.0):
    """What the device's power management does under the path's kernels: shader clock and socket
    power (amd-smi, sampled from a helper thread as fast as the tool answers) while one phase is
    launched back to back - idle, the fused int8 forward of the workload, its fp32 calibration forward,
    the statistics pass, and the register-resident MFMA probe on operand words of the workload."""
    import subprocess
    import threading
    wl, layers = setup_layers(P, synth, torch, cfg, dev, synth.WORKLOADS[cfg].m)
    run_step(P, layers)
    torch.cuda.synchronize()
    cus = torch.cuda.get_device_properties(dev).multi_processor_count
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    L0 = layers[0]
    words = torch.cat([L0.wq.contiguous().view(-1).view(torch.int32)[:2048].view(-1, 4),
                       L0.xq.contiguous().view(-1).view(torch.int32)[:2048].view(-1, 4)]).contiguous()

    def sample():
        """socket power (W) and the mean shader clock over the XCDs (MHz) from amd-smi."""
        try:
            out = subprocess.run(["amd-smi", "metric", "-g", "0", "--power", "--clock", "--json"],
                                 capture_output=True, text=True, timeout=20).stdout
            doc = json.loads(out[out.index("{"):])
            gpu = (doc.get("gpu_data") or doc)[0] if isinstance(doc.get("gpu_data", doc), list) else doc
            got = {}
            pw = gpu.get("power", {}).get("socket_power", {})
            if isinstance(pw, dict) and isinstance(pw.get("value"), (int, float)):
                got["power_w"] = float(pw["value"])
            clk = [v["clk"]["value"] for k, v in gpu.get("clock", {}).items()
                   if k.startswith("gfx_") and isinstance(v, dict) and isinstance(v.get("clk", {}).get("value"), (int, float))]
            if clk:
                got["sclk_mhz"] = sum(clk) / len(clk)
            return got
        except Exception as exc:  # amd-smi missing or unreadable: report it, do not fail the bench
            return {"error": str(exc)[:80]}

    def phase(name, fn):
        samples, stop = [], threading.Event()

        def watcher():
            while not stop.is_set():
                samples.append(sample())
                stop.wait(0.15)
        th = threading.Thread(target=watcher)
        launches = 0
        t_end = time.perf_counter() + seconds
        th.start()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        while time.perf_counter() < t_end:
            if fn is None:
                time.sleep(0.05)
            else:
                for _ in range(4):
                    fn()
                launches += 4
                torch.cuda.synchronize()
        e1.record()
        torch.cuda.synchronize()
        stop.set()
        th.join()
        ent = {"seconds": round(e0.elapsed_time(e1) / 1e3, 2), "passes": launches, "samples": len(samples)}
        keep = samples[len(samples) // 3:]                      # the settled part
        for key in ("sclk_mhz", "power_w"):
            vals = sorted(v[key] for v in keep if v.get(key) is not None)
            if vals:
                ent[key] = {"min": round(vals[0], 1), "median": round(vals[len(vals) // 2], 1), "max": round(vals[-1], 1)}
        if fn is not None and launches:
            ent["ms_per_pass"] = round(e0.elapsed_time(e1) / launches, 4)
        errs = [v["error"] for v in samples if "error" in v]
        if errs:
            ent["amd_smi_error"] = errs[0]
        return name, ent

    def fwd():
        for L in layers:
            _forward_int8(P, L, L.mult, L.offset, L.fbias)

    def cal():
        for L in layers:
            P.qlinear_cwac_forward(L.xq_cal, L.wq, None, L.deq_mult, L.deq_off,
                                   L.deq_fb if L.bias is not None else None, L.sx_row_cal, P.CWAC_OUT_FP32, L.yq)

    def stats():
        for L in layers:
            P.cwac_calibrate_stats_first(L.y_full, L.yq, L.stats, L.ws)

    def probe():
        P.cwac_mfma_probe(words, 20000, cus, sink)

    # the same forward launches on other operand VALUES (zeros; dense normal codes of standard deviation 30) and
    # on half of the compute units: what the power management makes of each
    gen = torch.Generator(device=dev)
    gen.manual_seed(9)
    k_max, n_max = max(L.k for L in layers), max(L.n for L in layers)
    m = layers[0].m
    xz = torch.zeros(m, k_max, dtype=torch.int8, device=dev)
    wz = torch.zeros(n_max, k_max, dtype=torch.int8, device=dev)
    xd = torch.clamp(torch.round(torch.randn(m, k_max, device=dev, generator=gen) * 30), -128, 127).to(torch.int8)
    wd = torch.clamp(torch.round(torch.randn(n_max, k_max, device=dev, generator=gen) * 30), -127, 127).to(torch.int8)
    half_cus = P.make_tuning(kernel=P.binding.CWAC_KERNEL_DIRECT_LDS, shape=P.binding.CWAC_SHAPE_256_PERSIST,
                             persist_workgroups=cus // 2)

    def fwd_on(x, w, tun=None):
        def run():
            for L in layers:
                xs, ws = (L.xq, L.wq) if x is None else (x[:, :L.k], w[:L.n, :L.k])
                P.qlinear_cwac_forward(xs, ws, L.qp, L.mult, L.offset, L.fbias if L.per_token else None,
                                       L.sx_row if L.per_token else None, P.CWAC_OUT_INT8, L.out, tuning=tun)
        return run

    fwd_ops = sum(2.0 * L.m * L.n * L.k for L in layers)
    fwd_keys = ("forward_int8", "forward_int8_zero_operands", "forward_int8_dense_normal_operands",
                "forward_int8_half_of_the_compute_units", "forward_int8_again")
    out = dict(phase(n, f) for n, f in (("idle", None), ("forward_int8", fwd), ("calibration_forward_fp32", cal),
                                        ("statistics", stats), ("mfma_probe_workload_operands", probe),
                                        ("forward_int8_zero_operands", fwd_on(xz, wz)),
                                        ("forward_int8_dense_normal_operands", fwd_on(xd, wd)),
                                        ("forward_int8_half_of_the_compute_units", fwd_on(None, None, half_cus)),
                                        ("forward_int8_again", fwd)))
    for key in fwd_keys:
        out[key]["pops"] = round(fwd_ops / (out[key]["ms_per_pass"] * 1e-3) / 1e15, 4)
    out["mfma_probe_workload_operands"]["pops"] = round(
        2.0 * 32768 * 16 * 20000 * 4 * cus / (out["mfma_probe_workload_operands"]["ms_per_pass"] * 1e-3) / 1e15, 4)
    return {"power_trace": f"config {cfg}: each phase launched back to back for {seconds} s; amd-smi sampled "
                           "from a helper thread; statistics of the last two thirds of the samples",
            "phases": out}


def tile_timeline(torch, synth, dev: str, cfgs, fp32_out: bool = False):
    """Where a tile's time goes inside the direct-to-LDS forward kernels: 100 MHz time stamps that every
    wavefront takes at five points of each tile (needs the development build of the library,
    `python -m paper_2505_20932_amd.build --timeline`, loaded here instead of the product library).
    One launch per layer after ten warm-up launches; means over all wavefronts of all tiles, us."""
    import ctypes
    import numpy as np
    from paper_2505_20932_amd import build as B
    if not os.path.exists(B.STAMP_LIB):
        raise SystemExit(f"{B.STAMP_LIB} is missing: python -m paper_2505_20932_amd.build --timeline")
    import paper_2505_20932_amd as P
    assert P.binding.LIB_PATH == B.STAMP_LIB, P.binding.LIB_PATH
    lib = P.binding.lib()
    lib.cwac_debug_stamps.restype = ctypes.c_int
    lib.cwac_debug_stamps.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    buf = torch.zeros(4096 * 8 * 5, dtype=torch.int64, device=dev)
    shapes = {"one workgroup per tile (CWAC_SHAPE_256_8W)": P.binding.CWAC_SHAPE_256_8W,
              "persistent workgroups (CWAC_SHAPE_256_PERSIST)": P.binding.CWAC_SHAPE_256_PERSIST}
    out = []
    for cfg in cfgs:
        wl, layers = setup_layers(P, synth, torch, cfg, dev, synth.WORKLOADS[cfg].m)
        layers = layers[:4] if cfg == 3 else layers
        run_step(P, layers)
        torch.cuda.synchronize()
        for L in layers:
            tiles = ((L.m + 255) // 256) * ((L.n + 255) // 256)
            if L.n < 256 or L.k % 128 or L.m < 256 or tiles > 4096:
                continue
            ent = {"workload": cfg, "layer": L.name, "m": L.m, "n": L.n, "k": L.k, "tiles_256x256": tiles,
                   "ideal_mfma_us_per_tile_at_2.4GHz": round(2.0 * 256 * 256 * L.k / (INT8_MFMA_PEAK_TOPS * 1e6 / 256), 2)}
            for name, shape in shapes.items():
                tun = P.make_tuning(kernel=P.binding.CWAC_KERNEL_DIRECT_LDS, shape=shape)

                def fwd():
                    if fp32_out:    # the calibration forward of the step: Y_quant in fp32
                        P.qlinear_cwac_forward(L.xq_cal, L.wq, None, L.deq_mult, L.deq_off,
                                               L.deq_fb if L.bias is not None else None, L.sx_row_cal,
                                               P.CWAC_OUT_FP32, L.yq, tuning=tun)
                    else:
                        P.qlinear_cwac_forward(L.xq, L.wq, L.qp, L.mult, L.offset, L.fbias if L.per_token else None,
                                               L.sx_row, P.CWAC_OUT_INT8, L.out, tuning=tun)
                for _ in range(10):
                    fwd()
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(20):
                    fwd()
                e1.record()
                torch.cuda.synchronize()
                launch_us = e0.elapsed_time(e1) / 20 * 1e3
                buf.zero_()
                fwd()
                torch.cuda.synchronize()
                assert lib.cwac_debug_stamps(buf.data_ptr(), buf.numel() * 8, None) == 0
                torch.cuda.synchronize()
                # work items of the launch: tiles, or, persistent, whole tiles followed by the two
                # 128-token halves of every tile of a thin last round
                items, wgs, n_whole, piece_rows = tiles, tiles, tiles, 256
                if shape == P.binding.CWAC_SHAPE_256_PERSIST:
                    wgs = min(tiles, torch.cuda.get_device_properties(0).multi_processor_count)
                    rest = tiles % wgs
                    # a thin last round is cut into quarters (64 tokens; K below 4096) or halves (128 tokens)
                    pieces = 1 if rest == 0 else (4 if 4 * rest <= wgs and L.k < 4096 else (2 if 2 * rest <= wgs else 1))
                    if pieces > 1:
                        n_whole, items, piece_rows = tiles - rest, tiles + (pieces - 1) * rest, 256 // pieces
                st = buf.cpu().numpy().reshape(4096, 8, 5)[:min(items, 4096)].astype(np.float64) * 0.01       # us
                st -= st[:, :, 0].min()
                whole = st[:n_whole]
                d = [float((whole[:, :, i + 1] - whole[:, :, i]).mean()) for i in range(4)]
                ent[name] = {"back_to_back_launch_us": round(launch_us, 1),
                             "kernel_span_us": round(float(st[:, :, 4].max()), 1), "workgroups": wgs,
                             "start_to_first_mfma_us": round(d[0], 2), "k_loop_us": round(d[1], 2),
                             "epilogue_us": round(d[2], 2), "store_drain_us": round(d[3], 2)}
                if shape == P.binding.CWAC_SHAPE_256_PERSIST:
                    # the rounds of the walk: work items [r * workgroups, (r + 1) * workgroups)
                    rounds = []
                    for r0 in range(0, st.shape[0], wgs):
                        blk = st[r0:r0 + wgs]
                        rounds.append({"items": int(blk.shape[0]), "rows": 256 if r0 < n_whole else piece_rows,
                                       "first_start_us": round(float(blk[:, :, 0].min()), 1),
                                       "mean_start_us": round(float(blk[:, :, 0].mean()), 1),
                                       "mean_end_us": round(float(blk[:, :, 4].mean()), 1),
                                       "last_end_us": round(float(blk[:, :, 4].max()), 1)})
                    ent[name]["rounds"] = rounds
            out.append(ent)
        del layers
        torch.cuda.empty_cache()
    return {"output": "fp32 (calibration forward)" if fp32_out else "int8 (fused CWAC forward)",
            "tile_timeline": "forward, 256 x 256 tiles of eight wavefronts; per tile and wavefront: from its start "
                             "(persistent: from the barrier that ends the previous tile) to the first MFMA, the K loop, "
                             "the epilogue up to its last store instruction, and the wait for the stores",
            "layers": out}


def stage_sweep(torch, synth, dev: str):
    """What sets the K loop's pace: the persistent 256 x 256 tile's time per 128-byte K stage (in-kernel time
    stamps, development build as for tile_timeline) against the operand values (all zero; normal values of
    standard deviation 4 and 30 codes; workload 5's own tensors), the number of compute units at work
    (cwac_tuning.persist_workgroups) and the problem's K and size.  20 back-to-back launches after 30 warm-up
    launches for the launch time, one more launch for the stamps."""
    import ctypes
    import numpy as np
    from paper_2505_20932_amd import build as B
    if not os.path.exists(B.STAMP_LIB):
        raise SystemExit(f"{B.STAMP_LIB} is missing: python -m paper_2505_20932_amd.build --timeline")
    import paper_2505_20932_amd as P
    assert P.binding.LIB_PATH == B.STAMP_LIB, P.binding.LIB_PATH
    lib = P.binding.lib()
    lib.cwac_debug_stamps.restype = ctypes.c_int
    lib.cwac_debug_stamps.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    buf = torch.zeros(4096 * 8 * 5, dtype=torch.int64, device=dev)
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    gen = torch.Generator(device=dev)
    gen.manual_seed(7)

    def operands(kind, m, n, k):
        if kind == "zeros":
            return torch.zeros(m, k, dtype=torch.int8, device=dev), torch.zeros(n, k, dtype=torch.int8, device=dev)
        sd = {"normal, sd 4": 4.0, "normal, sd 30": 30.0}[kind]
        x = torch.clamp(torch.round(torch.randn(m, k, device=dev, generator=gen) * sd), -128, 127).to(torch.int8)
        w = torch.clamp(torch.round(torch.randn(n, k, device=dev, generator=gen) * sd), -127, 127).to(torch.int8)
        return x, w

    def measure(x, w, wgs, label):
        m, k = x.shape
        n = w.shape[0]
        mult = torch.full((n,), 1e-3, dtype=torch.float32, device=dev)
        off = torch.zeros(n, dtype=torch.int32, device=dev)
        out = torch.empty(m, n, dtype=torch.int8, device=dev)
        qp = P.make_qparams(z_r=4)
        tun = P.make_tuning(kernel=P.binding.CWAC_KERNEL_DIRECT_LDS, shape=P.binding.CWAC_SHAPE_256_PERSIST,
                            persist_workgroups=wgs)

        def fwd():
            P.qlinear_cwac_forward(x, w, qp, mult, off, None, None, P.CWAC_OUT_INT8, out, tuning=tun)
        for _ in range(30):
            fwd()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(20):
            fwd()
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / 20 * 1e3
        buf.zero_()
        fwd()
        torch.cuda.synchronize()
        assert lib.cwac_debug_stamps(buf.data_ptr(), buf.numel() * 8, None) == 0
        torch.cuda.synchronize()
        tiles = ((m + 255) // 256) * ((n + 255) // 256)
        g = min(tiles, wgs or cus, cus)
        rest = tiles % g
        n_whole = tiles - rest if (0 < rest and 2 * rest <= g) else tiles
        st = buf.cpu().numpy().reshape(4096, 8, 5)[:min(n_whole, 4096)].astype(np.float64) * 0.01
        d = [float((st[:, :, i + 1] - st[:, :, i]).mean()) for i in range(3)]
        stages = k // 128
        return {"case": label, "m": m, "n": n, "k": k, "workgroups": g, "launch_us": round(us, 1),
                "tops": round(2.0 * m * n * k / us / 1e6, 1),
                "tops_per_workgroup": round(2.0 * m * n * k / us / 1e6 / g, 2),
                "start_to_first_mfma_us": round(d[0], 2), "k_loop_us": round(d[1], 2),
                "us_per_stage": round(d[1] / stages, 3),
                "stage_rate_of_peak": round(2.0 * 256 * 256 * 128 / (d[1] / stages) / (INT8_MFMA_PEAK_TOPS * 1e6 / 256), 3),
                "epilogue_us": round(d[2], 2)}

    rows = []
    # operand values, one shape (workload 5's o projection), every compute unit
    wl, layers = setup_layers(P, synth, torch, 5, dev, synth.WORKLOADS[5].m)
    L = [l for l in layers if l.name == "o"][0]
    xw, ww = L.xq.clone(), L.wq.clone()
    del layers, L
    torch.cuda.empty_cache()
    m, n, k = xw.shape[0], ww.shape[0], xw.shape[1]
    for kind in ("zeros", "normal, sd 4", "normal, sd 30"):
        x, w = operands(kind, m, n, k)
        rows.append(measure(x, w, 0, f"operands {kind}"))
        del x, w
    rows.append(measure(xw, ww, 0, "operands of workload 5 (o projection)"))
    # compute units at work, same tensors
    for wgs in (32, 64, 128, 192):
        rows.append(measure(xw, ww, wgs, f"workload 5 operands, {wgs} workgroups"))
    x0, w0 = operands("zeros", m, n, k)
    for wgs in (32, 128):
        rows.append(measure(x0, w0, wgs, f"operands zeros, {wgs} workgroups"))
    del x0, w0
    # K and problem size, same distribution of values
    for (mm, nn, kk) in ((16384, 4096, 768), (4096, 4096, 768), (4096, 4096, 4096), (25216, 768, 3072)):
        x, w = operands("normal, sd 4", mm, nn, kk)
        rows.append(measure(x, w, 0, "operands normal, sd 4"))
        del x, w
    return {"stage_sweep": "persistent 256 x 256 int8 tile: time per 128-byte K stage (ideal at the published peak: "
                           f"{2.0 * 256 * 256 * 128 / (INT8_MFMA_PEAK_TOPS * 1e6 / 256):.3f} us) against operand values, "
                           "compute units at work, K and problem size", "rows": rows}


def forward_shapes(P, synth, torch, dev: str, cfgs, reps: int = 20):
    """Every tile shape of the direct-to-LDS forward that a layer admits, chosen through cwac_tuning, timed
    on each distinct layer shape of the workloads (int8 output, the layer's own folded epilogue): `reps`
    back-to-back launches after 5 warm-up launches, HIP events.  `auto` is the dispatcher's own choice."""
    B = P.binding
    shapes = [("auto", None, 0), ("256_8W", B.CWAC_SHAPE_256_8W, 0), ("256_4W_K128", B.CWAC_SHAPE_256_4W_K128, 0),
              ("256_4W_K64", B.CWAC_SHAPE_256_4W_K64, 0), ("128_PAIR", B.CWAC_SHAPE_128_PAIR, 0),
              ("128_128", B.CWAC_SHAPE_128_128, 0), ("256_PERSIST", B.CWAC_SHAPE_256_PERSIST, 0),
              # the persistent tile with the panel loads issued by four / by all eight of its wavefronts
              ("256_PERSIST, 4 loading wavefronts", B.CWAC_SHAPE_256_PERSIST, 4),
              ("256_PERSIST, 8 loading wavefronts", B.CWAC_SHAPE_256_PERSIST, 8)]
    out = []
    for cfg in cfgs:
        wl, layers = setup_layers(P, synth, torch, cfg, dev, synth.WORKLOADS[cfg].m)
        run_step(P, layers)
        torch.cuda.synchronize()
        seen = set()
        for L in layers:
            if (L.n, L.k) in seen:
                continue
            seen.add((L.n, L.k))
            ent = {"workload": cfg, "layer": L.name, "m": L.m, "n": L.n, "k": L.k, "us": {}}
            for name, shape, loaders in shapes:
                tun = None if shape is None else P.make_tuning(kernel=B.CWAC_KERNEL_DIRECT_LDS, shape=shape,
                                                               persist_loaders=loaders)

                def fwd():
                    P.qlinear_cwac_forward(L.xq, L.wq, L.qp, L.mult, L.offset, L.fbias if L.per_token else None,
                                           L.sx_row, P.CWAC_OUT_INT8, L.out, tuning=tun)
                try:
                    for _ in range(5):
                        fwd()
                except Exception:   # the shape does not admit this layer (status code from the library)
                    ent["us"][name] = None
                    continue
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                torch.cuda.synchronize()
                e0.record()
                for _ in range(reps):
                    fwd()
                e1.record()
                torch.cuda.synchronize()
                ent["us"][name] = round(e0.elapsed_time(e1) / reps * 1e3, 1)
            # four against eight loading wavefronts once more, alternated (five rounds of `reps` launches each,
            # the median per side), so that clock and power drift over the sweep falls on both alike
            sides = {4: [], 8: []}
            for _ in range(5):
                for loaders in (4, 8):
                    tun = P.make_tuning(kernel=B.CWAC_KERNEL_DIRECT_LDS, shape=B.CWAC_SHAPE_256_PERSIST,
                                        persist_loaders=loaders)
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                    for _ in range(reps):
                        P.qlinear_cwac_forward(L.xq, L.wq, L.qp, L.mult, L.offset, L.fbias if L.per_token else None,
                                               L.sx_row, P.CWAC_OUT_INT8, L.out, tuning=tun)
                    e1.record()
                    torch.cuda.synchronize()
                    sides[loaders].append(e0.elapsed_time(e1) / reps * 1e3)
            med = {k: sorted(v)[2] for k, v in sides.items()}
            ent["loading_wavefronts_alternated_us"] = {"4": round(med[4], 1), "8": round(med[8], 1),
                                                       "4_over_8": round(med[4] / med[8], 4)}
            # the vendor library's int8 GEMM on the same operands: the raw int32 product, no epilogue
            try:
                wt = L.wq.t()
                for _ in range(5):
                    torch._int_mm(L.xq, wt)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                torch.cuda.synchronize()
                e0.record()
                for _ in range(reps):
                    torch._int_mm(L.xq, wt)
                e1.record()
                torch.cuda.synchronize()
                ent["us"]["torch._int_mm (int32 product only)"] = round(e0.elapsed_time(e1) / reps * 1e3, 1)
            except Exception as exc:
                ent["us"]["torch._int_mm (int32 product only)"] = f"unavailable: {type(exc).__name__}"
            ent["tops"] = {k: (round(2.0 * L.m * L.n * L.k / v / 1e6, 1) if isinstance(v, float) else None)
                           for k, v in ent["us"].items()}
            out.append(ent)
        del layers
        torch.cuda.empty_cache()
    return {"forward_shapes": "int8 forward per layer shape and tile shape (cwac_tuning.shape), microseconds per launch, "
                              f"{reps} back-to-back launches", "layers": out}


def small_batch_sweep(P, synth, torch, dev: str):
    """The weight-only layer at decode-sized batches (its own JSON line): every distinct layer shape of
    workload 5 at 1, 8, 16 and 32 tokens, the dispatcher's choice and every (wavefronts, ring depth) of the
    weight-streaming kernel; enough copies of the packed weights cycle that each launch reads them from HBM
    (more than 400 MB per shape); three passes over the copies replayed from a HIP graph."""
    layers = setup_weight_only(P, synth, torch, 5, dev)
    for L in layers:
        del L.y_full, L.xcal, L.wh
    torch.cuda.empty_cache()
    out = []
    seen = set()
    for L in layers:
        if (L.n, L.k) in seen:
            continue
        seen.add((L.n, L.k))
        wbytes = L.n * L.k // 2 + L.n * (L.k // 128) * 4
        copies = max(2, (400 << 20) // wbytes)
        pws = [L.pw.clone() for _ in range(copies)]
        pszs = [L.psz.clone() for _ in range(copies)]
        ent = {"n": L.n, "k": L.k, "weight_bytes": wbytes, "copies": copies, "us": {}}
        for sm in (1, 8, 16, 32, 64, 128, 256, 512):
            o = torch.empty(sm, L.n, dtype=torch.float16, device=dev)
            row = {}
            # up to 32 rows: every (wavefronts, ring depth) of the weight-streaming kernel; above: the dispatcher's
            # choice (passes of that kernel up to 128 rows, 128-token tiles while they fit one round) against the
            # tiled kernel with 128- and 256-token tiles
            choices = (((0, 0, 0), (4, 2, 0), (4, 3, 0), (4, 4, 0), (8, 2, 0), (8, 3, 0), (8, 4, 0)) if sm <= 32 else
                       ((0, 0, 0), (0, 0, 128), (0, 0, 256)))
            for waves, depth, tile in choices:
                tun = (P.make_tuning(w4_small_waves=waves, w4_small_depth=depth, w4_tile=tile)
                       if (waves or tile) else None)

                def one_pass():
                    for pw, psz in zip(pws, pszs):
                        P.qlinear_w4a16_cwac_forward(L.x[:sm], pw, psz, L.n, L.mult, L.fbias, o, tuning=tun)
                one_pass()
                torch.cuda.synchronize()
                side = torch.cuda.Stream()
                with torch.cuda.stream(side):
                    g = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(g, stream=side):
                        for _ in range(3):
                            one_pass()
                g.replay()
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                g.replay()
                e1.record()
                torch.cuda.synchronize()
                name = "auto" if not (waves or tile) else (f"tile{tile}" if tile else f"{waves}w_d{depth}")
                row[name] = round(e0.elapsed_time(e1) / (3 * copies) * 1e3, 2)
                del g
            row["auto_gbs"] = round(wbytes / row["auto"] / 1e3, 1)
            ent["us"][f"m={sm}"] = row
        out.append(ent)
        del pws, pszs
        torch.cuda.empty_cache()
    # one wide matrix (a vocabulary-sized head), random codes: what the stream sustains once the
    # fixed cost of a launch is small beside its bytes
    n, k, sm = 131072, 4096, 8
    pws = [torch.randint(0, 255, (n * k // 2,), dtype=torch.uint8, device=dev) for _ in range(2)]
    sc = torch.full((k // 128, n), 0.01, dtype=torch.float16, device=dev)
    psz = (sc.view(torch.int16).to(torch.int32) & 0xffff) | (8 << 16)
    x = torch.randn(sm, k, dtype=torch.float16, device=dev)
    o = torch.empty(sm, n, dtype=torch.float16, device=dev)
    for pw in pws:
        P.qlinear_w4a16_cwac_forward(x, pw, psz.view(-1), n, None, None, o)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(5):
        for pw in pws:
            P.qlinear_w4a16_cwac_forward(x, pw, psz.view(-1), n, None, None, o)
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) / 10 * 1e3
    wbytes = n * k // 2 + n * (k // 128) * 4
    out.append({"n": n, "k": k, "weight_bytes": wbytes, "copies": 2,
                "us": {f"m={sm}": {"auto": round(us, 1), "auto_gbs": round(wbytes / us / 1e3, 1)}}})
    return {"small_batch_sweep": "w4a16_small_m_kernel, microseconds per launch from a HIP graph, weights from HBM; "
                                 "columns: the dispatcher's choice, then <wavefronts per workgroup>w_d<ring depth> (up to 32 tokens) or "
                                 "the tiled kernel with tile<tokens per tile> (above)",
            "layers": out}


def time_steps(P, torch, layers, steps: int, warmup: int):
    """warmup untimed passes of run_step, then `steps` timed ones (host clock around the whole
    region, HIP events on the launch stream around every phase of every layer)."""
    for _ in range(warmup):
        run_step(P, layers)
    torch.cuda.synchronize()
    events = []
    t0 = time.perf_counter()
    for _ in range(steps):
        run_step(P, layers, events)
    torch.cuda.synchronize()
    return time.perf_counter() - t0, events


def forward_floors_us(m: int, n: int, k: int):
    """Lower bounds of one int8 forward launch: its operations at the published int8 MFMA peak and
    its compulsory bytes (activations, weights and int8 codes, each once) at the published HBM peak."""
    return 2.0 * m * n * k / INT8_MFMA_PEAK_TOPS / 1e6, (m * k + n * k + m * n) / HBM_PEAK_GBS / 1e3


def summarize(layers, events, steps: int, elapsed: float):
    """Phase totals (ms per step) and the per-layer table of one timed run."""
    nl = len(layers)
    ph = [sum(e[i].elapsed_time(e[i + 1]) for e in events) / steps for i in range(4)]
    t_cal, t_stats, t_fit, t_fwd = ph
    fwd_ops = sum(2.0 * L.m * L.n * L.k for L in layers)
    cal_ops = sum(2.0 * L.cal_rows * L.n * L.k for L in layers)
    stats_bytes = sum(8.0 * L.cal_rows * L.n for L in layers)
    per_layer = []
    for i, L in enumerate(layers):
        ev = [events[s * nl + i] for s in range(steps)]
        us = [sum(e[j].elapsed_time(e[j + 1]) for e in ev) / steps * 1e3 for j in range(4)]
        ops = 2.0 * L.m * L.n * L.k
        mfma_floor, hbm_floor = forward_floors_us(L.m, L.n, L.k)
        per_layer.append({
            "layer": L.name, "m": L.m, "n": L.n, "k": L.k, "calibration_rows": L.cal_rows,
            "forward_int8_us": round(us[3], 1), "forward_int8_tops": round(ops / us[3] / 1e6, 1),
            "forward_int8_frac": round(ops / us[3] / 1e6 / INT8_MFMA_PEAK_TOPS, 4),
            # what the two published peaks allow: the layer's operations at the int8 MFMA peak, its
            # compulsory bytes (X, W_q, int8 output, once each) at the HBM peak; a layer cannot
            # pass mfma_floor / max(mfma_floor, hbm_floor) of the MFMA peak
            "forward_int8_mfma_floor_us": round(mfma_floor, 2), "forward_int8_hbm_floor_us": round(hbm_floor, 2),
            "forward_int8_frac_ceiling": round(mfma_floor / max(mfma_floor, hbm_floor), 4),
            "calibration_forward_us": round(us[0], 1),
            "calibration_forward_tops": round(2.0 * L.cal_rows * L.n * L.k / us[0] / 1e6, 1),
            "statistics_us": round(us[1], 1),
            "statistics_gbs": round(8.0 * L.cal_rows * L.n / us[1] / 1e3, 1),
            "statistics_frac": round(8.0 * L.cal_rows * L.n / us[1] / 1e3 / HBM_PEAK_GBS, 4),
            "solve_fold_us": round(us[2], 1)})
    return {"ms_per_step": elapsed / steps * 1e3, "t_cal": t_cal, "t_stats": t_stats, "t_fit": t_fit,
            "t_fwd": t_fwd, "fwd_ops": fwd_ops, "cal_ops": cal_ops, "stats_bytes": stats_bytes,
            "fwd_tops": fwd_ops / (t_fwd * 1e-3) / 1e12, "stats_gbs": stats_bytes / (t_stats * 1e-3) / 1e9,
            "per_layer": per_layer}


def per_config_entry(wl, layers, sm, collapse=None):
    """One workload's entry of the per_config block.  collapse: (group size, groups) when the
    workload repeats a group of layer shapes (the 12 blocks of workload 3): the table then shows the
    mean over the repeats of each layer of the group."""
    table = sm["per_layer"]
    if collapse:
        g, reps = collapse
        merged = []
        for j in range(g):
            rows = [table[r * g + j] for r in range(reps)]
            ent = dict(rows[0])
            ent["layer"] = ent["layer"].split(".")[-1] + f" (mean of {reps} blocks)"
            for key in ent:
                if key.endswith("_us"):
                    ent[key] = round(sum(r[key] for r in rows) / reps, 1)
            ops = 2.0 * ent["m"] * ent["n"] * ent["k"]
            ent["forward_int8_tops"] = round(ops / ent["forward_int8_us"] / 1e6, 1)
            ent["forward_int8_frac"] = round(ent["forward_int8_tops"] / INT8_MFMA_PEAK_TOPS, 4)
            ent["calibration_forward_tops"] = round(2.0 * ent["calibration_rows"] * ent["n"] * ent["k"]
                                                    / ent["calibration_forward_us"] / 1e6, 1)
            ent["statistics_gbs"] = round(8.0 * ent["calibration_rows"] * ent["n"] / ent["statistics_us"] / 1e3, 1)
            ent["statistics_frac"] = round(ent["statistics_gbs"] / HBM_PEAK_GBS, 4)
            merged.append(ent)
        table = merged
    return {
        "workload": f"{wl.name}: {len(layers)} linear layers, M={wl.m} tokens, "
                    f"{layers[0].cal_rows} calibration rows per layer and step, "
                    + ("per-token" if wl.per_token else "per-tensor") + " activations",
        "ms_per_step": round(sm["ms_per_step"], 4),
        "forward_int8": {"tops": round(sm["fwd_tops"], 1), "frac": round(sm["fwd_tops"] / INT8_MFMA_PEAK_TOPS, 4),
                         "ms": round(sm["t_fwd"], 4), "bound": "mfma", "peak_tops": INT8_MFMA_PEAK_TOPS,
                         # sum of MFMA floors over sum of max(MFMA floor, HBM floor): the fraction of the
                         # MFMA peak that the two published peaks leave to this mix of layer shapes
                         "frac_ceiling": round(sum(forward_floors_us(L.m, L.n, L.k)[0] for L in layers)
                                               / sum(max(forward_floors_us(L.m, L.n, L.k)) for L in layers), 4)},
        "statistics": {"gbs": round(sm["stats_gbs"], 1), "frac": round(sm["stats_gbs"] / HBM_PEAK_GBS, 4),
                       "ms": round(sm["t_stats"], 4), "bound": "hbm", "peak_gbs": HBM_PEAK_GBS,
                       "launches": "cwac_calibrate_stats_first: stats_partial_kernel + stats_merge_kernel"},
        "calibration_forward_fp32_tops": round(sm["cal_ops"] / (sm["t_cal"] * 1e-3) / 1e12, 1),
        "solve_fold_ms": round(sm["t_fit"], 4),
        **({"note": "every launch of this workload is shorter than 30 us (a kernel that does nothing is recorded "
                    "at 4-5 us on this device): launch-bound, the fractions say nothing about the kernels"}
           if max(sm["t_fwd"], sm["t_stats"]) / len(layers) < 0.03 else {}),
        "layers": table}


def per_config_block(P, synth, torch, dev: str, steps: int, headline_cfg: int, headline_entry):
    """Every workload through the same step as the headline: workloads 1-4 with their WHOLE calibration
    set per layer and step (it fits the device many times over), workload 5 in chunks of its token
    count (the headline run itself)."""
    out = {}
    for cfg in (1, 2, 3, 4, 5):
        if cfg == headline_cfg and headline_entry is not None:
            out[str(cfg)] = headline_entry
            continue
        wl = synth.WORKLOADS[cfg]
        cal_rows = wl.cal_rows if cfg != 5 else wl.m
        wl, layers = setup_layers(P, synth, torch, cfg, dev, cal_rows)
        elapsed, events = time_steps(P, torch, layers, steps, 2)
        sm = summarize(layers, events, steps, elapsed)
        out[str(cfg)] = per_config_entry(wl, layers, sm, (4, 12) if cfg == 3 else None)
        # the calibration side as one fused call (statistics in the calibration GEMM's epilogue) on this workload
        fc = fused_calibration(P, torch, layers, 2, reps=3)
        if fc is not None:
            out[str(cfg)]["fused_calibration"] = fc
        del layers, events
        torch.cuda.empty_cache()
    return out


def full_calibration_stream(P, synth, torch, cfg: int, dev: str, chunk: int):
    """The workload's COMPLETE calibration set streamed into one state per layer: Y_full of all rows
    resident (upstream, torch fp32 matmul), then per chunk of `chunk` rows the fp32 calibration forward
    and one statistics call (the first reset-free), then the fit.  Timed: the whole stream per layer,
    and the statistics calls alone (HIP events on the launch stream)."""
    wl = synth.WORKLOADS[cfg]
    rows = wl.cal_rows
    n_chunks = (rows + chunk - 1) // chunk
    f32 = dict(dtype=torch.float32, device=dev)
    res_layers, tot_bytes, tot_stats_ms, tot_ms = [], 0.0, 0.0, 0.0
    yq = torch.empty(chunk * max(ly.n for ly in wl.layers), **f32)
    for li, ly in enumerate(wl.layers):
        w, b = synth.weights(wl, li, device=dev)
        wq = torch.empty(ly.n, ly.k, dtype=torch.int8, device=dev)
        sw = torch.empty(ly.n, **f32)
        P.cwac_quantize_rows_sym(w, sw, wq)
        colsum = torch.empty(ly.n, dtype=torch.int32, device=dev)
        P.cwac_colsum(wq, colsum)
        xq = torch.empty(rows, ly.k, dtype=torch.int8, device=dev)
        y_full = torch.empty(rows, ly.n, **f32)
        sx_row = torch.empty(rows, **f32) if wl.per_token else None
        sx, zx = 1.0, 0
        if not wl.per_token:
            x0 = synth.activations(wl, li, min(rows, chunk), calibration=True, device=dev)
            mm = torch.empty(2, **f32)
            ws = torch.empty(P.cwac_range_workspace(x0.numel()), dtype=torch.uint8, device=dev)
            P.cwac_range_f32(x0, mm, ws)
            mn, mx = (float(v) for v in mm.cpu())
            sx, z_u = P.cwac_qparams_from_range(mn, mx, 8)
            zx = z_u - 128
        for c0 in range(0, rows, chunk):                      # set-up, chunk by chunk (fp32 X is transient)
            c1 = min(rows, c0 + chunk)
            x = synth.activations(wl, li, c1 - c0, calibration=True, device=dev, row0=c0)
            if wl.per_token:
                P.cwac_quantize_rows_sym(x, sx_row[c0:c1], xq[c0:c1])
            else:
                P.cwac_quantize_act(x, sx, zx, xq[c0:c1])
            torch.matmul(x, w.t(), out=y_full[c0:c1])
            if b is not None:
                y_full[c0:c1] += b
            del x
        dm, dfb = torch.empty(ly.n, **f32), torch.empty(ly.n, **f32)
        do = torch.empty(ly.n, dtype=torch.int32, device=dev)
        P.cwac_fold(None, None, sw, b, colsum, P.make_qparams(P.CWAC_EPI_FP_BIAS, wl.per_token, sx, zx, 1.0, 0),
                    dm, do, dfb)
        stats = torch.empty(P.cwac_stats_bytes(ly.n) // 8 + 2, dtype=torch.float64, device=dev)
        wsp = torch.empty(P.cwac_calibrate_stats_workspace(chunk, ly.n), dtype=torch.uint8, device=dev)
        alpha, beta = torch.empty(ly.n, **f32), torch.empty(ly.n, **f32)
        yqv = yq[:chunk * ly.n].view(chunk, ly.n)

        def stream(ev=None):
            for ci, c0 in enumerate(range(0, rows, chunk)):
                c1 = min(rows, c0 + chunk)
                P.qlinear_cwac_forward(xq[c0:c1], wq, None, dm, do, dfb if b is not None else None,
                                       None if sx_row is None else sx_row[c0:c1], P.CWAC_OUT_FP32, yqv[:c1 - c0])
                if ev is not None:
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                P.cwac_calibrate_stats(y_full[c0:c1], yqv[:c1 - c0], stats, wsp, first=(ci == 0))
                if ev is not None:
                    e1.record()
                    ev.append((e0, e1))
            P.cwac_solve(stats, ly.n, alpha, beta)

        stream()
        torch.cuda.synchronize()
        ev = []
        a, z = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        stream(ev)
        z.record()
        torch.cuda.synchronize()
        ms_all = a.elapsed_time(z)
        ms_stats = sum(e0.elapsed_time(e1) for e0, e1 in ev)
        n_seen = int(stats.view(torch.int64)[0].item())
        assert n_seen == rows, (n_seen, rows)
        nbytes = 8.0 * rows * ly.n
        res_layers.append({"layer": ly.name, "n": ly.n, "rows": rows, "chunks": n_chunks,
                           "statistics_ms": round(ms_stats, 3),
                           "statistics_gbs": round(nbytes / ms_stats / 1e6, 1),
                           "statistics_frac": round(nbytes / ms_stats / 1e6 / HBM_PEAK_GBS, 4),
                           "stream_ms_with_calibration_forward": round(ms_all, 3)})
        tot_bytes += nbytes
        tot_stats_ms += ms_stats
        tot_ms += ms_all
        del w, wq, xq, y_full, stats, wsp
        torch.cuda.empty_cache()
    gbs = tot_bytes / tot_stats_ms / 1e6
    return {"workload": f"config {cfg}: all {rows} calibration rows of every layer into one state, "
                        f"{n_chunks} chunks of {chunk} rows",
            "statistics_gbs": round(gbs, 1), "statistics_frac": round(gbs / HBM_PEAK_GBS, 4),
            "statistics_bytes": tot_bytes, "statistics_ms": round(tot_stats_ms, 3),
            "stream_ms_with_calibration_forward": round(tot_ms, 3), "layers": res_layers}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=5, help="workload 1..5 (default: the LLM layer)")
    ap.add_argument("--cal-rows", type=int, default=0, help="calibration rows per step (default: "
                    "one batch = the workload's token count)")
    ap.add_argument("--cpu-sample-rows", type=int, default=1536)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-weight-only", action="store_true",
                    help="skip the INT4 weight-only section (reported for the LLM workload only)")
    ap.add_argument("--conv", action="store_true",
                    help="the convolutional-layer section instead: ResNet-50 bottleneck convolutions "
                         "(its own JSON line)")
    ap.add_argument("--conv-batch", type=int, default=128)
    ap.add_argument("--block", action="store_true",
                    help="the Transformer-block section instead: one ViT-B/16 block, linear layers chained "
                         "with the non-linear glue (its own JSON line)")
    ap.add_argument("--block-batch", type=int, default=128)
    ap.add_argument("--blocks", type=int, default=12, help="depth of the stack timed beside the single block")
    ap.add_argument("--block-shape", type=str, default="197,12,64,3072",
                    help="tokens,heads,head width (64 or 32),MLP width of the block (default: ViT-B/16); e.g. "
                         "49,16,32,2048 with --block-batch 512 is Swin-B's third stage at 8 images")
    ap.add_argument("--no-per-config", action="store_true",
                    help="skip the per_config block (workloads 1-5, each through the same step)")
    ap.add_argument("--step-only", action="store_true",
                    help="only the warm-up and timed steps (no graph replay, comparators, probe, CPU baseline, "
                         "per-config, streaming or weight-only sections): the launch mix of a profiler run then is "
                         "the timed region's own")
    ap.add_argument("--no-full-stream", action="store_true",
                    help="skip the leg that streams workload 5's whole calibration set (262144 rows per layer)")
    ap.add_argument("--per-config-steps", type=int, default=5)
    ap.add_argument("--power-trace", action="store_true",
                    help="instead of the benchmark: shader clock and socket power (amd-smi) under each of the "
                         "path's kernels launched back to back (its own JSON line)")
    ap.add_argument("--tile-timeline", action="store_true",
                    help="instead of the benchmark: in-kernel time stamps of the int8 forward's tiles on workloads "
                         "2-5 (needs `python -m paper_2505_20932_amd.build --timeline`; its own JSON line)")
    ap.add_argument("--stage-sweep", action="store_true",
                    help="instead of the benchmark: the persistent tile's time per K stage against operand values, "
                         "compute units at work, K and problem size (needs the --timeline build; its own JSON line)")
    ap.add_argument("--timeline-fp32", action="store_true",
                    help="with --tile-timeline: the fp32-output calibration forward instead of the int8 forward")
    ap.add_argument("--forward-shapes", action="store_true",
                    help="instead of the benchmark: the int8 forward of every distinct layer shape of workloads 2-5 "
                         "under each tile shape of the direct-to-LDS kernel (its own JSON line)")
    ap.add_argument("--small-batch", action="store_true",
                    help="instead of the benchmark: the weight-only layer at 1-32 tokens on workload 5's layer shapes, "
                         "every wavefront count and ring depth of its weight-streaming kernel (its own JSON line)")
    ap.add_argument("--probe", action="store_true",
                    help="profiling aid: one plain 1 GiB device copy (a kernel of known traffic, to "
                         "calibrate rocprofv3 byte counters) followed by ONE step, then exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives or sharding are part of "
              "it); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    if args.tile_timeline or args.stage_sweep:
        # the package reads the library path when it is first imported
        os.environ["CWAC_LIB"] = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_2505_20932_amd",
                                              "libcwac_hip_timeline.so")
        from paper_2505_20932_amd import synth
        assert torch.cuda.is_available(), "bench.py needs the MI355X"
        torch.cuda.set_device(0)
        if args.stage_sweep:
            print(json.dumps(stage_sweep(torch, synth, "cuda:0")))
        else:
            print(json.dumps(tile_timeline(torch, synth, "cuda:0", (2, 3, 4, 5), args.timeline_fp32)))
        return
    import paper_2505_20932_amd as P
    from paper_2505_20932_amd import synth
    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    P.binding.lib()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.conv:
        print(json.dumps(conv_section(P, synth, torch, dev, args.conv_batch, args.steps,
                                      0 if args.no_cpu_baseline else 8)))
        return
    if args.block:
        print(json.dumps(block_section(P, torch, dev, args.block_batch, args.steps, args.warmup,
                                       0 if args.no_cpu_baseline else 2, args.blocks,
                                       tuple(int(v) for v in args.block_shape.split(",")))))
        return
    if args.forward_shapes:
        print(json.dumps(forward_shapes(P, synth, torch, dev, (2, 3, 4, 5))))
        return
    if args.small_batch:
        print(json.dumps(small_batch_sweep(P, synth, torch, dev)))
        return
    if args.power_trace:
        print(json.dumps(power_trace(P, synth, torch, dev, args.config)))
        return
    wl = synth.WORKLOADS[args.config]
    cal_rows = args.cal_rows or wl.m
    wl, layers = setup_layers(P, synth, torch, args.config, dev, cal_rows)

    if args.probe:
        # plain copy kernel of known traffic: out = 1 * y + 0 over 2^28 floats (reads 1 GiB, writes 1 GiB)
        src = torch.empty(1 << 14, 1 << 14, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        one = torch.ones(1 << 14, dtype=torch.float32, device=dev)
        zero = torch.zeros(1 << 14, dtype=torch.float32, device=dev)
        torch.cuda.synchronize()
        P.cwac_apply_unfolded(src, one, zero, dst)
        run_step(P, layers)
        torch.cuda.synchronize()
        if args.config == 5 and not args.no_weight_only:
            del layers, src, dst
            torch.cuda.empty_cache()
            run_step_weight_only(P, setup_weight_only(P, synth, torch, args.config, dev))
            torch.cuda.synchronize()
        print(json.dumps({"probe": "copy of 1073741824 bytes, then one step (and one weight-only step)",
                          "workload": wl.name}))
        return

    elapsed, events = time_steps(P, torch, layers, args.steps, args.warmup)
    sm = summarize(layers, events, args.steps, elapsed)
    gemm_ops = sm["fwd_ops"] + sm["cal_ops"]                                   # both GEMMs of a step
    fwd_ops, fwd_tops, stats_gbs = sm["fwd_ops"], sm["fwd_tops"], sm["stats_gbs"]
    t_cal, t_stats, t_fit, t_fwd = sm["t_cal"], sm["t_stats"], sm["t_fit"], sm["t_fwd"]
    ms_step = sm["ms_per_step"]
    nl = len(layers)
    default_run = cal_rows == wl.m
    # the kernel the dispatcher takes for most of the int8 forward's launches
    direct = all(P.binding.cwac_forward_kernel_for(L.m, L.n, L.k, L.k, L.k, P.CWAC_OUT_INT8)
                 == P.binding.CWAC_KERNEL_DIRECT_LDS
                 for L in layers)
    fwd_kernel = ("qlinear_persist_kernel<CWAC_OUT_INT8, ...> (persistent 256 x 256 tile, eight wavefronts, one "
                  "workgroup per compute unit, direct-to-LDS panels; int8 out, fused CWAC epilogue)"
                  if direct and all(L.k % 128 == 0 for L in layers) else
                  "qlinear_persist_kernel / qlinear_fast_kernel / qlinear_kernel as the dispatcher picks per layer "
                  "(int8 out, fused CWAC epilogue)")
    result = {
        # the metric's named quantity: int8 operations of the fused forward over its own time inside
        # the step (HIP events); the whole step's blended rate is whole_step_tops
        "metric": METRIC, "value": round(fwd_tops, 2),
        "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": f"config {wl.cfg}: {wl.name}, {nl} linear layers, M={wl.m} tokens, "
                               f"{cal_rows} calibration rows per step, "
                               + ("per-token" if wl.per_token else "per-tensor") + " activations",
                   "layers": [f"{L.name} {L.n}x{L.k}" for L in layers]},
        "roofline": {"bound": "mfma", "achieved": round(fwd_tops / 1e3, 4),
                     "peak": INT8_MFMA_PEAK_TOPS / 1e3, "unit": "POP/s",
                     "frac": round(fwd_tops / INT8_MFMA_PEAK_TOPS, 4),
                     "traffic": PMC_TRAFFIC_BYTES.get(wl.cfg, {}).get("forward_int8") if default_run else None,
                     "traffic_source": PMC_TRAFFIC_SOURCE.get(wl.cfg) if default_run else None,
                     "kernel": fwd_kernel,
                     "launches_per_step": nl, "avg_launch_ms": round(t_fwd / nl, 4),
                     "ops_per_step": fwd_ops},
        "roofline_stats": {"bound": "hbm", "achieved": round(stats_gbs, 1), "peak": HBM_PEAK_GBS,
                           "unit": "GB/s", "frac": round(stats_gbs / HBM_PEAK_GBS, 4),
                           "traffic": PMC_TRAFFIC_BYTES.get(wl.cfg, {}).get("statistics") if default_run else None,
                           "traffic_source": PMC_TRAFFIC_SOURCE.get(wl.cfg) if default_run else None,
                           "kernel": "stats_partial_kernel<4> + stats_merge_kernel (cwac_calibrate_stats_first: "
                                     "two launches per layer, no reset)",
                           "avg_launch_ms": round(t_stats / nl, 4), "bytes_per_step": sm["stats_bytes"]},
        "phases_ms": {"calibration_forward_fp32": round(t_cal, 4), "statistics": round(t_stats, 4),
                      "solve_fold": round(t_fit, 4), "forward_int8": round(t_fwd, 4)},
        "forward_int8_tops": round(fwd_tops, 2),
        "whole_step_tops": round(gemm_ops / (elapsed / args.steps) / 1e12, 2),
        "calibration_forward_tops": round(sm["cal_ops"] / (t_cal * 1e-3) / 1e12, 2),
        "stats_gbs": round(stats_gbs, 1),
    }
    headline_entry = per_config_entry(wl, layers, sm, (4, 12) if wl.cfg == 3 else None) if default_run else None
    if args.step_only:
        result["layers"] = sm["per_layer"]
        print(json.dumps(result))
        return
    # the same step captured once in a HIP graph and replayed (what a launch-bound caller would do)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        run_step(P, layers)
    g.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        g.replay()
    torch.cuda.synchronize()
    t_graph = (time.perf_counter() - t0) / args.steps
    result["graph_replay"] = {"ms_per_step": round(t_graph * 1e3, 4),
                              "whole_step_tops": round(gemm_ops / t_graph / 1e12, 2)}
    result["epilogue_comparators"] = comparators(P, torch, layers)
    result["fused_calibration"] = fused_calibration(P, torch, layers, args.steps)
    result["mfma_ceiling_probe"] = mfma_ceiling(P, torch, layers)
    result["hbm_read_stream_probe"] = hbm_read_ceiling(P, torch, layers)
    if not args.no_cpu_baseline:
        v, cores, secs = cpu_baseline(synth, args.config, args.cpu_sample_rows)
        result["cpu_baseline"] = {
            "value": round(v, 5), "unit": "TOPS", "cores": cores, "kind": "oracle",
            "sample": f"the same step on {args.cpu_sample_rows} inference rows and "
                      f"{args.cpu_sample_rows} calibration rows of every layer "
                      f"({secs:.1f} s of oracle time)"}
    del layers, events
    torch.cuda.empty_cache()
    if not args.no_per_config:
        result["per_config"] = per_config_block(P, synth, torch, dev, args.per_config_steps, args.config,
                                                headline_entry)
    if args.config == 5 and not args.no_full_stream:
        result["full_calibration_stream"] = full_calibration_stream(P, synth, torch, 5, dev, wl.m)
    if args.config == 5 and not args.no_weight_only:
        result["weight_only_int4"] = weight_only_int4(
            P, synth, torch, args.config, dev, args.steps,
            0 if args.no_cpu_baseline else max(32, args.cpu_sample_rows // 8))
    print(json.dumps(result))


if __name__ == "__main__":
    main()
