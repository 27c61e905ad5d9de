#!/usr/bin/env python3
"""Benchmark of the SQ-format linear layer (sq_encode + sq_gemm) on one MI355X.

One "step" is one pass of the whole hot path over one batch: bf16 activations -> SQ-format ->
both integer products -> dequantised bf16 output, issued as ONE sq_linear call; the headline value is
wall time over K such calls between two device synchronisations.  The duration of each kernel comes from a
second loop over the same work issued as sq_encode + sq_gemm with HIP events between the launches (on the
stream they are launched on).  Inputs are synthetic, seeded, already in HBM.

Prints ONE JSON line: throughput of the step, the roofline of the dominant kernel, the encoder's rate, measured
chip rates, a dense W4A8 run of the same shape and the CPU oracle timed on a row sample.
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

INT8_PEAK_TOPS = 5000.0  # MI355X dense INT8 matrix peak (vendor figure, no sparsity), TOP/s
HBM_PEAK_GBS = 8000.0    # MI355X HBM3E peak, GB/s

# HBM-side bytes per sq_gemm launch, from rocprofv3's FETCH_SIZE and WRITE_SIZE counters (two runs of this
# script per workload, summaries under profiles/), each scaled by what the same counter reads for a plain
# device copy of known size (FETCH_SIZE x 2.0, WRITE_SIZE x 1.0).  Counters cannot be read from inside
# this process, so the figures are the recorded ones; they apply to the unmodified workload shapes only.
MEASURED_GEMM_TRAFFIC = {
    "c3": {"fetch_bytes": 642.3e6, "write_bytes": 211.4e6, "source": "profiles/sq_linear_c3_mlp7b.md"},
    "c4": {"fetch_bytes": 236.6e6, "write_bytes": 40.4e6, "source": "profiles/sq_linear_c4_down7b_static.md"},
    "c5": {"fetch_bytes": 3302.5e6, "write_bytes": 550.5e6, "source": "profiles/sq_linear_c5_up70b.md"},
}

WORKLOADS = {
    "c2": ("c2_qkv7b", {}),
    "c3": ("c3_mlp7b", {}),
    "c4": ("c4_down7b_static", {}),
    "c5": ("c5_up70b", {}),
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="c3", choices=sorted(WORKLOADS), help="benchmark configuration (default: the 7B MLP shape)")
    ap.add_argument("--M", type=int, default=None)
    ap.add_argument("--bank", type=int, default=None)
    ap.add_argument("--topk", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense-baseline", action="store_true")
    ap.add_argument("--graph", action="store_true",
                    help="also replay the steps from a captured HIP graph (launch overhead removed; matters for few-token shapes)")
    ap.add_argument("--weights-sq", action="store_true", help="also time the SQ-format-on-weights layer (sq_wsq_linear) of the same shape")
    ap.add_argument("--no-probes", action="store_true", help="skip the measured matrix-instruction and streaming rates")
    ap.add_argument("--cpu-rows", type=int, default=0, help="rows of the CPU-oracle sample (0: sized for about 20 s)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain device copy of 256 MiB (for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    return ap.parse_args()


def dev(a):
    import torch

    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    elif a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(a).cuda()


def cpu_baseline(wl, rows_req):
    """The oracle as it stands, timed on the host cores, on a bounded row sample of the same workload."""
    import oracle

    oracle.build()
    cores = oracle.num_threads()
    if wl.mode == "static":
        # the oracle calibrates its own mask: nothing it is given comes from the HIP path
        mask, _ = oracle.static_mask(wl.calib_bits, wl.wq_packed, wl.w_scale, wl.bank, wl.topk)
    else:
        mask = None
    # size the sample from a short probe so that the whole leg stays near 15 s
    probe_rows = np.linspace(0, wl.M - 1, num=min(wl.M, 2 * cores), dtype=np.int64)
    t0 = time.perf_counter()
    enc = oracle.encode(wl.x_bits[probe_rows], wl.bank, wl.topk, static_mask=mask)
    oracle.gemm(enc, wl.wq_packed, wl.w_scale, want_y64=False)
    t_probe = time.perf_counter() - t0
    if rows_req > 0:
        n = min(wl.M, rows_req)
    else:
        n = int(min(wl.M, max(len(probe_rows), len(probe_rows) * 20.0 / max(t_probe, 1e-3))))
        n = max(cores, (n // cores) * cores)
    rows = np.linspace(0, wl.M - 1, num=n, dtype=np.int64)
    xs = np.ascontiguousarray(wl.x_bits[rows])
    t0 = time.perf_counter()
    enc = oracle.encode(xs, wl.bank, wl.topk, static_mask=mask)
    t_enc = time.perf_counter() - t0
    oracle.gemm(enc, wl.wq_packed, wl.w_scale, want_y64=False)
    t_all = time.perf_counter() - t0
    tops = 2.0 * n * wl.N * wl.K / t_all / 1e12
    return {
        "value": tops, "unit": "TOPS", "cores": cores, "kind": "oracle",
        "sample": f"{n} of {wl.M} token rows (evenly spaced), all {wl.N} output channels: encode + both products + epilogue",
        "seconds": round(t_all, 3), "encode_seconds": round(t_enc, 3),
        "extrapolated_full_seconds": round(t_all * wl.M / n, 1),
    }


def probes(torch, sq, xs, enc_write_bytes):
    """What the chip sustains, measured here, beside the vendor peaks: the products' matrix instruction on
    register operands, and a plain streaming kernel with the encoder's mix of bytes read and written."""
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    blocks, iters = 2 * n_cu, 2000
    sink = torch.empty(blocks * 256, dtype=torch.int32, device="cuda")
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    rates = {}
    for random_operands in (False, True):
        sq.sq_probe_mfma_i8(blocks, iters, sink, random_operands)
        torch.cuda.synchronize()
        e0.record()
        sq.sq_probe_mfma_i8(blocks, iters, sink, random_operands)
        e1.record()
        torch.cuda.synchronize()
        rates[random_operands] = 2.0 * 32768 * 8 * iters * 4 * blocks / (e0.elapsed_time(e1) * 1e-3) / 1e12
    mfma_tops = rates[False]
    alt = {}
    for kind, name in ((0, "mfma_fp6_e3m2_register_only_tops"), (1, "smfmac_i8_2to4_register_only_dense_equivalent_tops")):
        sq.sq_probe_mfma_alt(kind, blocks, iters, sink)
        torch.cuda.synchronize()
        e0.record()
        sq.sq_probe_mfma_alt(kind, blocks, iters, sink)
        e1.record()
        torch.cuda.synchronize()
        alt[name] = 2.0 * 65536 * 8 * iters * 4 * blocks / (e0.elapsed_time(e1) * 1e-3) / 1e12

    read_bytes = xs[0].numel() * xs[0].element_size()
    write_bytes = (int(enc_write_bytes) + 15) // 16 * 16
    dst = torch.empty(max(16, write_bytes), dtype=torch.uint8, device="cuda")
    for i in range(3):
        sq.sq_probe_stream(xs[i % len(xs)], read_bytes, dst, write_bytes)
    torch.cuda.synchronize()
    reps = 30
    e0.record()
    for i in range(reps):
        sq.sq_probe_stream(xs[i % len(xs)], read_bytes, dst, write_bytes)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    return {"mfma_i8_register_only_tops": mfma_tops, "mfma_i8_frac_of_peak": mfma_tops / INT8_PEAK_TOPS,
            "mfma_i8_register_only_random_operands_tops": rates[True], **alt,
            "stream_encode_mix_gbs": (read_bytes + write_bytes) / (ms * 1e-3) / 1e9,
            "stream_encode_mix_ms": ms, "stream_read_bytes": read_bytes, "stream_write_bytes": write_bytes,
            "note": "sq_probe_mfma_i8: 8 independent v_mfma_i32_32x32x32_i8 per wave per iteration, 2 workgroups per CU, "
                    "constant operands / pseudo-random widened INT4 operands that change every instruction; "
                    "sq_probe_stream: coalesced 16-byte reads of X and writes of as many bytes as sq_encode writes"}


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding or collectives are part of it); "
              "run it with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2512_05409_amd as sq
    import workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    sq.lib()

    name, kw = WORKLOADS[args.workload]
    kw = dict(kw)
    if args.M is not None:
        kw["M"] = args.M
    if args.bank is not None:
        kw["bank"] = args.bank
    if args.topk is not None:
        kw["topk"] = args.topk
    wl = workloads.make(name, **kw)
    M, K, N, b, k = wl.M, wl.K, wl.N, wl.bank, wl.topk
    static = wl.mode == "static"

    p = sq.params(M, K, N, b, k, mode=sq.SQ_STATIC if static else sq.SQ_DYNAMIC, out_dtype=sq.SQ_OUT_BF16)
    wqd, swd = dev(wl.wq_packed), dev(wl.w_scale)
    mask, md, pre, calibration = None, None, None, None
    if static:
        # The channel mask comes from the library's own calibration (Algorithm 2) of the workload's calibration
        # batch, on the device; it is timed on its own, outside the step.
        cal = dev(wl.calib_bits)
        T = wl.calib_bits.shape[0]
        md = torch.zeros(K // 32, dtype=torch.int32, device="cuda")
        cws = torch.empty(sq.sq_calibrate_workspace_bytes(p, T), dtype=torch.uint8, device="cuda")
        w0 = sq.weight(wqd, swd, None)
        for _ in range(3):
            sq.sq_calibrate_static(p, cal, T, w0, md, None, cws)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            sq.sq_calibrate_static(p, cal, T, w0, md, None, cws)
        e1.record()
        torch.cuda.synchronize()
        cal_ms = e0.elapsed_time(e1) / 10
        cal_bytes = T * K * 2 + N * K // 2 + 4 * N + K // 8
        calibration = {"kernel": "sq_calibrate_static (4 kernels)", "bound": "hbm", "ms": cal_ms,
                       "algorithmic_bytes": cal_bytes, "achieved": cal_bytes / (cal_ms * 1e-3) / 1e9,
                       "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": cal_bytes / (cal_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                       "calibration_tokens": T, "note": "inputs not rotated: partly served from the Infinity Cache"}
        # the weights are reordered by the mask on the device, from the device copy of the mask alone
        pre = torch.empty(sq.sq_weight_prepack_bytes(p), dtype=torch.uint8, device="cuda")
        bad = torch.zeros(1, dtype=torch.int32, device="cuda")
        sq.sq_weight_prepack(p, wqd, None, md, pre, bad_banks=bad)
        torch.cuda.synchronize()
        assert int(bad.item()) == 0, "calibration produced a malformed mask"
    w = sq.weight(wqd, swd, pre)
    # Few tokens: the GEMM streams the weights once and is HBM-bound (the ridge of INT8 MFMA against HBM is near
    # M = 157), so the weights rotate over copies that together exceed the 256 MB Infinity Cache as well.
    hbm_bound = M <= 128
    ws = [w]
    if hbm_bound and not static:
        n_w = max(2, min(8, -(-300_000_000 // (N * K // 2))))
        w_copies = [wqd.clone() for _ in range(n_w - 1)]  # sq_weight holds raw addresses: keep the tensors alive
        ws += [sq.weight(c, swd, None) for c in w_copies]

    # Rotating buffers: X copies whose total exceeds the 256 MB Infinity Cache, so the encoder reads HBM.
    x_bytes = M * K * 2
    n_x = max(2, min(16, -(-300_000_000 // x_bytes)))
    x0 = dev(wl.x_bits)
    xs = [x0] + [x0.clone() for _ in range(n_x - 1)]
    n_y = 2
    ys = [torch.empty(M * N, dtype=torch.int16, device="cuda") for _ in range(n_y)]
    acts = [sq.Act(p, static_mask=md, with_hi_dense=True, with_lo_compact=True) for _ in range(2)]
    if static:
        for a_ in acts:
            a_.d_lo = None  # as in sq_linear: only the reordered low part is produced and multiplied

    lws = torch.empty(sq.sq_linear_workspace_bytes(p), dtype=torch.uint8, device="cuda")

    def step(i):
        """The timed step: one sq_linear call (encode + both products + epilogue on one stream)."""
        sq.sq_linear(p, xs[i % n_x], ws[i % len(ws)], ys[i % n_y], lws, static_mask=md)

    def split_step(i, ev):
        """The same work as two calls (what sq_linear enqueues), with events between them: per-kernel times."""
        a = acts[i % 2]
        ev[0].record()
        sq.sq_encode(p, xs[i % n_x], a, static_mask=md)
        ev[1].record()
        sq.sq_gemm(p, a, ws[i % len(ws)], ys[i % n_y], None)
        ev[2].record()

    if args.copy_calibration:
        # A copy kernel of known size: reads 2^28 bytes and writes 2^28 bytes per launch.
        src = torch.ones(1 << 28, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    # per-kernel durations: a second loop over the same work, outside the headline timing
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    for i in range(3):
        split_step(i, events[0])
    torch.cuda.synchronize()
    for i in range(args.steps):
        split_step(i, events[i])
    torch.cuda.synchronize()

    enc_ms = np.array([e[0].elapsed_time(e[1]) for e in events])
    gemm_ms = np.array([e[1].elapsed_time(e[2]) for e in events])
    ms_per_step = wall * 1e3 / args.steps
    ops_eff = 2.0 * M * N * K
    eff_tops = ops_eff / (ms_per_step * 1e-3) / 1e12

    # Algorithmic work of the dominant kernel (the GEMM): both products the layer is defined with.
    alg_ops = 2.0 * M * N * K * (1.0 + k / b)
    # dynamic: the high pass is zero-padded to dense; static: both operands reordered, low pass over K - K_hi
    issued_ops = 2.0 * M * N * K * (1.0 if static else 2.0)
    gemm_s = float(gemm_ms.mean()) * 1e-3
    enc_s = float(enc_ms.mean()) * 1e-3
    enc_bytes = M * K * 2 + (M * (K - (K // b) * k) // 2 if static else M * K // 2) + M * (K // b) * k + (0 if static else M * K // 8) + 8 * M
    enc_bytes_written_extra = 0 if static else M * K  # the matrix-core-ready image of the high part
    # what one GEMM launch has to move at least: the encoded activations, the weights, the scales, the output
    gemm_bytes = ((M * (K - (K // b) * k) // 2 if static else M * K // 2) + M * (K // b) * k
                  + (0 if static else M * K // 8) + 8 * M + N * K // 2 + 4 * N + 2 * M * N)

    traffic, traffic_detail = None, None
    if args.workload in MEASURED_GEMM_TRAFFIC and args.M is None and args.bank is None and args.topk is None:
        traffic_detail = dict(MEASURED_GEMM_TRAFFIC[args.workload])
        traffic = traffic_detail["fetch_bytes"] + traffic_detail["write_bytes"]
        a_bytes = (M * (K - (K // b) * k) // 2 + M * (K // b) * k) if static else (M * K // 2 + M * K)
        w_bytes = N * K // 2
        traffic_detail["compulsory_bytes"] = a_bytes + w_bytes + 8 * M + 4 * N + 2 * M * N

    if hbm_bound:
        roofline = {"kernel": "sq_gemm", "bound": "hbm", "achieved": gemm_bytes / gemm_s / 1e9, "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": gemm_bytes / gemm_s / 1e9 / HBM_PEAK_GBS, "traffic": traffic,
                    "traffic_detail": traffic_detail, "algorithmic_bytes": gemm_bytes,
                    "weight_buffers_rotated": len(ws)}
    else:
        roofline = {"kernel": "sq_gemm", "bound": "mfma", "achieved": alg_ops / gemm_s / 1e12, "peak": INT8_PEAK_TOPS,
                    "unit": "TOP/s", "frac": alg_ops / gemm_s / 1e12 / INT8_PEAK_TOPS, "traffic": traffic,
                    "traffic_detail": traffic_detail,
                    "algorithmic_ops": alg_ops, "issued_mfma_ops": issued_ops,
                    "issued_frac": issued_ops / gemm_s / 1e12 / INT8_PEAK_TOPS}
    roofline.update({"ms": gemm_s * 1e3, "ms_median": float(np.median(gemm_ms)), "ms_min": float(gemm_ms.min()),
                     "effective_tops_2MNK": ops_eff / gemm_s / 1e12})

    # Storage of the encoded activations: as laid out here (low part dense over K) and in the paper's own
    # accounting of equivalent bits (Section 4.1: the low part counted over its own channels only).
    storage = {"bytes_per_element_dense_low": 0.5 + k / b + (0.0 if static else 0.125),
               "equivalent_bits_paper": 8.0 * k / b + 4.0 * (1.0 - k / b)}

    out = {
        "metric": "SQ-format linear effective TOPS (encode+GEMM) and % of INT8 MFMA peak, 1 GPU",
        "value": eff_tops, "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "data": "synthetic",
        "config": {"workload": f"{name}: X bf16 [{M},{K}] -> SQ-format bank={b} topk={k} {wl.mode}; "
                               f"W INT4 [{N},{K}] per-row scales; Y bf16 [{M},{N}]",
                   "M": M, "K": K, "N": N, "bank": b, "topk": k, "mode": wl.mode, "out": "bf16",
                   "x_buffers_rotated": n_x},
        "pct_int8_peak_effective": 100.0 * eff_tops / INT8_PEAK_TOPS,
        "roofline": roofline,
        "encode": {"kernel": "sq_encode", "bound": "hbm", "achieved": enc_bytes / enc_s / 1e9, "peak": HBM_PEAK_GBS,
                   "unit": "GB/s", "frac": enc_bytes / enc_s / 1e9 / HBM_PEAK_GBS, "ms": enc_s * 1e3,
                   "ms_median": float(np.median(enc_ms)), "ms_min": float(enc_ms.min()),
                   "algorithmic_bytes": enc_bytes,
                   "extra_bytes_written_hi_dense": enc_bytes_written_extra,
                   "achieved_incl_hi_dense": (enc_bytes + enc_bytes_written_extra) / enc_s / 1e9},
        "activation_storage": storage,
    }
    if calibration is not None:
        out["calibration"] = calibration

    if args.graph:
        # The same steps replayed from a captured graph: the library only enqueues kernels, so a step can be
        # captured; one graph holds enough steps to walk through every rotating buffer.
        per_graph = int(np.lcm.reduce([n_x, n_y, 2, len(ws)]))
        while per_graph < 8:
            per_graph *= 2
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                for i in range(per_graph):
                    a = acts[i % 2]
                    sq.sq_encode(p, xs[i % n_x], a, static_mask=md, stream=side)
                    sq.sq_gemm(p, a, ws[i % len(ws)], ys[i % n_y], None, stream=side)
        torch.cuda.synchronize()
        replays = max(3, -(-args.steps // per_graph))
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(replays):
            graph.replay()
        torch.cuda.synchronize()
        g_ms = (time.perf_counter() - t0) * 1e3 / (replays * per_graph)
        out["graph"] = {"ms_per_step": g_ms, "steps_per_graph": per_graph, "replays": replays,
                        "effective_tops_2MNK": ops_eff / (g_ms * 1e-3) / 1e12,
                        "weight_stream_gbs": gemm_bytes / (g_ms * 1e-3) / 1e9 if hbm_bound else None}

    if not args.no_probes:
        out["achievable"] = probes(torch, sq, xs, enc_bytes + enc_bytes_written_extra - M * K * 2)

    if not args.no_dense_baseline:
        # Plain per-token W4A8 of the same shape on the same matrix-core kernel (what W4A8 falls back to).
        pd = sq.params(M, K, N, out_dtype=sq.SQ_OUT_BF16)
        a8 = torch.randint(-127, 128, (M, K), dtype=torch.int8, device="cuda")
        sa = torch.rand(M, dtype=torch.float32, device="cuda") * 0.1 + 0.01
        pre8 = torch.empty(N * K // 2, dtype=torch.uint8, device="cuda")
        sq.sq_dense_w4a8_prepack(pd, wqd, pre8)
        w8 = sq.weight(wqd, swd, pre8)
        for i in range(3):
            sq.sq_dense_w4a8_gemm(pd, a8, sa, w8, ys[i % n_y])
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = max(5, args.steps // 2)
        e0.record()
        for i in range(reps):
            sq.sq_dense_w4a8_gemm(pd, a8, sa, w8, ys[i % n_y])
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        out["dense_w4a8_baseline"] = {"ms": ms, "tops": ops_eff / (ms * 1e-3) / 1e12,
                                      "frac_int8_peak": ops_eff / (ms * 1e-3) / 1e12 / INT8_PEAK_TOPS,
                                      "note": "per-token INT8 activations x INT4 weights, same kernel, no SQ split"}

    if not static and not hbm_bound and (K // b) & (K // b - 1) == 0 and K // b <= 256:
        # The tied-scale variant of the same layer (s_lo = 16 s_hi: one INT8 operand, one accumulator), reported
        # beside the two-scale layer the headline is quoted on: a different numerical result with its own oracle.
        pt = sq.params(M, K, N, b, k, mode=sq.SQ_DYNAMIC_TIED, out_dtype=sq.SQ_OUT_BF16)
        wst = torch.empty(sq.sq_linear_workspace_bytes(pt), dtype=torch.uint8, device="cuda")
        for i in range(3):
            sq.sq_linear(pt, xs[i % n_x], w, ys[i % n_y], wst)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = max(5, args.steps // 2)
        e0.record()
        for i in range(reps):
            sq.sq_linear(pt, xs[i % n_x], w, ys[i % n_y], wst)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        out["tied_scale_variant"] = {"ms_per_step": ms, "tops_2MNK": ops_eff / (ms * 1e-3) / 1e12,
                                     "frac_int8_peak": ops_eff / (ms * 1e-3) / 1e12 / INT8_PEAK_TOPS,
                                     "kernel": sq.sq_gemm_variant(pt),
                                     "note": "sq_linear in mode SQ_DYNAMIC_TIED (encode + one INT8 x INT4 product): "
                                             "MACs issued = M*N*K; not the layer the headline value is quoted on"}

    if args.weights_sq and not hbm_bound:
        # The second workload of the paper, SQ-format on WEIGHTS (W(SQ)A8): the same shape with the weights encoded per
        # (output channel, bank) group (offline, not timed) and plain per-token INT8 activations.
        pw = sq.params(M, K, N, 64 if b < 64 else b, k if b >= 64 else 8, out_dtype=sq.SQ_OUT_BF16)
        w_bf16 = (torch.randn(N, K, device="cuda") * 0.04).to(torch.bfloat16).view(torch.int16)
        wsq = sq.WeightSQ(pw)
        sq.sq_wsq_encode(pw, w_bf16, wsq)
        prew = torch.empty(sq.sq_wsq_prepack_bytes(pw), dtype=torch.uint8, device="cuda")
        sq.sq_wsq_prepack(pw, wsq, prew)
        wsw = torch.empty(sq.sq_wsq_linear_workspace_bytes(pw), dtype=torch.uint8, device="cuda")
        for i in range(3):
            sq.sq_wsq_linear(pw, xs[i % n_x], wsq, prew, ys[i % n_y], wsw)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = max(5, args.steps // 4)
        e0.record()
        for i in range(reps):
            sq.sq_wsq_linear(pw, xs[i % n_x], wsq, prew, ys[i % n_y], wsw)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        # its bound: the per-bank fold, 5 vector instructions per output element and bank, against the chip's vector issue
        # rate (256 compute units x 4 SIMDs x 16 lanes x 2.4 GHz = 39.3 T lane-operations/s)
        fold_ops = 5.0 * M * N * (K // pw.bank)
        alu_peak = 256 * 4 * 16 * 2.4e9
        out["weights_sq_variant"] = {"ms_per_step": ms, "tops_2MNK": ops_eff / (ms * 1e-3) / 1e12, "bank": pw.bank, "topk": pw.topk,
                                     "roofline": {"bound": "alu", "achieved": fold_ops / (ms * 1e-3) / 1e12, "peak": alu_peak / 1e12,
                                                  "unit": "T lane-op/s", "frac": fold_ops / (ms * 1e-3) / alu_peak},
                                     "note": "sq_wsq_linear: per-token INT8 activations x SQ-format weights with per-(channel, bank) "
                                             "scales; bound by the per-bank fp32 fold (vector arithmetic), not by the matrix cores"}

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, args.cpu_rows)

    print(json.dumps(out))


if __name__ == "__main__":
    main()
