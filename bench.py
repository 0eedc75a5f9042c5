#!/usr/bin/env python3
"""Benchmark of the hot path: per-call activation step + fused forward of one quantized
linear layer with a quantized low-rank branch, on synthetic DiT-shaped layers, one MI355X.

A "step" is one pass of the whole per-call path (lq_quantize_act + lq_linear_lowrank_fwd)
over one batch of M tokens already resident in HBM; weight packing is offline and untimed.
Prints ONE JSON line.  Its top-level fields describe the headline workload (the largest layer, the 2240 -> 11200
expansion on 8192 tokens): metric, value (whole-path TOPS), ms_per_step, a `roofline` object for the forward kernel
(bound, achieved, peak, fraction, measured HBM traffic), an `act_kernel` object and a `cpu_baseline` object (the CPU
oracle timed on the host cores on a row sample of the same workload).  `layers` holds the same per-kernel figures for
every benchmark layer (the INT4 layers of both transformer shapes and the seven MX-format layers of one block).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# MI355X dense matrix peaks: FP8 / INT8 (the INT4 main product runs on the FP8 pipe) and FP4 (MXFP4)
PEAK_MFMA_TFLOPS = {"int": 5033.0, "mx": 10066.0, "mxb": 10066.0, "mxi": 5033.0}
# HBM bytes per forward launch from two rocprofv3 --pmc runs (FETCH_SIZE, then WRITE_SIZE, KiB per dispatch; the
# commands and the raw figures are in profiles/hbm_traffic_forward_kernels.md), each scaled by the factor a plain copy
# of known size gives for the same counter.  A workload without an entry reports "traffic": null.
TRAFFIC_KIB = {    # name -> (FETCH_SIZE KiB, WRITE_SIZE KiB) per forward dispatch
    "c2_qkv": (23067.7, 55296.0), "c3_fc1": (34074.1, 74752.0), "c3_fc2": (50272.8, 18432.0),
    "c4_qkv": (85620.8, 107520.0), "c4_expand": (141964.1, 179200.0),
    "c5_qkv": (32643.3, 110592.0), "c5_attn_out": (11150.8, 36864.0), "c5_cross_kv": (17891.1, 73728.0),
    "c5_fc1": (44283.0, 147456.0), "c5_fc2": (56317.4, 36864.0),
    # same shape, same kernel as c5_attn_out (1152 -> 1152 on 16384 tokens)
    "c5_cross_q": (11150.8, 36864.0), "c5_cross_out": (11150.8, 36864.0),
}
TRAFFIC_SCALE = (2.0, 1.0)   # copy-kernel calibration of FETCH_SIZE and WRITE_SIZE
HEADLINE = "c4_expand"
BENCH_LAYERS = ["c2_qkv", "c3_fc1", "c3_fc2", "c4_qkv", "c4_expand", "c5_qkv", "c5_attn_out", "c5_cross_q", "c5_cross_kv",
                "c5_cross_out", "c5_fc1", "c5_fc2"]


def layer_ops(l):
    return 2.0 * l.M * l.N * l.K + 2.0 * l.M * l.r * l.K + 2.0 * l.M * l.N * l.r


def bench_calib(args, layer, np, torch, lq, wl):
    """K Adam steps of the factor optimisation (Eq. 4) on the layer's weight shape, SVD-free synthetic start
    (the start does not change the work per step).  value = steps per second; the error kernel's roofline is HBM:
    it reads W and writes the error matrix, 8 bytes per weight."""
    _, W, L, R = wl.make_inputs(layer)
    cfg = lq.config_for_layer(layer)
    Wd = torch.from_numpy(W).cuda()
    scale = np.float32(10.0)                       # factors of the size an SVD start would have
    state = lq.lq_calib_init(cfg, torch.from_numpy(L * scale).cuda(), torch.from_numpy(R * scale).cuda())
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    t = 0
    t_ramp = time.perf_counter()
    while time.perf_counter() - t_ramp < args.ramp_seconds:
        for _ in range(50):
            t += 1
            lq.lq_calib_step(cfg, Wd, state, t, loss=loss)
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        t += 1
        lq.lq_calib_step(cfg, Wd, state, t, loss=loss)
    torch.cuda.synchronize()
    K = args.steps
    t0 = time.perf_counter()
    for _ in range(K):
        t += 1
        lq.lq_calib_step(cfg, Wd, state, t, loss=loss)
    torch.cuda.synchronize()
    ms_step = (time.perf_counter() - t0) * 1e3 / K
    N, Kd, r = layer.N, layer.K, layer.r
    flops = 3 * 2.0 * N * Kd * r                   # W + L R, E R^T, L^T E
    hbm = 8.0 * N * Kd                             # error kernel: W in, E out
    out = {"metric": "data-free calibration (Eq. 4) Adam steps per second", "value": round(1e3 / ms_step, 1), "unit": "steps/s",
           "n_gpus": 1, "steps": K, "warmup": args.warmup, "ms_per_step": round(ms_step, 5), "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": layer.name + "_calib", "N": N, "K": Kd, "rank": r,
                      "main": {"mx": "MXFP4", "mxb": "MXFP4", "mxi": "MXINT4"}.get(
                          layer.family, "SINT4 blocks" if layer.a_group == 64 else f"INT4 g{layer.g}"),
                      "launches_per_step": 4},
           "work_per_step": {"flops": flops, "hbm_bytes_error_kernel": hbm, "loss": float(loss.item())}}
    if args.oracle_seconds > 0:
        from oracle import lq_ref
        st = lq_ref.calib_init(L * scale, R * scale)
        t0 = time.perf_counter()
        q1 = {"mx": "mxfp4", "mxb": "mxfp4", "mxi": "mxint4"}.get(layer.family, "sint4" if layer.a_group == 64 else "int")
        lq_ref.calib_step(W, st, layer.g, q1=q1)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(1.0 / dt, 3), "unit": "steps/s", "cores": lq_ref.num_threads(), "kind": "oracle",
                               "sample": "one full step of the same layer"}
    print(json.dumps(out))


def bench_rot(args, layer, np, torch, lq, wl):
    """K steps of the rotation search (Section 3.3, Eq. 6-7) on the layer's factor shapes.  value = steps per second."""
    _, _, L, R = wl.make_inputs(layer)
    cfg = lq.config_for_layer(layer)
    scale = np.float32(10.0)
    Ld, Rd = torch.from_numpy(L * scale).cuda(), torch.from_numpy(R * scale).cuda()
    state = lq.lq_rot_init(cfg)
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    opt = dict(lr=0.5, beta=0.9, s=2, grad_scale=1.0)
    t_ramp = time.perf_counter()
    while time.perf_counter() - t_ramp < args.ramp_seconds:
        for _ in range(50):
            lq.lq_rot_step(cfg, Ld, Rd, state, loss=loss, **opt)
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        lq.lq_rot_step(cfg, Ld, Rd, state, loss=loss, **opt)
    torch.cuda.synchronize()
    K = args.steps
    t0 = time.perf_counter()
    for _ in range(K):
        lq.lq_rot_step(cfg, Ld, Rd, state, loss=loss, **opt)
    torch.cuda.synchronize()
    ms_step = (time.perf_counter() - t0) * 1e3 / K
    N, Kd, r = layer.N, layer.K, layer.r
    out = {"metric": "rotation search (Eq. 7) Cayley-SGD steps per second", "value": round(1e3 / ms_step, 1), "unit": "steps/s",
           "n_gpus": 1, "steps": K, "warmup": args.warmup, "ms_per_step": round(ms_step, 5), "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": layer.name + "_rot", "N": N, "K": Kd, "rank": r, "q2_bits": layer.br_w_bits,
                      "launches_per_step": 5},
           "work_per_step": {"flops": 2.0 * (2 * 2 + 1) * (N + Kd) * r * r + 2.0 * 8 * r ** 3, "loss": float(loss.item())}}
    if args.oracle_seconds > 0:
        from oracle import lq_ref
        st = lq_ref.rot_init(r)
        t0 = time.perf_counter()
        q2 = {"mx": "fp8", "mxi": "mxint"}.get(layer.family, ("mxfp6" if layer.br_w_bits == 6 else "mxfp8") if layer.family == "mxb" else "int")
        lq_ref.rot_step(L * scale, R * scale, st, bits=layer.br_w_bits, q2=q2)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(1.0 / dt, 3), "unit": "steps/s", "cores": lq_ref.num_threads(), "kind": "oracle",
                               "sample": "one full step of the same layer"}
    print(json.dumps(out))


def measure_layer(args, layer, np, torch, lq, wl, keep=False):
    """All timings of one layer.  Returns (result dict, context for the oracle leg or None)."""
    X, W, L, R = wl.make_inputs(layer)
    cfg = lq.config_for_layer(layer)
    M = layer.M
    packed = lq.lq_pack_weights(cfg, torch.from_numpy(W).cuda(), torch.from_numpy(L).cuda(),
                                torch.from_numpy(R).cuda())
    nsets = max(1, args.sets)
    rng = np.random.default_rng(123)
    Xs, acts, Ys = [], [], []
    for i in range(nsets):
        Xi = X if i == 0 else X[rng.permutation(M)]      # same distribution, different bytes
        Xs.append(wl.to_dev_x(Xi, layer.x_dtype))
        acts.append(torch.empty(lq.lq_act_sizes(cfg, M), dtype=torch.uint8, device="cuda"))
        Ys.append(torch.empty((M, layer.N), dtype=torch.bfloat16, device="cuda"))

    def step(i):
        k = i % nsets
        lq.lq_quantize_act(cfg, packed, Xs[k], act=acts[k])
        lq.lq_linear_lowrank_fwd(cfg, packed, acts[k], M, Y=Ys[k])

    t_ramp = time.perf_counter()
    while time.perf_counter() - t_ramp < args.ramp_seconds:
        for i in range(100):
            step(i)
        torch.cuda.synchronize()
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    # ---- timed region: exactly K steps, whole-path wall clock, nothing but the two launches -----
    K = args.steps
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K):
        step(i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_step = (t1 - t0) * 1e3 / K

    # ---- per-kernel durations, HIP events on the stream the kernels run on, two ways; each can only overstate a kernel's
    # duration, and the smaller one is reported (both are in the output; rocprofv3's kernel-trace average of the same
    # command is lower than either, profiles/):
    # (1) a second run of the same step sequence (activation step, forward, rotating buffer sets) with an event before and
    #     after every launch: includes what an event pair costs (a few us; dominates for the short kernels);
    # (2) KK launches of ONE kernel back to back between two events: includes the inter-dispatch gaps, and a loop of
    #     forward launches alone heats the chip into lower clocks than the real step loop (5-8 % on the long kernels).
    KK = max(K, args.kernel_iters)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(KK)]
    torch.cuda.synchronize()
    for i in range(KK):
        k = i % nsets
        ev[i][0].record()
        lq.lq_quantize_act(cfg, packed, Xs[k], act=acts[k])
        ev[i][1].record()
        lq.lq_linear_lowrank_fwd(cfg, packed, acts[k], M, Y=Ys[k])
        ev[i][2].record()
    torch.cuda.synchronize()
    act_ms_step = sum(e[0].elapsed_time(e[1]) for e in ev) / KK
    fwd_ms_step = sum(e[1].elapsed_time(e[2]) for e in ev) / KK
    e = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
    e[0].record()
    for i in range(KK):
        lq.lq_linear_lowrank_fwd(cfg, packed, acts[i % nsets], M, Y=Ys[i % nsets])
    e[1].record()
    torch.cuda.synchronize()
    e[2].record()
    for i in range(KK):
        lq.lq_quantize_act(cfg, packed, Xs[i % nsets], act=acts[i % nsets])
    e[3].record()
    torch.cuda.synchronize()
    fwd_ms_b2b = e[0].elapsed_time(e[1]) / KK
    act_ms_b2b = e[2].elapsed_time(e[3]) / KK
    fwd_ms, act_ms = min(fwd_ms_step, fwd_ms_b2b), min(act_ms_step, act_ms_b2b)

    ops = layer_ops(layer)
    fwd_ops = 2.0 * layer.M * layer.N * (layer.K + layer.r)
    tops = ops / (ms_step * 1e-3) / 1e12
    fwd_tops = fwd_ops / (fwd_ms * 1e-3) / 1e12
    # activation kernel: algorithmic HBM bytes = X in, 4-bit codes + scales + tq out
    xb = 2 if layer.x_dtype == "bf16" else 4
    act_bytes = layer.M * layer.K * (xb + 0.5) + layer.M * (layer.r + 8)
    act_gbs = act_bytes / (act_ms * 1e-3) / 1e9

    mx = layer.family in ("mx", "mxb", "mxi")      # block-scaled main product (E8M0 per 32 values)
    mxb = layer.family == "mxb"
    mxi = layer.family == "mxi"
    peak = PEAK_MFMA_TFLOPS[layer.family]
    # algorithmic HBM bytes of the forward launch: 4-bit codes of both operands and their scales, the
    # rank-r operands, per-token / per-channel scales in, bf16 Y out
    rp = 0 if layer.r == 0 else (-(-layer.r // 64) * 64 if mx else -(-layer.r // 32) * 32)
    if mxi:  # branch elements travel as bf16 (2 bytes each), one scale byte per 32 values
        rp = 2 * layer.r
    if mx:
        scale_bytes = (layer.M + layer.N) * (layer.K // 32) + (0 if mxi else rp // 32 if mxb else 4) * (layer.M + layer.N)
    else:
        # (SINT4 blocks: an FP16 scale per 64 values of either operand, counted at the 4 bytes the layouts store)
        scale_bytes = 4 * layer.N * (layer.K // layer.g) + 4 * (2 * layer.M + layer.N) + \
            (4 * layer.M * (layer.K // 64) if layer.a_group == 64 else 0)
    fwd_bytes = (layer.M + layer.N) * layer.K / 2 + scale_bytes + (layer.M + layer.N) * rp + 2.0 * layer.M * layer.N
    t_mfma = fwd_ops / (peak * 1e12)
    t_hbm = fwd_bytes / 8.0e12
    fwd_gbs = fwd_bytes / (fwd_ms * 1e-3) / 1e9
    kib = TRAFFIC_KIB.get(layer.name)
    res = {
        "value": round(tops, 2), "ms_per_step": round(ms_step, 5),
        "dtype": "mxint4" if mxi else "mxfp4" if mx else "int4",
        "config": {"workload": layer.name, "M": layer.M, "K": layer.K, "N": layer.N, "rank": layer.r,
                   "main": "W4A4 MXINT4 block 32" if mxi else "W4A4 MXFP4 block 32" if mx else
                           "W4A4 SINT4 blocks of 64, FP16 scales" if layer.a_group == 64 else f"W4A4 INT4 g{layer.g}",
                   "branch": f"W{layer.br_w_bits}A8 MXINT block 32" if mxi else ("W6A6 MXFP6e2 block 32" if layer.br_w_bits == 6 else "W8A8 MXFP8e4 block 32") if mxb else "W8A8 FP8 E4M3" if mx else f"W{layer.br_w_bits}A{layer.br_a_bits}",
                   "x_dtype": layer.x_dtype, "buffer_sets": nsets,
                   "arithmetic": ("int4 codes as FP8 subnormals with E8M0 block scales on the scaled FP8 MFMA, "
                                  "bf16-exact MXINT branch, fp32 accumulate" if mxi else
                                  "e2m1 x e8m0 on the scaled FP4 MFMA, e4m3 branch, fp32 accumulate" if mx else
                                  "int4 codes (exact; 6-bit E2M3 fields on the f8f6f4 MFMA), int8 branch, fp32 dequantisation")},
        # the bound is whichever of ops/peak and bytes/bandwidth is the longer time for this layer (the
        # K = 1152 MXFP4 layers write 2 bytes per 2*1152 ops at the FP4 rate: below the ridge)
        "roofline": ({"bound": "mfma", "achieved": round(fwd_tops, 2), "peak": peak, "unit": "TFLOP/s",
                      "frac": round(fwd_tops / peak, 4)} if t_mfma >= t_hbm else
                     {"bound": "hbm", "achieved": round(fwd_gbs, 1), "peak": 8000.0, "unit": "GB/s",
                      "frac": round(fwd_gbs / 8000.0, 4)}),
        "act_kernel": {"bound": "hbm", "avg_kernel_ms": round(act_ms, 5), "achieved": round(act_gbs, 1),
                       "peak": 8000.0, "unit": "GB/s", "frac": round(act_gbs / 8000.0, 4)},
    }
    res["roofline"].update({
        "kernel": "mxi_fwd_kernel" if mxi else "mx_fwd_kernel" if mx else "fwd_int_kernel",
        "traffic": None if kib is None else (kib[0] * TRAFFIC_SCALE[0] + kib[1] * TRAFFIC_SCALE[1]) * 1024.0,
        "algorithmic_ops": fwd_ops, "algorithmic_bytes": fwd_bytes, "avg_kernel_ms": round(fwd_ms, 5),
        "kernel_timing": f"HIP events, the smaller of two overstating means over {KK} launches: per-launch event pairs inside the step sequence (event cost included), and back-to-back launches of the one kernel (dispatch gaps included)",
        "kernel_ms_in_step_sequence": round(fwd_ms_step, 5), "kernel_ms_back_to_back": round(fwd_ms_b2b, 5),
        "frac_of_mfma_peak": round(fwd_tops / peak, 4), "frac_of_hbm_peak": round(fwd_gbs / 8000.0, 4)})
    if kib is None:
        res["roofline"]["traffic_note"] = "no counter run recorded for this workload"
    if not mx:
        # the INT4 product is priced against the INT8 / FP8 dense peak (there is no 4-bit integer matrix instruction); the
        # instruction that multiplies the 6-bit code fields has the FP6 peak, quoted beside it
        res["roofline"]["frac_of_fp6_instruction_peak"] = round(fwd_tops / 10066.0, 4)
    ctx = (X, W, L, R, cfg, packed, Xs, acts, Ys, ops) if keep else None
    return res, ctx


def oracle_leg(args, layer, ctx, np, torch, lq, wl):
    """CPU oracle (reported baseline only): bounded row sample of the same workload."""
    from oracle import lq_ref
    X, W, L, R, cfg, packed, Xs, acts, Ys, ops = ctx
    M = layer.M
    mx = layer.family in ("mx", "mxb", "mxi")
    if layer.family == "mxi":
        pk = lq_ref.pack_mxi(W, L, R, layer.br_w_bits)
        run_rows = lambda n_rows: lq_ref.fwd_mxi(pk, lq_ref.quantize_act_mxi(X[:n_rows], pk))
    elif layer.family == "mxb":
        pk = lq_ref.pack_mxb(W, L, R, elem=layer.br_w_bits)
        run_rows = lambda n_rows: lq_ref.fwd_mxb(pk, lq_ref.quantize_act_mxb(X[:n_rows], pk))
    elif mx:
        pk = lq_ref.pack_mx(W, L, R)
        run_rows = lambda n_rows: lq_ref.fwd_mx(pk, lq_ref.quantize_act_mx(X[:n_rows], pk))
    else:
        pk = lq_ref.pack_int(W, L, R, layer.g, layer.br_w_bits, sint4_blocks=layer.a_group == 64)
        run_rows = lambda n_rows: lq_ref.fwd_int(pk, lq_ref.quantize_act_int(X[:n_rows], pk, layer.br_a_bits))
    probe = 16
    t = time.perf_counter()
    run_rows(probe)
    dt = time.perf_counter() - t
    rows = int(max(probe, min(M, probe * args.oracle_seconds / max(dt, 1e-6))))
    rows = max(16, rows // 16 * 16)
    t = time.perf_counter()
    o = run_rows(rows)
    dt = time.perf_counter() - t
    cpu_tops = ops * (rows / M) / dt / 1e12
    # parity spot check of the bench's own launch against those rows
    lq.lq_quantize_act(cfg, packed, Xs[0], act=acts[0])
    lq.lq_linear_lowrank_fwd(cfg, packed, acts[0], M, Y=Ys[0])
    torch.cuda.synchronize()
    gy = wl.bf16_to_bits(Ys[0][:rows])
    out = {"value": round(cpu_tops, 5), "unit": "TOPS", "cores": lq_ref.num_threads(),
           "kind": "oracle", "seconds": round(dt, 2),
           "sample": f"first {rows} of {M} token rows of {layer.name}, activation step + forward, "
                     f"scaled linearly in M"}
    if mx:  # fp32 accumulation order differs from the oracle's fp64: one-ulp bf16 flips at rounding boundaries
        out["gpu_rows_bf16_flip_rate"] = float(np.mean(gy != o.Y))
    else:
        out["gpu_rows_bit_exact"] = bool(np.array_equal(gy, o.Y))
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--ramp-seconds", type=float, default=0.5,
                    help="untimed run of the same step loop before the warm-up steps: the GPU leaves its idle "
                         "clock state only after some 0.2 s of load (a cold 10 ms loop runs ~15 %% slower)")
    ap.add_argument("--workload", default=HEADLINE, help="headline layer (name from workloads.LAYERS)")
    ap.add_argument("--layers", default="all",
                    help="'all' = every benchmark layer in the `layers` array, 'none' = headline only, or a comma-separated list")
    ap.add_argument("--kernel-iters", type=int, default=200,
                    help="launches per kernel in the per-kernel timing runs (at least --steps)")
    ap.add_argument("--oracle-seconds", type=float, default=15.0, help="CPU budget of the oracle leg (0 = skip)")
    ap.add_argument("--sets", type=int, default=4, help="distinct buffer sets rotated through")
    ap.add_argument("--calib", action="store_true",
                    help="time the data-free calibration step (lq_calib_step) on the workload's weight shape instead "
                         "of the per-call path; prints its own JSON line")
    ap.add_argument("--rot", action="store_true",
                    help="time the rotation search step (lq_rot_step) on the workload's factor shapes; prints its own JSON line")
    ap.add_argument("--copy-probe", type=int, default=0, metavar="BYTES",
                    help="only run a plain device-to-device copy of BYTES (calibrates the HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU (token rows are independent through the whole path, so it "
              "would shard over tokens with no collective); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2604_18117_amd import binding as lq
    from paper_2604_18117_amd import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.copy_probe:
        src = torch.empty(args.copy_probe, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe_bytes": args.copy_probe, "copies": 3}))
        return
    layer = wl.LAYERS[args.workload]
    if args.calib:
        return bench_calib(args, layer, np, torch, lq, wl)
    if args.rot:
        return bench_rot(args, layer, np, torch, lq, wl)

    head, ctx = measure_layer(args, layer, np, torch, lq, wl, keep=args.oracle_seconds > 0)
    out = {
        "metric": "fused W4A4+low-rank linear TOPS and % of MFMA roofline on MI355X",
        "value": head["value"], "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": head["dtype"], "data": "synthetic",
        "config": head["config"], "roofline": head["roofline"], "act_kernel": head["act_kernel"],
    }
    if args.oracle_seconds > 0:
        out["cpu_baseline"] = oracle_leg(args, layer, ctx, np, torch, lq, wl)
    del ctx
    torch.cuda.empty_cache()
    names = [] if args.layers == "none" else BENCH_LAYERS if args.layers == "all" else args.layers.split(",")
    layers = []
    for name in names:
        if name == layer.name:
            r = head
        else:
            r, _ = measure_layer(args, wl.LAYERS[name], np, torch, lq, wl)
            torch.cuda.empty_cache()
        layers.append({"workload": name, "M": r["config"]["M"], "K": r["config"]["K"], "N": r["config"]["N"],
                       "rank": r["config"]["rank"], "main": r["config"]["main"], "branch": r["config"]["branch"],
                       "tops": r["value"], "ms_per_step": r["ms_per_step"], "bound": r["roofline"]["bound"],
                       "frac": r["roofline"]["frac"], "avg_kernel_ms": r["roofline"]["avg_kernel_ms"],
                       "frac_of_mfma_peak": r["roofline"]["frac_of_mfma_peak"],
                       "frac_of_hbm_peak": r["roofline"]["frac_of_hbm_peak"], "traffic": r["roofline"]["traffic"],
                       "act_kernel_ms": r["act_kernel"]["avg_kernel_ms"], "act_kernel_gbs": r["act_kernel"]["achieved"],
                       "act_kernel_frac": r["act_kernel"]["frac"]})
    if layers:
        out["layers"] = layers
    print(json.dumps(out))


if __name__ == "__main__":
    main()
