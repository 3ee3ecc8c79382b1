#!/usr/bin/env python3
"""Benchmark of the W4A8 GEMM hot path on one MI355X.

Default workload (`llama2_7b_decode_m64`): the four Llama-2-7B-shaped linear layers (fused
QKV, O-proj, fused gate+up, down) at M = 64 tokens, group size 128, seeded synthetic FP16
weights/activations with 1% outlier channels.  One step = one pass over the four layers;
each layer runs per-token activation quantization and the W4A8 GEMM through qoq_w4a8_linear
(two kernels back to back; weights are packed once, offline, before the timed region).  Several independently packed copies of the layer
set are rotated so the weights of a step come from HBM, not from the 256 MB Infinity Cache,
as they do when a whole model's layers stream through.

Prints ONE JSON line: effective TOPS (2*M*K*N summed over the layers / step time), the HBM
roofline of the GEMM launch with a plain streaming read of the same weights timed beside it
(`roofline.read_floor`), the same GEMMs fed by the producers with the quantizer fused in
(`fused_producer_step`), the compute-bound leg (`compute_leg`: Llama-3-70B-shaped layers at
M = 2048 with their own roofline and the matrix cores' measured ceiling), and the CPU oracle
timed on the host cores as a baseline.
`--sweep FILE` additionally writes per-layer, per-M timings of every configuration family.
`--attention` times the KV4 decode attention kernel instead (its own JSON line, same fields).
`--producers` times RMSNorm and SiLU*up with the quantizer fused in, at --m tokens (its own JSON line, same fields).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0       # MI355X HBM3E, published
INT8_PEAK_TOPS = 5033.0     # MI355X dense INT8 matrix, published (5.0 POP/s)
CALIB_BYTES = 256 << 20     # size of the calibration copy
# HBM traffic per GEMM launch is a counter figure (two `rocprofv3 --pmc` runs: FETCH_SIZE, WRITE_SIZE, scaled by the
# calibration copy); a benchmark run cannot count it itself.  The committed counter summary of a workload carries one
# machine-readable line
#     traffic_bytes_per_launch: <bytes> config: <layer>=<tile_m>/<split_k>,...
# and the figure is reported only while the launch configurations the library picks today are the ones that line
# was measured with (otherwise null: the figure would be stale).
TRAFFIC_PROFILES = {"llama2_7b_decode_m64": "profiles/w4a8_gemm_llama2_7b_decode_m64.txt"}


def profile_traffic(workload, config_now):
    """(bytes per launch, source file) from the committed counter summary, or (None, None)."""
    rel = TRAFFIC_PROFILES.get(workload)
    if rel is None:
        return None, None
    try:
        with open(os.path.join(ROOT, rel)) as f:
            for line in f:
                if line.startswith("traffic_bytes_per_launch:"):
                    head, _, cfg = line.partition("config:")
                    if cfg.strip() == config_now:
                        return float(head.split(":", 1)[1]), rel
    except (OSError, ValueError):
        pass
    return None, None


def load_read_probe():
    """The measurement probe built next to the library (a plain streaming read; see csrc/probe_read.hip)."""
    import ctypes

    from paper_2405_04532_amd import build as qbuild
    if not os.path.exists(qbuild.PROBE_LIB):
        raise RuntimeError(qbuild.PROBE_LIB + " is missing: run `python -m paper_2405_04532_amd.build` first")
    lib = ctypes.CDLL(qbuild.PROBE_LIB)
    lib.qoq_probe_read.restype = ctypes.c_int
    lib.qoq_probe_read.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p]
    lib.qoq_probe_mfma.restype = ctypes.c_int
    lib.qoq_probe_mfma.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
    return lib


def mfma_ceiling(dev):
    """What the INT8 matrix cores sustain on this machine, with no memory traffic at all (csrc/probe_mfma.hip): one
    wave per SIMD issuing nothing but the compute-bound kernel's matrix instruction, about 3 ms per mode so that the
    clock settles.  Fractions of the published peak."""
    import torch
    probe = load_read_probe()
    sink = torch.zeros(16, dtype=torch.int32, device=dev)
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    stream = torch.cuda.current_stream().cuda_stream
    out = {}
    names = {0: "constant_operands", 1: "random_operands", 2: "random_operands_with_dequant_valu",
             3: "gemm_like_operands_with_dequant_valu"}
    iters = 12000
    for mode, name in names.items():
        if probe.qoq_probe_mfma(mode, iters // 10, cus, sink.data_ptr(), stream) != 0:
            raise RuntimeError("qoq_probe_mfma refused its arguments")
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        probe.qoq_probe_mfma(mode, iters, cus, sink.data_ptr(), stream)
        e1.record()
        torch.cuda.synchronize()
        tops = 2.0 * 32 ** 3 * 16 * iters * 4 * cus / (e0.elapsed_time(e1) * 1e-3) / 1e12
        out[name] = round(tops / INT8_PEAK_TOPS, 4)
    out["kernel"] = ("v_mfma_i32_32x32x32_i8 back to back, one wave per SIMD on %d compute units, 16 accumulator tiles, "
                     "no memory or LDS traffic; fractions of the published peak" % cus)
    return out


def graph_schedule(steps, per_graph):
    """How `steps` timed steps are replayed from captured graphs: (replays of the full graph of `per_graph`
    consecutive steps, steps in one shorter graph replayed once after them).  Any steps >= 1 is timed exactly."""
    if steps < 1 or per_graph < 1:
        raise ValueError("steps and per_graph must be at least 1")
    return steps // per_graph, steps % per_graph


def algorithmic_bytes(M, N, K, mode=0):
    """Bytes the GEMM must move: packed codes, level-2 metadata (1.5 B per group), FP16
    channel scales, INT8 activations with their FP16 scales, FP16 output."""
    meta = 1.5 * N * (K // 128) if mode == 0 else N
    return K * N / 2 + meta + 2 * N + M * K + 2 * M + 2 * M * N


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--m", type=int, default=64, help="tokens per step (default workload: 64)")
    ap.add_argument("--copies", type=int, default=8, help="independently packed layer sets rotated per step")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-compute-leg", action="store_true",
                    help="skip the compute-bound leg (Llama-3-70B layers at M = 2048) that the default run appends")
    ap.add_argument("--compute-leg-only", action="store_true",
                    help="run only the compute-bound leg and print its object (for profiling that leg alone)")
    ap.add_argument("--sweep", type=str, default=None, help="also write a per-layer/per-M table to this file")
    ap.add_argument("--attention", action="store_true",
                    help="time the KV4 decode attention kernel instead (64 sequences x --seq tokens, Llama-2-7B heads)")
    ap.add_argument("--seq", type=int, default=1024, help="--attention: tokens in every sequence's cache")
    ap.add_argument("--batch", type=int, default=64, help="--attention: sequences decoded per launch")
    ap.add_argument("--family", type=str, default="llama2_7b", help="--attention: head configuration")
    ap.add_argument("--producers", action="store_true",
                    help="time the producers with the quantizer fused in (RMSNorm, SiLU*up) at --m tokens instead of the GEMM")
    ap.add_argument("--ablation", action="store_true",
                    help="dequantization-overhead ablation of the GEMM main loop and timings of the offline transforms")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(column-parallel layers would split N, row-parallel ones K on group boundaries with an exact INT32 "
              "reduce-scatter; none of that is built)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2405_04532_amd import api, workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    api.lib()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.attention:
        print(json.dumps(attention_bench(args, api, wl, dev)))
        return
    if args.ablation:
        print(json.dumps(ablation_bench(args, api, wl, dev)))
        return
    if args.producers:
        print(json.dumps(producers_bench(args, api, wl, dev)))
        return
    if args.compute_leg_only:
        print(json.dumps(compute_leg(args, api, wl, dev)))
        return
    M = args.m
    layers = list(wl.LLAMA2_7B.items())          # name -> (K, N)

    # ---- setup (untimed): weights packed offline, activations resident in HBM
    blobs = {name: [] for name, _ in layers}
    for name, (K, N) in layers:
        w = wl.layer_weights("llama2_7b", name, 1, dev)
        first = api.pack_weights(w)
        blobs[name].append(first)
        for _ in range(args.copies - 1):
            blobs[name].append(first.clone())
        del w
    xs = {name: wl.layer_activations("llama2_7b", name, M, 1, dev) for name, _ in layers}
    # A plain streaming kernel of known size (256 MiB read, 256 MiB written), launched three times during
    # set-up: under `rocprofv3 --pmc FETCH_SIZE|WRITE_SIZE` its reading gives the factor that converts the
    # counters of the GEMM launches of the same run into bytes.
    calib_src = torch.zeros(CALIB_BYTES // 4, dtype=torch.int32, device=dev)
    calib_dst = torch.empty_like(calib_src)
    for _ in range(3):
        torch.mul(calib_src, 1, out=calib_dst)
    del calib_src, calib_dst
    bufs = {}
    for name, (K, N) in layers:
        bufs[name] = dict(
            qx=torch.empty((M, K), dtype=torch.int8, device=dev),
            sx=torch.empty(M, dtype=torch.float16, device=dev),
            out=torch.empty((M, N), dtype=torch.float16, device=dev),
            rowsum=torch.empty(M, dtype=torch.int32, device=dev),
            ws=api.new_workspace(api.gemm_workspace_bytes(M, N, K), dev))
    L = api.lib()
    stream = torch.cuda.current_stream()
    sp = stream.cuda_stream
    P = lambda t: t.data_ptr()

    def check(rc):
        if rc != 0:
            raise RuntimeError(api.status_string(rc))

    def gemm_only(step, s=None):
        s = sp if s is None else s
        for name, (K, N) in layers:
            b = bufs[name]
            check(L.qoq_w4a8_gemm(P(b["qx"]), P(b["sx"]), None, P(blobs[name][step % args.copies]), M, N, K, 0,
                                  P(b["out"]), P(b["ws"]), b["ws"].numel(), s))

    def full_step(step, s=None):
        s = sp if s is None else s
        for name, (K, N) in layers:
            b = bufs[name]
            # per-token activation quantization, then the GEMM (two kernels back to back)
            # (group mode: the token sums of the per-channel epilogue are not needed and not asked for)
            check(L.qoq_w4a8_linear(P(xs[name]), P(blobs[name][step % args.copies]), M, N, K, 0, P(b["out"]),
                                    P(b["qx"]), P(b["sx"]), None, P(b["ws"]), b["ws"].numel(), s))

    def timed(fn, steps, warmup, per_graph=None):
        """Warm up eagerly, then time exactly `steps` steps.  The launches of `copies` consecutive steps are
        captured once into a HIP graph (launch-bound inner loops belong in graphs) and replayed steps // copies
        times; the remaining steps % copies steps come from a second, shorter graph.  Both events are recorded on
        the stream the graphs are launched on."""
        for i in range(warmup):
            fn(i)
        torch.cuda.synchronize()
        per_graph = args.copies if per_graph is None else per_graph
        full, rem = graph_schedule(steps, per_graph)

        def capture(n):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                cs = torch.cuda.current_stream().cuda_stream
                for i in range(n):
                    fn(i, cs)
            g.replay()                              # untimed first replay (uploads the graph)
            return g

        g_full = capture(per_graph) if full else None
        g_rem = capture(rem) if rem else None
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(full):
            g_full.replay()
        if rem:
            g_rem.replay()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / steps      # ms per step

    ms_step = timed(full_step, args.steps, args.warmup)
    ms_gemm = timed(gemm_only, args.steps, args.warmup)   # the four GEMM launches alone

    # The same four GEMMs fed the way Section 5.1 places the activation quantization: inside the memory-bound kernel
    # that produces the activations -- RMSNorm in front of QKV and gate+up, SiLU(gate) * up (on the gate+up GEMM's own
    # FP16 output) in front of down; the attention output in front of O has no such producer here and keeps the
    # stand-alone quantizer.  Eight launches per step, as in `full_step`, but the producers' work is done as well.
    fused = None
    if M <= 128:
        gamma = (1.0 + 0.1 * torch.randn(4096, generator=torch.Generator().manual_seed(5))).to(torch.float16).to(dev)
        K_of = dict((name, K) for name, (K, N) in layers)
        N_of = dict((name, N) for name, (K, N) in layers)
        assert N_of["gate_up"] == 2 * K_of["down"] and K_of["qkv"] == K_of["gate_up"] == gamma.numel()

        def gemm(name, step, s):
            b = bufs[name]
            check(L.qoq_w4a8_gemm(P(b["qx"]), P(b["sx"]), None, P(blobs[name][step % args.copies]), M, N_of[name],
                                  K_of[name], 0, P(b["out"]), P(b["ws"]), b["ws"].numel(), s))

        def fused_step(step, s=None):
            s = sp if s is None else s
            for name in ("qkv", "gate_up"):
                b = bufs[name]
                check(L.qoq_rmsnorm_quant(P(xs[name]), P(gamma), 1e-5, M, K_of[name], None, P(b["qx"]), P(b["sx"]),
                                          None, None, s))
                gemm(name, step, s)
            b = bufs["o"]
            check(L.qoq_quant_act_per_token(P(xs["o"]), M, K_of["o"], P(b["qx"]), P(b["sx"]), None, None, s))
            gemm("o", step, s)
            b = bufs["down"]
            check(L.qoq_silu_mul_quant(P(bufs["gate_up"]["out"]), M, K_of["down"], None, P(b["qx"]), P(b["sx"]),
                                       None, None, s))
            gemm("down", step, s)

        ms_fused = timed(fused_step, args.steps, min(args.warmup, 5))
        fused = {"step": "qoq_rmsnorm_quant + QKV GEMM, qoq_quant_act_per_token + O GEMM, qoq_rmsnorm_quant + gate+up GEMM, "
                         "qoq_silu_mul_quant (on the gate+up output) + down GEMM",
                 "ms_per_step": round(ms_fused, 5),
                 "value": round(sum(2.0 * M * K * N for _, (K, N) in layers) / (ms_fused * 1e-3) / 1e12, 3), "unit": "TOPS"}

    # What a plain read reaches in the same launch regime: the simplest streaming kernel over the same packed
    # weights (same rotation, same graph replay), best of four grid sizes.  Context for `frac`, which stays
    # measured against the published peak.
    probe = load_read_probe()
    sink = torch.zeros(65536, dtype=torch.int32, device=dev)
    floor = None
    for nwg in (256, 512, 1024, 2048):
        def read_step(step, s=None, nwg=nwg):
            s = sp if s is None else s
            for name, _ in layers:
                blob = blobs[name][step % args.copies]
                if probe.qoq_probe_read(P(blob), blob.numel() // 16 * 16, P(sink), nwg, s) != 0:
                    raise RuntimeError("qoq_probe_read refused its arguments")
        ms = timed(read_step, args.steps, min(args.warmup, 3))
        if floor is None or ms < floor[0]:
            floor = (ms, nwg)
    read_bytes = sum(blobs[name][0].numel() // 16 * 16 for name, _ in layers)

    ops = sum(2.0 * M * K * N for _, (K, N) in layers)
    byts = sum(algorithmic_bytes(M, N, K) for _, (K, N) in layers)
    tops = ops / (ms_step * 1e-3) / 1e12
    gemm_gbs = byts / (ms_gemm * 1e-3) / 1e9
    gemm_tops = ops / (ms_gemm * 1e-3) / 1e12

    workload = ("llama2_7b_decode_m%d" if M <= 128 else "llama2_7b_prefill_m%d") % M
    picked = {name: api.query_gemm_config(M, N, K, 0) for name, (K, N) in layers}
    config_now = ",".join("%s=%d/%d" % (name, picked[name][0], picked[name][1]) for name, _ in layers)
    traffic, traffic_src = profile_traffic(workload, config_now)

    # The GEMM launch is bound by HBM at decode sizes and by the INT8 matrix cores once there are a few hundred
    # tokens (ridge of the published peaks: 629 ops per byte, i.e. about 160 tokens for 4-bit weights).
    if M <= 128:
        roofline = {"bound": "hbm", "achieved": round(gemm_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(gemm_gbs / HBM_PEAK_GBS, 4),
                    "traffic": traffic, "traffic_source": traffic_src}
    else:
        roofline = {"bound": "mfma", "achieved": round(gemm_tops, 1), "peak": INT8_PEAK_TOPS, "unit": "TOP/s",
                    "frac": round(gemm_tops / INT8_PEAK_TOPS, 4), "traffic": None}
    roofline.update({"kernel": "qoq_w4a8_gemm launch (average over the four layers)",
                     "avg_launch_us": round(ms_gemm * 1e3 / len(layers), 3),
                     "algorithmic_bytes_per_launch": round(byts / len(layers)),
                     "algorithmic_ops_per_launch": round(ops / len(layers)),
                     "gemm_only_tops": round(gemm_tops, 3), "gemm_only_gbs": round(gemm_gbs, 1),
                     "int8_mfma_frac": round(gemm_tops / INT8_PEAK_TOPS, 4),
                     "hbm_frac": round(gemm_gbs / HBM_PEAK_GBS, 4),
                     "read_floor": {
                         "kernel": "plain streaming read of the same packed weights, one launch per layer, same "
                                   "rotation and graph replay (best of 256/512/1024/2048 workgroups)",
                         "workgroups": floor[1], "avg_launch_us": round(floor[0] * 1e3 / len(layers), 3),
                         "bytes_per_launch": read_bytes // len(layers),
                         "gbs": round(read_bytes / (floor[0] * 1e-3) / 1e9, 1),
                         "frac_of_peak": round(read_bytes / (floor[0] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)},
                     "gemm_time_over_read_floor": round(ms_gemm / floor[0], 3)})

    result = {
        "metric": "W4A8 GEMM effective TOPS (Llama-2-7B-shaped layers, M=%d, g128)" % M,
        "value": round(tops, 3), "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "data": "synthetic",
        "config": {"workload": workload, "layers": {n: {"K": k, "N": nn} for n, (k, nn) in layers},
                   "M": M, "group": 128, "mode": "group128", "weight_copies_rotated": args.copies,
                   "gemm_config": config_now,
                   "step": "4 x qoq_w4a8_linear (per-token activation quantization + W4A8 GEMM), launches replayed from a HIP graph"},
        "roofline": roofline,
    }

    if fused is not None:
        result["fused_producer_step"] = fused
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(M, xs, wl)

    if M == 64 and not args.no_compute_leg:
        # second half of the target: the compute-bound side, on the largest configuration (its own fields; `value`,
        # `ms_per_step` and `roofline` above stay those of the decode workload)
        del blobs, bufs, xs
        torch.cuda.empty_cache()
        leg = compute_leg(args, api, wl, dev)
        result["compute_leg"] = leg
        result["config"]["workload"] = workload + " (value, roofline) + " + leg["workload"] + " (compute_leg)"

    if args.sweep:
        sweep(args.sweep, api, wl, dev)

    print(json.dumps(result))


def compute_leg(args, api, wl, dev, family="llama3_70b", M=2048):
    """The compute-bound half of the target on the largest single-GPU configuration: the four Llama-3-70B-shaped
    layers at M = 2048 tokens (g128), one step = 4 x (activation quantization + W4A8 GEMM) like the decode
    workload.  The 429 MB of packed weights of the four layers exceed the 256 MB Infinity Cache, so every layer's
    weights come from HBM without rotating copies.  Reports the step and the GEMM launches alone against the
    published INT8 matrix-core peak."""
    import torch

    shapes = {"llama3_70b": wl.LLAMA3_70B, "llama2_7b": wl.LLAMA2_7B}[family]
    layers = list(shapes.items())
    L = api.lib()
    P = lambda t: t.data_ptr()
    st = {}
    for name, (K, N) in layers:
        w = wl.layer_weights(family, name, 3, dev)
        blob = api.pack_weights(w)
        del w
        st[name] = dict(blob=blob, x=wl.layer_activations(family, name, M, 3, dev),
                        qx=torch.empty((M, K), dtype=torch.int8, device=dev),
                        sx=torch.empty(M, dtype=torch.float16, device=dev),
                        out=torch.empty((M, N), dtype=torch.float16, device=dev),
                        ws=api.new_workspace(api.gemm_workspace_bytes(M, N, K), dev))
    torch.cuda.empty_cache()

    def check(rc):
        if rc != 0:
            raise RuntimeError(api.status_string(rc))

    def full_step(s):
        for name, (K, N) in layers:
            b = st[name]
            check(L.qoq_w4a8_linear(P(b["x"]), P(b["blob"]), M, N, K, 0, P(b["out"]), P(b["qx"]), P(b["sx"]), None,
                                    P(b["ws"]), b["ws"].numel(), s))

    def gemm_only(s):
        for name, (K, N) in layers:
            b = st[name]
            check(L.qoq_w4a8_gemm(P(b["qx"]), P(b["sx"]), None, P(b["blob"]), M, N, K, 0, P(b["out"]), P(b["ws"]),
                                  b["ws"].numel(), s))

    steps = max(1, min(args.steps, 20))
    warm = max(1, min(args.warmup, 3))

    def timed(fn):
        for _ in range(warm):
            fn(torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            fn(torch.cuda.current_stream().cuda_stream)
        g.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / steps

    ms_step = timed(full_step)
    ms_gemm = timed(gemm_only)
    ops = sum(2.0 * M * K * N for _, (K, N) in layers)
    byts = sum(algorithmic_bytes(M, N, K) for _, (K, N) in layers)
    gemm_tops = ops / (ms_gemm * 1e-3) / 1e12
    cfg = ",".join("%s=%d/%d" % ((name,) + tuple(api.query_gemm_config(M, N, K, 0))) for name, (K, N) in layers)
    return {"workload": "%s_prefill_m%d" % (family, M), "metric": "W4A8 GEMM effective TOPS", "unit": "TOPS",
            "value": round(ops / (ms_step * 1e-3) / 1e12, 3), "ms_per_step": round(ms_step, 5), "steps": steps, "warmup": warm,
            "layers": {n: {"K": k, "N": nn} for n, (k, nn) in layers}, "M": M, "gemm_config": cfg,
            "step": "4 x qoq_w4a8_linear (per-token activation quantization + W4A8 GEMM), launches replayed from a HIP graph",
            "roofline": {"bound": "mfma", "achieved": round(gemm_tops, 1), "peak": INT8_PEAK_TOPS, "unit": "TOP/s",
                         "frac": round(gemm_tops / INT8_PEAK_TOPS, 4), "traffic": None,
                         "kernel": "qoq_w4a8_gemm launch (average over the four layers)",
                         "avg_launch_us": round(ms_gemm * 1e3 / len(layers), 3),
                         "algorithmic_ops_per_launch": round(ops / len(layers)),
                         "algorithmic_bytes_per_launch": round(byts / len(layers)),
                         "mfma_ceiling": mfma_ceiling(dev)}}


def attention_bench(args, api, wl, dev):
    """KV4 decode attention: one new token for each of 64 sequences with `--seq` cached tokens (the shape of the
    paper's attention latency table, Section 5.3), heads of `--family`.  Four independently filled caches are
    rotated so that every call reads its cache from HBM.  One step = one qoq_kv4_attention_decode call."""
    import numpy as np
    import torch

    cfg = wl.KV4_DECODE[args.family]
    B, S, H, Hkv, D = args.batch, args.seq, cfg["H"], cfg["Hkv"], cfg["D"]
    k, v = wl.make_kv(B, Hkv, S, D, 7, dev)
    q = wl.make_queries(B, H, D, 7, dev)
    kt, vt = k.permute(0, 2, 1, 3).contiguous(), v.permute(0, 2, 1, 3).contiguous()
    zero = torch.zeros(B, dtype=torch.int32, device=dev)
    n_caches = 4
    caches = []
    for _ in range(n_caches):
        c = api.kv4_new_cache(B, Hkv, S, dev)
        api.kv4_append(c, kt, vt, zero, S)
        caches.append(c)
    del kt, vt
    seq = torch.full((B,), S, dtype=torch.int32, device=dev)
    out = torch.empty((B, H, D), dtype=torch.float16, device=dev)
    L = api.lib()

    # scratch for the split variant (grouped-query shapes with few (sequence, KV head) pairs); 0 bytes = single pass
    ws = torch.empty(max(16, api.kv4_attention_workspace_bytes(B, H, Hkv, S)), dtype=torch.uint8, device=dev)

    def call(i, s):
        rc = L.qoq_kv4_attention_decode_split(q.data_ptr(), caches[i % n_caches].data_ptr(), seq.data_ptr(), B, H, Hkv, D, S,
                                              out.data_ptr(), ws.data_ptr(), ws.numel(), s)
        if rc != 0:
            raise RuntimeError(api.status_string(rc))

    sp = torch.cuda.current_stream().cuda_stream
    for i in range(args.warmup):
        call(i, sp)
    torch.cuda.synchronize()
    per_graph = 10 * n_caches                    # enough launches per replay that the replay's own start-up does not show
    steps = max(1, args.steps // per_graph) * per_graph
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        cs = torch.cuda.current_stream().cuda_stream
        for i in range(per_graph):
            call(i, cs)
    graph.replay()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps // per_graph):
        graph.replay()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    # bytes one call must move: codes and (scale, zero) pairs of keys and values of every cached token, q, out
    byts = B * Hkv * S * (2 * (D // 2) + 2 * 4) + 2 * B * H * D * 2
    gbs = byts / (ms * 1e-3) / 1e9
    result = {
        "metric": "KV4 decode attention time per call (64 sequences x %d cached tokens)" % S,
        "value": round(ms, 5), "unit": "ms", "n_gpus": 1, "steps": steps, "warmup": args.warmup, "ms_per_step": round(ms, 5),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": "%s_kv4_decode_b%d_s%d" % (args.family, B, S), "B": B, "S": S, "H": H, "Hkv": Hkv, "D": D,
                   "caches_rotated": n_caches, "step": "1 x qoq_kv4_attention_decode_split, launches replayed from a HIP graph",
                   "sequence_ranges": max(1, api.kv4_attention_workspace_bytes(B, H, Hkv, S) // (B * H * 130 * 4)),
                   "paper_context": "0.28 ms on A100 for 64 x 1024 (its heads are not stated); another machine, not a target"},
        "roofline": {"bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(gbs / HBM_PEAK_GBS, 4),
                     # from the counter runs summarised in profiles/kv4_decode_attention_llama2_7b_b64_s1024.txt
                     "traffic": 286.52e6 if (S == 1024 and args.family == "llama2_7b") else None,
                     "kernel": "kv4_decode_kernel", "avg_launch_us": round(ms * 1e3, 3), "algorithmic_bytes_per_launch": byts},
    }
    if not args.no_cpu_baseline:
        from oracle import kv4
        picks = [(b, h) for b in range(0, B, 8) for h in range(0, H, 8)]
        t0 = time.perf_counter()
        done = 0
        for b, h in picks:
            hk = h // (H // Hkv)
            kc, ks, kz = kv4.kv4_quantize(k[b:b + 1, hk:hk + 1].cpu().numpy())
            vc, vs, vz = kv4.kv4_quantize(v[b:b + 1, hk:hk + 1].cpu().numpy())
            t1 = time.perf_counter()
            kv4.attention_decode(q[b:b + 1, h:h + 1].cpu().numpy(), kc, ks, kz, vc, vs, vz, np.array([S]))
            done += 1
            if time.perf_counter() - t0 > 12.0:
                break
        dt = time.perf_counter() - t0
        result["cpu_baseline"] = {"value": round(dt / done * B * H * 1e3, 3), "unit": "ms", "cores": 1, "kind": "oracle",
                                  "sample": "%d of %d (sequence, head) pairs incl. their cache quantization, scaled to all pairs (%.1f s)"
                                            % (done, B * H, dt)}
    return result


def producers_bench(args, api, wl, dev):
    """The producers with the per-token quantizer fused in (Section 5.1): RMSNorm in front of the QKV / first FFN
    projection (K = 4096) and SiLU(gate) * up in front of the second FFN projection (K = 11008), Llama-2-7B widths,
    --m tokens.  One step = one qoq_rmsnorm_quant + one qoq_silu_mul_quant call (FP16 activations not written: the
    fused path's point), over six rotated inputs so that every call reads its input from HBM.  The stand-alone
    quantizer is timed on the same shapes for comparison."""
    import numpy as np
    import torch

    M = args.m
    K1, K2 = 4096, 11008
    n_in = 6
    xs = [wl.make_activations(M, K1, 100 + i, dev) for i in range(n_in)]
    gus = [wl.make_activations(M, 2 * K2, 200 + i, dev) for i in range(n_in)]
    ys = [wl.make_activations(M, K2, 300 + i, dev) for i in range(n_in)]
    gamma = (1.0 + 0.1 * torch.randn(K1, generator=torch.Generator().manual_seed(5))).to(torch.float16).to(dev)
    q1 = torch.empty((M, K1), dtype=torch.int8, device=dev)
    q2 = torch.empty((M, K2), dtype=torch.int8, device=dev)
    sx = torch.empty(M, dtype=torch.float16, device=dev)
    L = api.lib()

    def check(rc):
        if rc != 0:
            raise RuntimeError(api.status_string(rc))

    def rms(i, s):
        check(L.qoq_rmsnorm_quant(xs[i % n_in].data_ptr(), gamma.data_ptr(), 1e-5, M, K1, None, q1.data_ptr(), sx.data_ptr(),
                                  None, None, s))

    def silu(i, s):
        check(L.qoq_silu_mul_quant(gus[i % n_in].data_ptr(), M, K2, None, q2.data_ptr(), sx.data_ptr(), None, None, s))

    def plain1(i, s):
        check(L.qoq_quant_act_per_token(xs[i % n_in].data_ptr(), M, K1, q1.data_ptr(), sx.data_ptr(), None, None, s))

    def plain2(i, s):
        check(L.qoq_quant_act_per_token(ys[i % n_in].data_ptr(), M, K2, q2.data_ptr(), sx.data_ptr(), None, None, s))

    def timed(fns, steps):
        for i in range(args.warmup):
            for fn in fns:
                fn(i, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        per_graph = 2 * n_in
        steps = max(1, steps // per_graph) * per_graph
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            cs = torch.cuda.current_stream().cuda_stream
            for i in range(per_graph):
                for fn in fns:
                    fn(i, cs)
        graph.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps // per_graph):
            graph.replay()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / steps, steps

    ms, steps = timed([rms, silu], args.steps)
    us_rms = timed([rms], args.steps)[0] * 1e3
    us_silu = timed([silu], args.steps)[0] * 1e3
    us_p1 = timed([plain1], args.steps)[0] * 1e3
    us_p2 = timed([plain2], args.steps)[0] * 1e3
    # algorithmic bytes: FP16 in (gate and up for SiLU), INT8 codes out, gamma once, one scale per token
    b_rms = M * K1 * 3 + 2 * K1 + 2 * M
    b_silu = M * K2 * 5 + 2 * M
    byts = b_rms + b_silu
    gbs = byts / (ms * 1e-3) / 1e9
    elems = M * (K1 + K2)
    result = {
        "metric": "fused producer throughput (RMSNorm+quant K=4096, SiLU*up+quant K=11008, M=%d)" % M,
        "value": round(elems / (ms * 1e-3) / 1e9, 3), "unit": "G elements/s", "n_gpus": 1, "steps": steps, "warmup": args.warmup,
        "ms_per_step": round(ms, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f64",
        "data": "synthetic",
        "config": {"workload": "llama2_7b_fused_producers_m%d" % M, "M": M, "K_rmsnorm": K1, "K_silu_mul": K2,
                   "inputs_rotated": n_in, "y_written": False,
                   "step": "1 x qoq_rmsnorm_quant + 1 x qoq_silu_mul_quant, launches replayed from a HIP graph"},
        "roofline": {"bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": None,
                     "kernel": "rmsnorm_quant_kernel + silu_mul_quant_kernel", "avg_launch_us": round(ms * 1e3 / 2, 3),
                     "algorithmic_bytes_per_launch": byts // 2,
                     "rmsnorm_us": round(us_rms, 2), "rmsnorm_gbs": round(b_rms / us_rms / 1e3, 1),
                     "silu_mul_us": round(us_silu, 2), "silu_mul_gbs": round(b_silu / us_silu / 1e3, 1),
                     "plain_quant_us": {"K4096": round(us_p1, 2), "K11008": round(us_p2, 2)}},
    }
    if not args.no_cpu_baseline:
        from oracle import qoq_quant as qq
        rows = min(M, 64)
        xn = xs[0][:rows].cpu().numpy()
        gn = gus[0][:rows].cpu().numpy()
        t0 = time.perf_counter()
        reps = 0
        while time.perf_counter() - t0 < 10.0:
            qq.act_quant(qq.rmsnorm_fp16(xn, gamma.cpu().numpy(), 1e-5))
            qq.act_quant(qq.silu_mul_fp16(gn))
            reps += 1
        dt = time.perf_counter() - t0
        result["cpu_baseline"] = {"value": round(reps * rows * (K1 + K2) / dt / 1e9, 4), "unit": "G elements/s", "cores": 1,
                                  "kind": "oracle", "sample": "%d tokens of both producers, %d passes (%.1f s)" % (rows, reps, dt)}
    return result


def ablation_bench(args, api, wl, dev):
    """(1) What the level-2 dequantization costs in the main loop (the paper's dequantization-overhead ablation,
    Section 6.4): the same layers and M through the g128 kernels (unpack + multiply-add + sign flip per operand) and
    through the per-channel kernels (unpack only; the zero point moves to the epilogue) -- the difference is the
    overhead.  (2) Run-time cost of the channel reordering (gather fused into the activation quantizer) and the
    speed of the offline Hadamard rotation."""
    import torch

    def timed(fn, reps):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for _ in range(reps):
                fn()
        g.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        g.replay()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / reps          # us

    M = args.m if args.m != 64 else 4096
    rows = {}
    tot = [0.0, 0.0]
    for name, (K, N) in wl.LLAMA2_7B.items():
        w = wl.layer_weights("llama2_7b", name, 1, dev)
        x = wl.layer_activations("llama2_7b", name, M, 1, dev)
        qx, sx, rowsum, _ = api.quant_act_per_token(x)
        out = torch.empty((M, N), dtype=torch.float16, device=dev)
        us = []
        for mode in (0, 1):
            blob = api.pack_weights(w, mode)
            ws = api.new_workspace(api.gemm_workspace_bytes(M, N, K, mode), dev)
            us.append(timed(lambda: api.w4a8_gemm(qx, sx, blob, N, mode, rowsum=rowsum, out=out, workspace=ws), 10))
            del blob
        rows[name] = {"g128_us": round(us[0], 2), "per_channel_us": round(us[1], 2), "overhead": round(us[0] / us[1] - 1, 4)}
        tot[0] += us[0]; tot[1] += us[1]
        del w, x
    overhead = tot[0] / tot[1] - 1
    # transforms
    K, N = wl.LLAMA2_7B["gate_up"]
    tr = {}
    for m in (64, 4096):
        x = wl.layer_activations("llama2_7b", "gate_up", m, 1, dev)
        perm = api.channel_order(api.channel_absmax(x))
        L = api.lib()
        qx = torch.empty((m, K), dtype=torch.int8, device=dev); sx = torch.empty(m, dtype=torch.float16, device=dev)
        s = torch.cuda.current_stream
        plain = timed(lambda: L.qoq_quant_act_per_token(x.data_ptr(), m, K, qx.data_ptr(), sx.data_ptr(), None, None, s().cuda_stream), 20)
        reord = timed(lambda: L.qoq_quant_act_per_token_reordered(x.data_ptr(), perm.data_ptr(), m, K, qx.data_ptr(), sx.data_ptr(), None, None, s().cuda_stream), 20)
        tr["act_quant_m%d" % m] = {"plain_us": round(plain, 2), "reordered_us": round(reord, 2)}
    w = wl.layer_weights("llama2_7b", "gate_up", 1, dev)
    out = torch.empty_like(w)
    us = timed(lambda: api.hadamard_rotate(w, K, out=out), 5)
    tr["hadamard_rotate_%dx%d" % (N, K)] = {"us": round(us, 1), "gbs": round(4.0 * N * K / us / 1e3, 1)}
    return {"metric": "level-2 dequantization overhead of the W4A8 g128 main loop (Llama-2-7B layers, M=%d)" % M,
            "value": round(100.0 * overhead, 2), "unit": "%", "n_gpus": 1, "steps": 10, "warmup": 3,
            "ms_per_step": round(tot[0] * 1e-3, 5), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
            "dtype": "int8", "data": "synthetic",
            "config": {"workload": "llama2_7b_dequant_ablation_m%d" % M, "M": M,
                       "ablation": "g128 kernels vs per-channel kernels (no level-2 multiply-add in the loop), GEMM launches only"},
            "layers": rows, "transforms": tr}


def cpu_baseline(M, xs, wl, budget_s=12.0):
    """The CPU oracle as it stands on the same workload: whole steps (all four layers at the same M: activation
    quantization + INT8 GEMM in int64 + FP64 epilogue) repeated until about `budget_s` seconds of wall time have
    been spent; weights are quantized by the oracle beforehand, untimed, like the offline packing.  For large M
    a step is cut down to the first tokens so that one pass stays within the budget."""
    import numpy as np

    from oracle import gemm as ogemm
    from oracle import qoq_quant as qq

    Ms = min(M, 256)                                  # bounded sample of the tokens for prefill-sized runs
    prepared = []
    for name, (K, N) in wl.LLAMA2_7B.items():
        w = wl.layer_weights("llama2_7b", name, 1, "cuda:0").cpu().numpy()
        wq = qq.progressive_quant(w)
        prepared.append((name, K, N, np.ascontiguousarray(wq["w_hat"].astype(np.int8)), wq["s0"],
                         xs[name][:Ms].cpu().numpy()))
        del w, wq
    ogemm.gemm_i64(np.zeros((1, 128), np.int8), np.zeros((1, 128), np.int8))   # load the library
    t0 = time.perf_counter()
    ops = 0.0
    passes = 0
    while True:
        for name, K, N, w_hat, s0, x in prepared:
            qx, sx, _, _ = qq.act_quant(x)
            acc = ogemm.gemm_i64(qx, w_hat)
            qq.output_fp16(acc, sx, s0)
            ops += 2.0 * Ms * K * N
        passes += 1
        dt = time.perf_counter() - t0
        if dt >= budget_s or passes >= 1000:
            break
    return {"value": round(ops / dt / 1e12, 6), "unit": "TOPS", "cores": ogemm.num_threads(), "kind": "oracle",
            "sample": "all four layers at M=%d, %d passes (%.1f s)" % (Ms, passes, dt)}


def sweep(path, api, wl, dev):
    """Per-layer timings over M for the three layer families (GEMM launch only, rotated copies)."""
    import torch
    rows = []
    fams = [("llama2_7b", wl.LLAMA2_7B, 0, (1, 8, 32, 64, 128, 256, 512, 1024, 2048, 4096)),
            ("llama3_70b", wl.LLAMA3_70B, 0, (512, 2048)),
            ("llama3_8b", wl.LLAMA3_8B, 1, (64, 1024))]
    stream = torch.cuda.current_stream()
    for fam, shapes, mode, ms in fams:
        for name, (K, N) in shapes.items():
            w = wl.layer_weights(fam, name, 2, dev)
            blob0 = api.pack_weights(w, mode)
            del w
            copies = max(2, -(-640_000_000 // blob0.numel()))   # rotate at least 640 MB: past L2 and Infinity Cache
            blobs = [blob0] + [blob0.clone() for _ in range(copies - 1)]
            # what a plain streaming read of the same packed weights takes in the same regime (graph replay, rotated
            # copies): the practical floor of the memory-bound rows of this layer
            probe = load_read_probe()
            sink = torch.zeros(65536, dtype=torch.int32, device=dev)
            read_us = 1e9
            for nwg in (256, 512):
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph):
                    cs = torch.cuda.current_stream().cuda_stream
                    for i in range(max(copies, 16)):
                        b = blobs[i % copies]
                        if probe.qoq_probe_read(b.data_ptr(), b.numel() // 16 * 16, sink.data_ptr(), nwg, cs) != 0:
                            raise RuntimeError("qoq_probe_read refused its arguments")
                graph.replay()
                torch.cuda.synchronize()
                for _ in range(3):
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                    graph.replay()
                    e1.record()
                    torch.cuda.synchronize()
                    read_us = min(read_us, e0.elapsed_time(e1) * 1e3 / max(copies, 16))
                del graph
            for M in ms:
                x = wl.layer_activations(fam, name, M, 2, dev)
                qx, sx, rowsum, _ = api.quant_act_per_token(x)
                out = torch.empty((M, N), dtype=torch.float16, device=dev)
                ws = api.new_workspace(api.gemm_workspace_bytes(M, N, K, mode), dev)
                reps = max(copies, 16 if M >= 1024 else 48)
                for i in range(3):
                    api.w4a8_gemm(qx, sx, blobs[i % copies], N, mode, rowsum=rowsum, out=out, workspace=ws)
                torch.cuda.synchronize()

                def timed(n_copies):
                    graph = torch.cuda.CUDAGraph()      # launches replayed from a graph, like the main measurement
                    with torch.cuda.graph(graph):
                        for i in range(reps):
                            api.w4a8_gemm(qx, sx, blobs[i % n_copies], N, mode, rowsum=rowsum, out=out, workspace=ws)
                    graph.replay()
                    torch.cuda.synchronize()
                    best = 1e9
                    for _ in range(3):
                        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                        e0.record()
                        graph.replay()
                        e1.record()
                        torch.cuda.synchronize()
                        best = min(best, e0.elapsed_time(e1) * 1e3 / reps)
                    del graph
                    return best

                us = timed(copies)                      # HBM-cold: rotated copies
                us_hot = timed(1)                       # cache-hot: the same weights every launch
                ops = 2.0 * M * K * N
                byts = algorithmic_bytes(M, N, K, mode)
                # roofline for this shape: the lower of the matrix-core peak and intensity x HBM peak
                roof = min(INT8_PEAK_TOPS, ops / byts * HBM_PEAK_GBS / 1e3)
                rows.append({"family": fam, "layer": name, "mode": mode, "M": M, "K": K, "N": N, "us": round(us, 2),
                             "tops": round(ops / us / 1e6, 2), "mfma_frac": round(ops / us / 1e6 / INT8_PEAK_TOPS, 4),
                             "gbs": round(byts / us / 1e3, 1), "hbm_frac": round(byts / us / 1e3 / HBM_PEAK_GBS, 4),
                             "roof_tops": round(roof, 1), "roof_frac": round(ops / us / 1e6 / roof, 4),
                             "us_cache_hot": round(us_hot, 2), "weights_read_us": round(read_us, 2)})
                del x, qx, sx, out, ws
            del blobs, blob0
            torch.cuda.empty_cache()
    os.makedirs(os.path.dirname(os.path.abspath(path)), exist_ok=True)
    with open(path, "w") as f:
        for r in rows:
            f.write(json.dumps(r) + "\n")
    with open(path + ".txt", "w") as f:               # the same rows as a table
        f.write("%-10s %-8s %4s %5s %6s %6s %9s %8s %6s %8s %6s %8s %6s %9s %9s\n" % (
            "family", "layer", "mode", "M", "K", "N", "us", "TOP/s", "mfma", "GB/s", "hbm", "roof", "frac", "us(hot)", "read(us)"))
        for r in rows:
            f.write("%-10s %-8s %4d %5d %6d %6d %9.2f %8.1f %6.3f %8.1f %6.3f %8.1f %6.3f %9.2f %9.2f\n" % (
                r["family"], r["layer"], r["mode"], r["M"], r["K"], r["N"], r["us"], r["tops"], r["mfma_frac"],
                r["gbs"], r["hbm_frac"], r["roof_tops"], r["roof_frac"], r["us_cache_hot"], r["weights_read_us"]))


if __name__ == "__main__":
    main()
