#!/usr/bin/env python3
"""Benchmark of the LRQ-DiT quantized-linear hot path on one MI355X.

A "step" is one pass of the whole runtime path (lrq_qlinear = rotate + per-token quantize + TLQ
decode + int8 MFMA GEMM + rescale) over every linear of the chosen workload, inputs resident in HBM.
Weight calibration/packing (lrq_tlq_quantize_pack) is the offline step; it is timed once and reported
beside the step, not inside it.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c1|c2|c3|c4|c5] [--no-cpu-baseline]
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

INT8_MFMA_PEAK_TOPS = 5000.0     # MI355X dense int8 matrix peak
BF16_MFMA_PEAK_TFLOPS = 2500.0   # MI355X dense bf16 matrix peak (the --levels path)
HBM_PEAK_GBS = 8000.0            # MI355X HBM3E peak
FP64_VEC_PEAK_TFLOPS = 78.6


class Probes:
    """The benchmark's own measurement kernels (libbench_probes.so, built next to liblrq.so): a pure int8 MFMA loop
    and a plain device copy, timed with events."""

    def __init__(self):
        import ctypes
        from paper_2508_03485_amd.build import PROBES
        if not os.path.exists(PROBES):
            raise ImportError(f"{PROBES} is not built: run `python -m paper_2508_03485_amd.build`")
        self.L = ctypes.CDLL(PROBES)
        vp, ci = ctypes.c_void_p, ctypes.c_int
        self.L.bench_probe_mfma_i8.restype = ci
        self.L.bench_probe_mfma_i8.argtypes = [vp, ci, ci, ci, vp, ctypes.POINTER(ctypes.c_double)]
        self.L.bench_probe_copy.restype = ci
        self.L.bench_probe_copy.argtypes = [vp, vp, vp, ctypes.c_size_t]

    def launch_mfma(self, blocks, iters, pattern, out, ops=None):
        import torch
        rc = self.L.bench_probe_mfma_i8(torch.cuda.current_stream().cuda_stream, blocks, iters, pattern, out.data_ptr(), ops)
        assert rc == 0

    def mfma_i8_tops(self, pattern=1, blocks=2048, iters=4096, reps=5):
        """Sustained int8 MFMA rate in TOP/s; pattern 0 = constant operands, 1 = pseudo-random operands (16x16x64, the
        GEMM's instruction); 2, 3 = the same with the 32x32x32 instruction."""
        import ctypes
        import torch
        out = torch.zeros(1, dtype=torch.int32, device="cuda")
        ops = ctypes.c_double(0.0)
        self.launch_mfma(blocks, iters, pattern, out, ctypes.byref(ops))
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            self.launch_mfma(blocks, iters, pattern, out)
        b.record()
        torch.cuda.synchronize()
        return ops.value * reps / (a.elapsed_time(b) * 1e-3) / 1e12

    def copy_gbs(self, nbytes=1 << 30, reps=10):
        """Device copy bandwidth in GB/s counting read + written bytes."""
        import torch
        src = torch.empty(nbytes, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        st = torch.cuda.current_stream().cuda_stream
        assert self.L.bench_probe_copy(st, src.data_ptr(), dst.data_ptr(), nbytes) == 0
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            self.L.bench_probe_copy(st, src.data_ptr(), dst.data_ptr(), nbytes)
        b.record()
        torch.cuda.synchronize()
        return 2.0 * nbytes * reps / (a.elapsed_time(b) * 1e-3) / 1e9


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0,
                    help="timed steps; 0 (default) = as many as fill about 0.6 s, found with a short pilot run "
                         "(the chip needs a few milliseconds of load to reach its steady clocks)")
    ap.add_argument("--warmup", type=int, default=-1, help="untimed warm-up steps; -1 (default) = a tenth of the timed steps")
    ap.add_argument("--workload", default="c4", choices=["c1", "c2", "c3", "c4", "c5"],
                    help="synthetic workload; the default is the largest configuration (config 4), the one the metric is quoted on")
    ap.add_argument("--blocks", type=int, default=0, help="c5 only: number of transformer blocks (0 = all 28)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--structured", type=int, default=0, metavar="B",
                    help="run the layers that take the dense outlier-aware rotation with its structured form "
                         "X.R1.P.R2 instead (block size B, seeded block rotations and permutation)")
    ap.add_argument("--no-prepared-rotation", action="store_true",
                    help="dense rotations: let every call derive R's transpose and statistics itself instead of handing over "
                         "the result of lrq_ars_dense_prepare (computed once, untimed, like the weight packing)")
    ap.add_argument("--clocks", action="store_true",
                    help="also sample the shader clock (rocm-smi) while single kernels run back to back for ~2 s each and "
                         "report it under 'sustained_clocks' (the int8 matrix peak scales with that clock)")
    ap.add_argument("--lower-clip", action="store_true",
                    help="calibrate the weights with the lower clip factor gamma (grid 1.00 .. 0.30 step 0.05) searched "
                         "jointly with alpha / beta (lrq_tlq_quantize_pack_clip)")
    ap.add_argument("--graph", action="store_true",
                    help="capture each step (all layers) in a HIP graph once and time the replays")
    ap.add_argument("--smooth", action="store_true",
                    help="give every layer a smoothing pre-scale (from lrq_smooth_factor on its own inputs), multiplied "
                         "into the activations inside the rotate+quantize kernels")
    ap.add_argument("--calibration", action="store_true",
                    help="also time the calibration-time entry points (J metric, smoothing factor, greedy rotation "
                         "builder) on the workload's first layer and report them under 'calibration'")
    ap.add_argument("--asym", action="store_true",
                    help="use the zero-point form of the activation quantizer (the paper's Eq. 1 as printed)")
    ap.add_argument("--levels", action="store_true",
                    help="run the GEMM on the TLQ levels themselves (lrq_qlinear_levels: bf16 matrix cores, the paper's value "
                         "map without the int8 level table) - the fidelity-reference path, priced against the bf16 peak")
    ap.add_argument("--packed4", action="store_true",
                    help="layers with 4-bit activations keep their codes two per byte between rotate+quantize and the GEMM "
                         "(lrq_qlinear_packed4)")
    ap.add_argument("--fp8", action="store_true",
                    help="layers with 4-bit activations run with FP8 E4M3 operands on both sides (lrq_qlinear_fp8: levels with "
                         "three mantissa bits, v_mfma_f32_32x32x64_f8f6f4)")
    ap.add_argument("--probes-only", action="store_true",
                    help="run only the pure-MFMA and copy probes (calibration of rocprofv3 byte counters)")
    ap.add_argument("--cpu-rows", type=int, default=16384, help="token rows per layer in the oracle sample")
    ap.add_argument("--cpu-channels", type=int, default=4608, help="output channels per layer in the oracle sample")
    ap.add_argument("--cache-bytes", type=int, default=768 << 20,
                    help="cycle through enough buffer copies that a step's working set exceeds this")
    args = ap.parse_args()
    if args.levels and args.asym:
        ap.error("--levels and --asym cannot be combined (the levels path has no zero-point form)")
    return args


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); --gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2508_03485_amd as lrq
    import synth

    if not os.path.exists(lrq.LIB_PATH):
        from paper_2508_03485_amd.build import build
        build()
    lrq.lib()
    probes = Probes()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.probes_only:
        print(json.dumps(dict(copy_gbs=round(probes.copy_gbs(1 << 30, 5), 1), copy_bytes_per_launch=1 << 30,
                              mfma_i8_tops_constant_operands=round(probes.mfma_i8_tops(0), 1),
                              mfma_i8_tops_random_operands=round(probes.mfma_i8_tops(1), 1),
                              mfma_i8_32x32x32_tops_random_operands=round(probes.mfma_i8_tops(3), 1))))
        return
    cfg = int(args.workload[1])
    specs = synth.config_layers(cfg)
    if cfg == 5 and args.blocks:
        specs = [s for s in specs if s.block < args.blocks]
    grid = torch.from_numpy(synth.DEFAULT_GRID).to(dev)
    gamma_grid = None
    if args.lower_clip:
        gamma_grid = torch.tensor([1.0 - 0.05 * i for i in range(15)], dtype=torch.float32, device=dev)

    # ---------------------------------------------------------------- inputs (seeded, synthetic), resident in HBM
    t_gen = time.time()
    layers = []
    shape_cache = {}
    pack_ms = 0.0
    prepare_ms = 0.0
    for s in specs:
        # config 5 re-uses one set of activations per distinct shape (seeded by the first block that has it): the
        # kernels' work does not depend on the values, and 140 separate 8192-token inputs would not fit the run time
        skey = (s.M, s.K, s.N, s.rotation) if cfg == 5 else s.key
        if skey not in shape_cache:
            Xb = synth.make_activations(s.M, s.K, s.key, s.p_mild, s.n_salient, s.gain)
            X = torch.from_numpy(Xb.view(np.int16)).to(dev).view(torch.bfloat16)
            W = torch.from_numpy(synth.make_weights(s.N, s.K, s.key)).to(dev)
            R = None
            if s.rotation == "dense" and args.structured:
                B = args.structured
                bf = lambda a: torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)
                R = lrq.Rotation("blockperm", block=B, R1=bf(synth.make_block_rotations(s.K, B, s.key, 0)),
                                 perm=torch.from_numpy(synth.make_channel_permutation(s.K, s.key)).to(dev),
                                 R2=bf(synth.make_block_rotations(s.K, B, s.key, 1)))
            elif s.rotation == "dense":
                R = torch.from_numpy(synth.make_rotation(s.K, s.key).view(np.int16)).to(dev).view(torch.bfloat16)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            w = lrq.tlq_quantize_pack(W, s.w_bits, 7, grid, grid, gamma_grid=gamma_grid)
            e1.record()
            torch.cuda.synchronize()
            pack_ms += e0.elapsed_time(e1)
            del W
            shape_cache[skey] = (X, w, R)
        X, w, R = shape_cache[skey]
        rot = R if isinstance(R, lrq.Rotation) else lrq.Rotation(s.rotation, s.had_block, R)
        if (rot.kind == "dense" and not args.no_prepared_rotation and not args.smooth and not args.asym and s.M > 64
                and lrq.lib().lrq_ars_dense_prepared_bytes(s.K) > 0):
            # offline like the weight packing: the rotation is fixed at calibration time, so is everything derived from it
            if ("prepared", skey) not in shape_cache:
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                shape_cache[("prepared", skey)] = lrq.ars_dense_prepare(R)
                e1.record()
                torch.cuda.synchronize()
                prepare_ms += e0.elapsed_time(e1)
            rot.prepared = shape_cache[("prepared", skey)]
        if args.smooth:
            if "inv" not in shape_cache.setdefault(("smooth", skey), {}):
                Wd = torch.from_numpy(synth.make_weights(s.N, s.K, s.key)).to(dev)
                shape_cache[("smooth", skey)]["inv"] = lrq.smooth_factor(X[:1024], Wd, 0.5, smooth_weights=False)[1]
                del Wd
            rot.prescale = shape_cache[("smooth", skey)]["inv"]
        layers.append(dict(spec=s, X=[X], w=w, rot=rot))
    gen_s = time.time() - t_gen

    # buffer copies so that consecutive steps do not find their inputs in the 256 MB Infinity Cache
    step_bytes = sum(l["spec"].M * l["spec"].K * 3 + l["spec"].M * l["spec"].N * 2 for l in layers)
    copies = max(1, min(8, math.ceil(args.cache_bytes / max(step_bytes, 1))))
    for l in layers:
        s = l["spec"]
        while len(l["X"]) < copies:
            l["X"].append(l["X"][0].clone())
        l["Y"] = [torch.empty((s.M, s.N), dtype=torch.bfloat16, device=dev) for _ in range(copies)]
        nws = lrq.workspace_bytes(s.M, s.N, s.K, l["rot"], s.a_bits, asym=args.asym)
        if args.packed4 and s.a_bits == 4:
            import ctypes
            nws = max(nws, lrq.lib().lrq_workspace_bytes_packed4(s.M, s.N, s.K, ctypes.byref(l["rot"].c_struct())))
        l["ws"] = [torch.empty(nws, dtype=torch.uint8, device=dev) for _ in range(copies)]
        l["q"] = [torch.empty((s.M, s.K), dtype=torch.int8, device=dev) for _ in range(copies)]
        l["sc"] = [torch.empty(s.M, dtype=torch.float32, device=dev) for _ in range(copies)]
        l["zr"] = [torch.empty(s.M, dtype=torch.int32, device=dev) for _ in range(copies)]
        na = lrq.ars_workspace_bytes(s.M, s.K, l["rot"], s.a_bits)
        l["aws"] = torch.empty(na, dtype=torch.uint8, device=dev) if na else None

    packed = args.packed4 and not (args.asym or args.levels or args.fp8)
    fp8 = args.fp8 and not (args.asym or args.levels)

    def step(i):
        c = i % copies
        for l in layers:
            if packed and l["spec"].a_bits == 4:
                lrq.qlinear_packed4(l["X"][c], l["rot"], l["w"], out=l["Y"][c], workspace=l["ws"][c])
            elif fp8 and l["spec"].a_bits == 4:
                lrq.qlinear_fp8(l["X"][c], l["rot"], l["w"], out=l["Y"][c], workspace=l["ws"][c])
            else:
                lrq.qlinear(l["X"][c], l["rot"], l["spec"].a_bits, l["w"], out=l["Y"][c], workspace=l["ws"][c], asym=args.asym,
                            levels=args.levels)

    if args.graph:
        eager_step = step
        eager_step(0)                       # one-time set-up (kernel attributes) outside the capture
        torch.cuda.synchronize()
        graphs = []
        for c in range(copies):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                eager_step(c)
            graphs.append(g)

        def step(i):                        # noqa: F811
            graphs[i % copies].replay()

    if args.steps <= 0:                     # pilot: size the timed region to about 0.6 s
        for i in range(3):
            step(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(10):
            step(3 + i)
        torch.cuda.synchronize()
        pilot = (time.perf_counter() - t0) / 10
        args.steps = int(min(4000, max(20, round(0.6 / pilot))))
    if args.warmup < 0:
        args.warmup = max(5, args.steps // 10)
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt * 1e3 / args.steps
    total_ops = sum(l["spec"].ops for l in layers)
    tops = total_ops / (ms_per_step * 1e-3) / 1e12
    # the same steps on one set of buffers (inputs, workspaces and outputs stay in the 256 MB Infinity Cache when the
    # working set is small): reported next to the rotated-buffer figure, which is the one in `value`
    hot = None
    if copies > 1:
        nh = max(20, args.steps // 4)
        for i in range(5):
            step(0)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(nh):
            step(0)
        torch.cuda.synchronize()
        hot_ms = (time.perf_counter() - t0) * 1e3 / nh
        hot = dict(ms_per_step=round(hot_ms, 4), value=round(total_ops / (hot_ms * 1e-3) / 1e12, 2), steps=nh,
                   note="same buffers every step (working set resident in the Infinity Cache); `value` rotates among "
                        "%d buffer sets" % copies)

    # ---------------------------------------------------------------- per-kernel durations (HIP events on the launch stream)
    ksteps = int(min(300, max(3, min(args.steps, round(0.25 / (ms_per_step * 1e-3))))))
    ev = []
    lead = torch.zeros(1, dtype=torch.int32, device=dev)
    for i in range(ksteps):
        # a ~0.5 ms lead-in kernel keeps the host ahead of the device, so that an interval between two events holds
        # one kernel and no host-side launch gap (short kernels would otherwise be timed at the host's launch rate)
        probes.launch_mfma(2048, 512, 1, lead)
        c = (args.warmup + args.steps + i) % copies
        for li, l in enumerate(layers):
            s = l["spec"]
            a, b, d = (torch.cuda.Event(enable_timing=True) for _ in range(3))
            a.record()
            if packed and s.a_bits == 4:
                q4 = l["q"][c].view(torch.uint8).view(-1)[:s.M * s.K // 2].view(s.M, s.K // 2)
                lrq.ars_rotate_quant_packed4(l["X"][c], l["rot"], q4=q4, scale=l["sc"][c], workspace=l["ws"][c])
                b.record()
                lrq.qgemm_packed4(q4, l["sc"][c], l["w"], out=l["Y"][c])
            elif fp8 and s.a_bits == 4:
                q8 = l["q"][c].view(torch.uint8)
                lrq.ars_rotate_quant_fp8(l["X"][c], l["rot"], q8=q8, scale=l["sc"][c], workspace=l["aws"])
                b.record()
                lrq.qgemm_fp8(q8, l["sc"][c], l["w"], out=l["Y"][c])
            else:
                lrq.ars_rotate_quant(l["X"][c], l["rot"], s.a_bits, q=l["q"][c], scale=l["sc"][c], workspace=l["aws"],
                                     asym=args.asym, zero=l["zr"][c] if args.asym else None)
                b.record()
                lrq.qgemm(l["q"][c], l["sc"][c], l["w"], out=l["Y"][c], zero=l["zr"][c] if args.asym else None,
                          levels=args.levels)
            d.record()
            ev.append((li, a, b, d))
    torch.cuda.synchronize()
    rot_ms = [0.0] * len(layers)
    gemm_ms = [0.0] * len(layers)
    for li, a, b, d in ev:
        rot_ms[li] += a.elapsed_time(b) / ksteps
        gemm_ms[li] += b.elapsed_time(d) / ksteps

    per_layer = []
    agg = {}
    for li, l in enumerate(layers):
        s = l["spec"]
        key = s.name.split(".")[-1] if cfg == 5 else s.name
        if cfg == 5 and s.rotation == "dense":
            key += "(dense)"
        rq_bytes = 3 * s.M * s.K + 4 * s.M
        e = agg.setdefault(key, dict(name=key, M=s.M, K=s.K, N=s.N, rotation=s.rotation, count=0, rot_ms=0.0,
                                     gemm_ms=0.0, ops=0, rq_bytes=0))
        e["count"] += 1
        e["rot_ms"] += rot_ms[li]
        e["gemm_ms"] += gemm_ms[li]
        e["ops"] += s.ops
        e["rq_bytes"] += rq_bytes
    for e in agg.values():
        e["gemm_tops"] = round(e["ops"] / (e["gemm_ms"] * 1e-3) / 1e12, 2) if e["gemm_ms"] > 0 else None
        e["rotate_quant_gbs"] = round(e["rq_bytes"] / (e["rot_ms"] * 1e-3) / 1e9, 1) if e["rot_ms"] > 0 else None
        e["rot_ms"] = round(e["rot_ms"], 4)
        e["gemm_ms"] = round(e["gemm_ms"], 4)
        del e["ops"], e["rq_bytes"]
        per_layer.append(e)

    # dominant kernel: the decode + MFMA GEMM.  Algorithmic ops per launch = 2*M*N*K.
    gemm_total_ms = sum(gemm_ms)
    gemm_tops = total_ops / (gemm_total_ms * 1e-3) / 1e12
    mfma_peak = BF16_MFMA_PEAK_TFLOPS if args.levels else INT8_MFMA_PEAK_TOPS      # the FP8 peak equals the int8 one (5.0 PFLOP/s)
    roofline = dict(bound="mfma", kernel=("qgemm_levels_kernel (decode + bf16 MFMA + rescale)" if args.levels else
                                          "qgemm_kernel (decode + int8 MFMA + rescale)"), achieved=round(gemm_tops, 2),
                    peak=mfma_peak, unit="TFLOP/s", frac=round(gemm_tops / mfma_peak, 4),
                    traffic=None, note="multiply-accumulates counted as 2 ops; averaged over the "
                    "workload's layers, %d launches each" % ksteps,
                    avg_launch_ms=round(gemm_total_ms / len(layers), 4))
    # Hadamard rotate+quantize: algorithmic bytes = 2 (bf16 in) + 1 (code out) per element + 4 per token
    had = [(li, l) for li, l in enumerate(layers) if l["spec"].rotation == "hadamard"]
    roofline_rq = None
    if had:
        b = sum(3 * l["spec"].M * l["spec"].K + 4 * l["spec"].M for _, l in had)
        t = sum(rot_ms[li] for li, _ in had)
        gbs = b / (t * 1e-3) / 1e9
        roofline_rq = dict(bound="hbm", kernel="hadamard rotate + quantize", achieved=round(gbs, 1), peak=HBM_PEAK_GBS,
                           unit="GB/s", frac=round(gbs / HBM_PEAK_GBS, 4), traffic=None,
                           avg_launch_ms=round(t / len(had), 4))

    # outlier-aware dense rotation + quantizer (whole lrq_ars_rotate_quant call of the layers that take it): the bulk
    # product runs on the bf16 matrix cores, algorithmic flops 2*M*K*K per launch
    dense = [(li, l) for li, l in enumerate(layers) if l["spec"].rotation == "dense" and not isinstance(l["rot"].R, type(None))
             and l["rot"].kind == "dense" and l["spec"].M > 64]
    roofline_dense = None
    if dense:
        fl = sum(2.0 * l["spec"].M * l["spec"].K * l["spec"].K for _, l in dense)
        t = sum(rot_ms[li] for li, _ in dense)
        tf = fl / (t * 1e-3) / 1e12
        roofline_dense = dict(bound="mfma", kernel="dense rotation + quantize (bf16 MFMA product in 32-k runs, fp32 group sums, "
                              "fp64 totals, error bound, exact recomputation of undecided elements)", achieved=round(tf, 2),
                              peak=BF16_MFMA_PEAK_TFLOPS, unit="TFLOP/s", frac=round(tf / BF16_MFMA_PEAK_TFLOPS, 4), traffic=None,
                              avg_launch_ms=round(t / len(dense), 4),
                              note="time of the whole call (seven kernels with R prepared offline, ten without), flops of the product alone")
        # what the error bound left undecided in the first such layer's last call, and how far the approximate product
        # really is from the fp64 evaluation (LRQ_ROT_DENSE_F64 leaves u in fp64 at the head of its workspace)
        l0 = dense[0][1]
        s0 = l0["spec"]
        rot64 = lrq.Rotation("dense_f64", 0, l0["rot"].R)
        ws64 = torch.empty(lrq.ars_workspace_bytes(s0.M, s0.K, rot64, s0.a_bits), dtype=torch.uint8, device=dev)
        lrq.ars_rotate_quant(l0["X"][0], rot64, s0.a_bits, workspace=ws64)
        lrq.ars_rotate_quant(l0["X"][0], l0["rot"], s0.a_bits, workspace=l0["aws"])
        torch.cuda.synchronize()
        ut, eps, cnt, whole = lrq.ars_dense_diagnostics(l0["aws"], s0.M, s0.K)
        u64 = ws64[:s0.M * s0.K * 8].view(torch.float64).view(s0.M, s0.K)
        ratio = 0.0
        for r0 in range(0, s0.M, 4096):           # in slabs: the difference in fp64 would double the footprint otherwise
            r1 = min(r0 + 4096, s0.M)
            ratio = max(ratio, float(((ut[r0:r1].double() - u64[r0:r1]).abs() / eps[r0:r1].view(-1, 1)).max().item()))
        roofline_dense["diagnostics"] = dict(layer=s0.name, undecided_fraction=round(float(cnt.sum().item()) / (s0.M * s0.K), 6),
                                             max_undecided_per_row=int(cnt.max().item()), rows_recomputed_whole=int(whole.sum().item()),
                                             max_error_over_bound=round(ratio, 4))
        del ws64, u64

    out = dict(metric="fused W-TLQ/A-ARS qlinear TOPS + % int8 MFMA peak; rotate+quant HBM GB/s",
               value=round(tops, 2), unit="TOPS", n_gpus=1, steps=args.steps, warmup=args.warmup,
               ms_per_step=round(ms_per_step, 4), higher_is_better=True, scaling="weak", vs_baseline=None,
               dtype="bf16" if args.levels else ("fp8" if args.fp8 else "int8"), data="synthetic",
               config=dict(workload={1: "config1: single 256x1152->1152 W4A8 Hadamard",
                                     2: "config2: PixArt-style block linears, 8192 tokens, hidden 1152, W4A8, Hadamard",
                                     3: "config3: FLUX-style block linears, 4608 tokens, hidden 3072, W4A4, Hadamard",
                                     4: "config4: video-DiT block linears, 35100 tokens, hidden 3072, W4A8, per-layer ARS",
                                     5: "config5: 28-block PixArt-style stack, W3A4, per-layer ARS"}[cfg],
                           layers=len(layers), ops_per_step=total_ops, buffer_copies=copies,
                           outlier_rotation=(f"structured R1.P.R2, block {args.structured}" if args.structured else "dense K x K"),
                           dense_rotation_prepared_offline=any(l["rot"].prepared is not None for l in layers),
                           smoothing_prescale=bool(args.smooth), hip_graph=bool(args.graph),
                           tlq_lower_clip=bool(args.lower_clip), packed_4bit_activation_codes=bool(args.packed4),
                           fp8_operands=bool(args.fp8),
                           activation_quantizer="zero-point (Eq. 1)" if args.asym else "symmetric absmax",
                           value_map="levels round(2^r 2^I) 2^(f-I) as bf16 operands" if args.levels else "per-channel int8 level table",
                           step=("lrq_qlinear_levels per layer: rotate + quantize + TLQ decode + bf16 MFMA GEMM + rescale, bf16 out" if args.levels else
                                 "lrq_qlinear per layer: rotate + quantize + TLQ decode + int8 MFMA GEMM + rescale, bf16 out")),
               roofline=roofline, roofline_rotate_quant=roofline_rq, roofline_dense_rotation=roofline_dense, per_layer=per_layer,
               offline=dict(tlq_quantize_pack_ms=round(pack_ms, 2), dense_prepare_ms=round(prepare_ms, 3),
                            input_generation_s=round(gen_s, 1)))

    if hot:
        out["hot_cache"] = hot
    if args.calibration:
        out["calibration"] = calibration_timings(lrq, layers[0], dev)
    if args.clocks:
        out["sustained_clocks"] = sustained_clocks(lrq, probes, max(layers, key=lambda l: l["spec"].ops), dev)

    # what this device sustains on a pure int8 MFMA loop and on a plain copy kernel (context for the published peaks)
    out["measured_ceilings"] = dict(mfma_i8_tops_constant_operands=round(probes.mfma_i8_tops(0), 1),
                                    mfma_i8_tops_random_operands=round(probes.mfma_i8_tops(1), 1),
                                    mfma_i8_32x32x32_tops_random_operands=round(probes.mfma_i8_tops(3), 1),
                                    copy_gbs=round(probes.copy_gbs(1 << 30, 5), 1),
                                    note="pure int8 MFMA loops, v_mfma_i32_16x16x64_i8 (the GEMM's instruction) unless named "
                                         "otherwise: operand toggling lowers the sustained clock, and the 32x32x32 shape "
                                         "sustains less; 1 GiB device copy, read + written bytes")
    traffic_file = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(traffic_file):
        tr = json.load(open(traffic_file)).get(args.workload)
        if tr:
            if not args.levels:
                out["roofline"]["traffic"] = tr.get("qgemm")
            if out["roofline_rotate_quant"]:
                out["roofline_rotate_quant"]["traffic"] = tr.get("rotate_quant")
            if out["roofline_dense_rotation"] and not args.structured:
                out["roofline_dense_rotation"]["traffic"] = tr.get("dense_rotation")
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(specs, args.cpu_rows, args.cpu_channels)
    print(json.dumps(out))


def sustained_clocks(lrq, probes, layer, dev):
    """Shader clock reported by `rocm-smi --showclocks` while one kernel runs back to back (about 2 s of queued
    launches, sampled after 1 s): the workload's largest GEMM on its real codes and on all-zero activation codes, the
    pure MFMA probe with pseudo-random and with constant operands, and the layer's rotate+quantize."""
    import re
    import subprocess
    import torch
    s = layer["spec"]
    X, w, rot = layer["X"][0], layer["w"], layer["rot"]
    q, sc = lrq.ars_rotate_quant(X, rot, s.a_bits)
    qz = torch.zeros_like(q)
    Y = torch.empty((s.M, s.N), dtype=torch.bfloat16, device=dev)
    scratch = torch.zeros(64, dtype=torch.int32, device=dev)
    cases = [("qgemm, the layer's own codes", lambda: lrq.qgemm(q, sc, w, out=Y)),
             ("qgemm, all-zero activation codes", lambda: lrq.qgemm(qz, sc, w, out=Y)),
             ("int8 MFMA loop (16x16x64), pseudo-random operands", lambda: probes.launch_mfma(4096, 2048, 1, scratch)),
             ("int8 MFMA loop (32x32x32), pseudo-random operands", lambda: probes.launch_mfma(4096, 2048, 3, scratch)),
             ("int8 MFMA loop (16x16x64), constant operands", lambda: probes.launch_mfma(4096, 2048, 0, scratch)),
             ("rotate + quantize", lambda: lrq.ars_rotate_quant(X, rot, s.a_bits, q=q, scale=sc))]

    def sclk():
        r = subprocess.run(["rocm-smi", "--showclocks"], capture_output=True, text=True)
        m = re.search(r"sclk clock level:[^(]*\((\d+)Mhz\)", r.stdout)
        return int(m.group(1)) if m else None

    out = dict(layer=s.name, shape=[s.M, s.K, s.N], idle_mhz=sclk(), samples=[])
    for name, fn in cases:
        fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        fn()
        b.record()
        torch.cuda.synchronize()
        one = max(a.elapsed_time(b), 0.02)
        for _ in range(int(2000 / one)):
            fn()
        time.sleep(1.0)
        mhz = sclk()
        torch.cuda.synchronize()
        out["samples"].append(dict(kernel=name, ms_per_launch=round(one, 4), sclk_mhz=mhz))
    return out


def calibration_timings(lrq, layer, dev):
    """Calibration-time entry points on the first layer's shapes: fluctuation metric J over the whole activation
    matrix (HBM-bound: 2 bytes per element), smoothing factor, and the greedy rotation builder on 1024 tokens."""
    import torch
    import synth
    s = layer["spec"]
    X = layer["X"][0]

    def timed(fn, n=5):
        fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(n):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / n

    j_ms = timed(lambda: lrq.fluctuation_metric(X), 20)
    J = float(lrq.fluctuation_metric(X).cpu()[0])
    W = torch.from_numpy(synth.make_weights(s.N, s.K, s.key)).to(dev)
    T = min(1024, s.M)
    sm_ms = timed(lambda: lrq.smooth_factor(X[:T], W, 0.5))
    B, n = 128, 8
    out = dict(layer=s.name, J=round(J, 4), selected=lrq.ars_select(J, 1.0), fluctuation_metric_ms=round(j_ms, 4),
               fluctuation_metric_gbs=round(2.0 * s.M * s.K / (j_ms * 1e-3) / 1e9, 1),
               smooth_factor_ms=round(sm_ms, 4), smooth_factor_tokens=T)
    if s.K % B == 0:
        nb = s.K // B
        Rt = torch.from_numpy(synth.make_spreading_matrix(B)).to(dev)
        Q1 = torch.from_numpy(synth.make_step_rotations(nb, n, B, s.key, 0)).to(dev)
        Q2 = torch.from_numpy(synth.make_step_rotations(nb, n, B, s.key, 1)).to(dev)
        Xc = X[:T].contiguous()
        out.update(build_rotation_ms=round(timed(lambda: lrq.ars_build_rotation(Xc, B, Rt, Q1, Q2), 2), 2),
                   build_rotation=dict(tokens=T, block=B, greedy_steps=n))
    return out


def cpu_baseline(specs, rows, channels):
    """The oracle as it stands, timed on this host's cores on a bounded sample of the same workload:
    the first `rows` token rows of up to four distinct layers (rows are independent under per-token
    quantization), runtime path only (rotate + quantize + integer GEMM + rescale); its own weight
    calibration is done beforehand and not timed, like the GPU's."""
    import oracle
    import synth
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    seen, sample = set(), []
    for s in specs:
        k = (s.K, s.N, s.rotation)
        if k in seen or len(sample) >= 4:
            continue
        seen.add(k)
        sample.append(s)
    ops, t_run = 0, 0.0
    for s in sample:
        m = min(rows, s.M)
        if s.rotation == "dense":
            m = min(m, 128)                 # the oracle's dense rotation accumulates k by k
        # the sample's weights are restricted to `channels` output channels to bound the calibration time
        n = min(s.N, channels)
        X = synth.make_activations(s.M, s.K, s.key, s.p_mild, s.n_salient, s.gain, rows=(0, m))
        W = synth.make_weights(s.N, s.K, s.key)[:n]
        R = synth.make_rotation(s.K, s.key) if s.rotation == "dense" else None
        p = oracle.tlq_calibrate(W, s.w_bits, synth.DEFAULT_GRID, synth.DEFAULT_GRID)
        codes = oracle.tlq_encode(W, p)
        lut, wscale = oracle.tlq_lut(p, 7)
        t0 = time.perf_counter()
        q, sc = oracle.ars_rotate_quant(X, s.a_bits, s.rotation, s.had_block, R)
        y = oracle.qlinear_from_parts(q, sc, codes, lut, wscale, s.w_bits)
        oracle.f64_to_bf16_bits(y)
        t_run += time.perf_counter() - t0
        ops += 2 * m * n * s.K
    return dict(value=round(ops / t_run / 1e12, 5), unit="TOPS", cores=int(cores), kind="oracle",
                seconds=round(t_run, 2),
                sample="first %d token rows (128 where the oracle's k-by-k dense rotation applies) x first %d output channels "
                       "of %d distinct layers (%s); runtime path only (rotate + quantize + integer GEMM + rescale), "
                       "calibration untimed" % (rows, channels, len(sample), ", ".join(s.name for s in sample)))


if __name__ == "__main__":
    main()
