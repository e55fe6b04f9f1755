#!/usr/bin/env python3
"""Benchmark of the DuQuant++ online hot path on one MI355X.

A step is one pass of the whole path over one batch: rotate + MXFP4-quantise the activations
(duqpp_rotate_quantize) and multiply them with the pre-rotated MXFP4 weights (duqpp_mxfp4_gemm).
The default workload is LLaMA-3-8B down_proj prefill (T=2048, K=14336, N=4096, bf16 output) with seeded
synthetic inputs carrying injected outlier channels; the weights are prepared once, before timing.
--config selects the other single-layer shapes or the seven-linear decoder-layer set (one step = every
linear of the set once).
Batches rotate through several buffer sets so that inputs come from HBM rather than from the
256 MB last-level cache.  Prints one JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "rotate+MXFP4-quant GB/s (%HBM peak); W4A4 MXFP4 GEMM TFLOPS (%MFMA peak)"
HBM_PEAK_GBPS = 8000.0        # MI355X HBM3E, published
FP4_PEAK_TFLOPS = 10100.0     # MI355X dense MXFP4 matrix peak, published (256 CU x 2.4 GHz x 16384 flop/clk/CU)

# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE (x 2.000) + WRITE_SIZE (x 1.000), the factors a plain
# 256 MiB device copy gives for the same counters; workload c2_8b_down_prefill.  Counter runs are separate runs of
# this script under the profiler: the figures are copied from their summary, not measured by the run that prints them.
MEASURED_TRAFFIC = {"gemm": 125.12e6 + 16.78e6, "rotq": 61.54e6 + 15.60e6}
TRAFFIC_SOURCE = ("profiles/gemm_tiled_and_rotq_c2_8b_down_prefill_hbm_traffic.md (rocprofv3 --pmc FETCH_SIZE and "
                  "WRITE_SIZE runs of this workload, scaled by a plain copy's readings); not measured in this run")


def rotq_algorithmic_bytes(T, K):
    # bf16 in (2 B) + code out (0.5 B) + scale out (1/32 B) per element, plus R once (4 KiB per block)
    return T * K * (2.0 + 0.5 + 1.0 / 32.0) + 4096.0 * (K // 32)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", default="c2_8b_down_prefill")
    ap.add_argument("--sets", type=int, default=8, help="distinct buffer sets the batches rotate through")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--one-kernel", action="store_true",
                    help="time the one-kernel form (duqpp_rotq_gemm_fused_decode) also at more than 32 tokens, where it "
                         "takes milliseconds per step: use with a small --steps")
    ap.add_argument("--no-two-stream", action="store_true", help="skip the two-stream graph of the steps (an extra figure)")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="default workload only: skip the short runs of the decode and 70B workloads whose figures are "
                         "added to the result line under other_workloads")
    ap.add_argument("--no-machine-probe", action="store_true",
                    help="skip the measurement of the copy rate the machine sustains (1 GiB device copy)")
    ap.add_argument("--no-library-yardstick", dest="library_yardstick", action="store_false",
                    help="skip timing the vendor library's block-scaled FP4 matmul on the same operands (context only)")
    ap.add_argument("--library-yardstick-child", action="store_true", help="internal: time the vendor library's matmul and print it")
    ap.add_argument("--eager", action="store_true", help="time eager launches only (no HIP graph capture)")
    ap.add_argument("--two-stream-child", action="store_true",
                    help="(used by bench.py itself) time only the two-stream graph of the steps and print that figure")
    ap.add_argument("--smoothing", action="store_true",
                    help="run the smoothed form of the path (Eq. 5 as written): a synthetic smoothing diagonal is "
                         "merged into the rotation blocks offline; the timed kernels are the same")
    ap.add_argument("--zero-operands", action="store_true",
                    help="diagnostic, not the metric: time the GEMM on all-zero codes (weights and activations), "
                         "which takes the data-dependent power draw of the matrix cores out of the measurement")
    ap.add_argument("--construct", action="store_true",
                    help="time the offline greedy construction of the shared rotation block (128 steps) on the "
                         "workload's activations and its oracle, print one JSON line, and exit")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="instead of the workload, run a plain device copy of known size (256 MiB, 20 times): "
                         "the reference against which rocprofv3's FETCH_SIZE / WRITE_SIZE readings are scaled")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (the path shards by tokens or output channels "
              "without any exchange between GPUs); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2604_17789_amd as duqpp
    import workloads as wl

    assert torch.cuda.is_available(), "no GPU visible"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.copy_calibration:
        nbytes = 256 << 20
        srcs = [torch.full((nbytes // 4,), float(i), dtype=torch.float32, device=dev) for i in range(4)]
        dsts = [torch.empty_like(t) for t in srcs]
        for i in range(20):
            dsts[i % 4].copy_(srcs[i % 4])
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": {"bytes_read_per_launch": nbytes, "bytes_written_per_launch": nbytes,
                                               "launches": 20}}))
        return
    if args.construct:
        # Offline step, not part of the timed hot path: the calibration batch is the workload's own activations.
        cfg = wl.CONFIGS[args.config]
        Tc, Kc = cfg["T"], cfg["K"]
        xb = wl.make_activations(f"bench-construct-{args.config}", Tc, Kc, cfg["outliers"])
        q = wl.make_orthogonal_steps(f"bench-construct-{args.config}", 128)
        x, qd = torch.from_numpy(xb.view(np.int16)).view(torch.bfloat16).to(dev), torch.from_numpy(q).to(dev)
        duqpp.construct_rotation(x, qd)                     # warm-up
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        R, block, kept, peaks = duqpp.construct_rotation(x, qd, return_peaks=True)
        torch.cuda.synchronize()
        gpu_ms = (time.perf_counter() - t0) * 1e3
        from oracle import construction
        t0 = time.perf_counter()
        ref = construction.greedy_rotation(wl.bf16_bits_to_f32(xb), q)
        cpu_ms = (time.perf_counter() - t0) * 1e3
        pk = peaks.cpu().numpy()
        print(json.dumps({"construct_rotation": {
            "workload": args.config, "T": Tc, "K": Kc, "steps": 128, "ms": round(gpu_ms, 3),
            "oracle_ms": round(cpu_ms, 1), "block": block, "steps_kept": kept, "peak_before": float(pk[0]),
            "peak_after": float(pk[kept]), "identical_to_oracle": bool(
                block == ref["block"] and kept == ref["steps"] and np.array_equal(R.cpu().numpy()[0], ref["R"]))}}))
        return
    # A workload is a list of linears (name, K, N, outliers) run over the same T tokens: one for the single-layer
    # configurations, seven for the decoder-layer set.
    if args.config in wl.LAYER_SET_CONFIGS:
        cfg = wl.LAYER_SET_CONFIGS[args.config]
        linears = [(nm, k, n, cfg["outliers"] if has else ()) for nm, k, n, has in cfg["layers"]]
        if args.sets == 8:
            # 0.64 GB of activations per set; four, so that the per-linear loops below (one linear's buffers of
            # every set: 4 x 85 MB for the 4096-wide ones) also cycle more than the 256 MB last-level cache holds
            args.sets = 4
    else:
        cfg = wl.CONFIGS[args.config]
        linears = [("linear", cfg["K"], cfg["N"], cfg["outliers"])]
    T = cfg["T"]
    out_dtype = duqpp.binding.BF16 if cfg["out"] == "bf16" else duqpp.binding.F32
    single = len(linears) == 1
    K, N = linears[-1][1], linears[-1][2]                   # the linear the oracle sample is taken from

    def dev_bf16(bits):
        return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(dev)

    # ---- inputs: resident in HBM before the timed region --------------------------------
    nsets = max(1, args.sets)
    sets = []
    x0_bits = None
    R0 = None
    lam0 = None
    for s in range(nsets):
        layers = []
        for nm, k, n, outl in linears:
            tag = f"bench-{args.config}-{s}" if single else f"bench-{args.config}-{nm}-{s}"
            xb = wl.make_activations(tag, T, k, outl)
            wb = wl.make_weights(tag, n, k, cfg["w_std"])
            R = wl.make_rotation_blocks(tag, k // 32)
            lam = wl.make_smoothing_scales(tag, k) if args.smoothing else None
            if s == 0 and nm == linears[-1][0]:
                x0_bits, R0, lam0 = xb, R, lam
            x, Rd = dev_bf16(xb), torch.from_numpy(R).to(dev)
            w = dev_bf16(wb)
            Rw = Rd
            if args.smoothing:                            # offline: diag(1/lambda) R for X, diag(lambda) R for W
                Rd, Rw = duqpp.fold_smoothing(Rd, torch.from_numpy(lam).to(dev))
            bc, bs = duqpp.quantize_weights_tiled(w, Rw)  # offline weight transform (tiled layout), not timed
            Rp = duqpp.pack_rotation(Rd)                  # offline: the activation-side blocks in the kernel's operand form
            del w, wb, xb
            cb, sb = duqpp.tiled_bytes(T, k)
            layers.append(dict(
                name=nm, K=k, N=n, x=x, R=Rd, Rp=Rp, bc=bc, bs=bs,
                ac=torch.empty(cb, dtype=torch.uint8, device=dev),
                asc=torch.empty(sb, dtype=torch.uint8, device=dev),
                ws=torch.empty(((cb + 255) // 256 + (sb + 255) // 256) * 256, dtype=torch.uint8, device=dev),
                y=torch.empty((T, n), dtype=torch.bfloat16 if cfg["out"] == "bf16" else torch.float32, device=dev)))
        sets.append(layers)
    torch.cuda.synchronize()

    # the timed path: activations rotated + quantised into the tiled operand layout, then the tiled GEMM
    def rotq1(l):
        duqpp.rotate_quantize_tiled_packed(l["x"], l["Rp"], out=(l["ac"], l["asc"]))

    if args.zero_operands:
        for s_ in sets:
            for l in s_:
                l["bc"].zero_()
                l["x"].zero_()
        torch.cuda.synchronize()

    def gemm1(l):
        duqpp.mxfp4_gemm_tiled(l["ac"], l["asc"], l["bc"], l["bs"], T, l["N"], l["K"], out_dtype=out_dtype, out=l["y"])

    def rotq(s):
        for l in s:
            rotq1(l)

    def gemm(s):
        for l in s:
            gemm1(l)

    def step(s):
        for l in s:
            rotq1(l)
            gemm1(l)

    # the same step through the fused entry point (duqpp_rotq_gemm_tiled_packed): one call per linear, the activation
    # operand in a caller-provided workspace
    def fused1(l):
        duqpp.rotq_gemm_tiled_packed(l["x"], l["Rp"], l["bc"], l["bs"], l["N"], out_dtype=out_dtype, out=l["y"],
                                     workspace=l["ws"])

    def fused_step(s):
        for l in s:
            fused1(l)

    # ---- timing ---------------------------------------------------------------------------
    # `fn` is run args.steps times over the rotating buffer sets between two events on the launch stream, bracketed by
    # device synchronisation.  The figure comes from a HIP graph of exactly those launches (the kernels record no memset
    # nodes): issued one by one from Python, launches of a 3-10 us kernel measure the interpreter, and a graph is never
    # bound by the host.  The figure of eager launches is kept beside it.
    # The chip's clock follows its power draw.  After an idle stretch (the host-side capture of a graph is one) the
    # first few dozen launches run faster than the sustained rate and the next 10-30 ms slower than it (at c2, replays
    # of 20 rotate+quantise launches back to back: 16.3, 16.3, 16.7, 18.0, 18.1, 18.6, 19.7, ... and 16.2 from the 40th
    # millisecond on), so a short timed region measures where in that transient it happens to sit.  Every timed region
    # is therefore preceded, without a pause, by untimed runs of the same work: at least kSustain eager runs (more if
    # --warmup asks for more), and, for a graph, as many untimed replays as fill kLeadMs of GPU time.  Then the graph is
    # replayed kReps times more, back to back, each replay of exactly args.steps steps between its own pair of events;
    # the figure is their median.  The host enqueues replays far ahead of the GPU, so none of them contains the host's
    # latency of launching a graph (some 100 us: 5-10 us per step when only 20 steps are timed).
    kSustain, kReps, kLeadMs = 64, 5, 40.0
    n_warm = max(args.warmup, kSustain)

    def time_replay(g):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        g.replay()
        e1.record()
        torch.cuda.synchronize()
        lead = int(min(2000, max(1, kLeadMs / max(e0.elapsed_time(e1), 1e-3))))
        for _ in range(lead):
            g.replay()
        marks = []
        for _ in range(kReps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            g.replay()
            e1.record()
            marks.append((e0, e1))
        torch.cuda.synchronize()
        return sorted(a.elapsed_time(b) for a, b in marks)[kReps // 2] * 1e3 / args.steps

    def time_region(fn, eager_only=False):
        for i in range(n_warm):
            fn(sets[i % nsets])
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        for i in range(args.steps):
            fn(sets[i % nsets])
        e1.record()
        torch.cuda.synchronize()
        eager_wall_us = (time.perf_counter() - t0) * 1e6 / args.steps
        eager_us = e0.elapsed_time(e1) * 1e3 / args.steps
        graph_us = graph_wall_us = None
        if not eager_only:
            try:
                side = torch.cuda.Stream()
                side.wait_stream(torch.cuda.current_stream())
                g = torch.cuda.CUDAGraph()
                with torch.cuda.stream(side):
                    with torch.cuda.graph(g, stream=side):
                        for i in range(args.steps):
                            fn(sets[i % nsets])
                torch.cuda.synchronize()
                g.replay()
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                g.replay()
                torch.cuda.synchronize()
                graph_wall_us = (time.perf_counter() - t0) * 1e6 / args.steps   # host clock: launch and sync included
                graph_us = time_replay(g)
            except Exception as exc:  # capture unavailable: keep the eager figures
                print(f"bench.py: graph capture failed ({exc}); using eager launches", file=sys.stderr)
        use_graph = graph_us is not None
        return dict(us=graph_us if use_graph else eager_us, eager_us=eager_us, graph_us=graph_us,
                    wall_us=graph_wall_us if graph_wall_us is not None else eager_wall_us,
                    eager_wall_us=eager_wall_us, graph=use_graph)

    # The same steps as a graph of two streams: every rotate+quantise on one, every GEMM on the other, a GEMM waiting
    # for the codes it reads and a rotate+quantise for the GEMM that last read the buffers it overwrites.  Batches are
    # independent, so the rotate+quantise of the next batch may start on the CUs the GEMM of this one has already left,
    # and the launch-to-launch gap between the two kernels is hidden.  Same launches, same results (tests/), default
    # stream priorities.
    def time_steps_two_streams():
        try:
            sg, sr = torch.cuda.Stream(), torch.cuda.Stream()
            sg.wait_stream(torch.cuda.current_stream())
            g = torch.cuda.CUDAGraph()
            with torch.cuda.stream(sg):
                with torch.cuda.graph(g, stream=sg):
                    sr.wait_stream(sg)
                    free = {}                              # (set, linear) -> event after the GEMM that last read its codes
                    events = []                            # every event stays alive until the capture has ended
                    for i in range(args.steps):
                        k = i % nsets
                        for li, l in enumerate(sets[k]):
                            with torch.cuda.stream(sr):
                                if (k, li) in free:
                                    sr.wait_event(free[(k, li)])
                                rotq1(l)
                                ready = torch.cuda.Event()
                                ready.record(sr)
                            sg.wait_event(ready)
                            gemm1(l)
                            free[(k, li)] = torch.cuda.Event()
                            free[(k, li)].record(sg)
                            events += [ready, free[(k, li)]]
                    sg.wait_stream(sr)
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            return time_replay(g)
        except Exception as exc:
            print(f"bench.py: two-stream graph capture failed ({exc})", file=sys.stderr)
            return None

    # ---- the vendor library on the same operands, as a yardstick ----------------------------------------------------
    # torch.nn.functional.scaled_mm (hipBLASLt underneath) multiplies the same E2M1 codes under the same E8M0 scales of
    # 32-element groups, from the row-major layout, with bf16 results (its block-scaled form offers no fp32 output).
    # It is timed like the GEMM, on the operands of the workload's last linear.  Context only: nothing in the product
    # calls it, a torch build without the call just leaves the key out, and it runs in a child process of its own so
    # that nothing that happens inside that library can cost this run its result line.
    def library_yardstick():
        import torch.nn.functional as F
        fp4, e8m0 = torch.float4_e2m1fn_x2, torch.float8_e8m0fnu
        recipe, noswz = F.ScalingType.BlockWise1x32, F.SwizzleType.NO_SWIZZLE
        for s_ in sets:
            l = s_[-1]
            rotq1(l)
            a, sa = duqpp.untile_operand(l["ac"], l["asc"], T, l["K"])
            b, sb = duqpp.untile_operand(l["bc"], l["bs"], l["N"], l["K"])
            l["lib"] = (a.view(fp4), sa.view(e8m0), b.view(fp4).t(), sb.view(e8m0))

        def lib1(s_):
            a, sa, bt, sb = s_[-1]["lib"]
            return F.scaled_mm(a, bt, sa, recipe, sb, recipe, swizzle_a=noswz, swizzle_b=noswz,
                               output_dtype=torch.bfloat16)

        l0 = sets[0][-1]
        y_lib = lib1(sets[0]).float()
        y_own = duqpp.mxfp4_gemm_tiled(l0["ac"], l0["asc"], l0["bc"], l0["bs"], T, l0["N"], l0["K"],
                                       out_dtype=duqpp.binding.BF16).float()
        rel = float((y_lib - y_own).norm() / y_own.norm())
        del y_lib, y_own
        lib_us = time_region(lib1)["us"]
        own_us = time_region(lambda s_: gemm1(s_[-1]))["us"]
        fl = 2.0 * T * l0["N"] * l0["K"]
        return {"what": "torch.nn.functional.scaled_mm (hipBLASLt) on the same MXFP4 operands, row-major, bf16 out",
                "us": round(lib_us, 2), "TFLOP/s": round(fl / lib_us / 1e6, 1),
                "this_library_us": round(own_us, 2), "this_library_TFLOP/s": round(fl / own_us / 1e6, 1),
                "library_time_over_this_library": round(lib_us / own_us, 3),
                "rel_frobenius_difference_of_bf16_results": float(f"{rel:.3e}")}

    if args.library_yardstick_child:
        try:
            print(json.dumps({"library_yardstick": library_yardstick()}))
        except (AttributeError, RuntimeError, TypeError, ValueError) as exc:
            print(json.dumps({"library_yardstick": None, "reason": str(exc)[:200]}))
        return

    if args.two_stream_child:
        for i in range(n_warm):
            step(sets[i % nsets])
        print(json.dumps({"two_stream_us": time_steps_two_streams()}))
        return
    whole = time_region(step, eager_only=args.eager)
    # exactly args.steps steps between two events on the launch stream (a one-stream graph replay; eager launches with
    # --eager): the figure the result line's value is computed from
    one_stream_us = whole["us"]
    fused = time_region(fused_step, eager_only=args.eager)
    # up to 32 tokens: the one-kernel form (rotation and quantiser in the prologue of every product workgroup)
    one_kernel = None
    if T <= 32 or args.one_kernel:
        one_kernel = time_region(lambda s: [duqpp.rotq_gemm_fused_decode(l["x"], l["Rp"], l["bc"], l["bs"], l["N"],
                                                                         out_dtype=out_dtype, out=l["y"]) for l in s],
                                 eager_only=args.eager)
    # A second launch form is reported beside it, never as the metric: the same steps as a graph over two streams.  It
    # is measured in a child process of its own (same inputs, same kernels), so that nothing that happens to a capture
    # over several streams can cost this run its result line.  Prefill workloads only.
    two_stream_us = None
    if not args.eager and T > 128 and not args.no_two_stream:
        import subprocess
        cmd = [sys.executable, os.path.abspath(__file__), "--two-stream-child", "--config", args.config, "--steps",
               str(args.steps), "--warmup", str(args.warmup), "--sets", str(nsets)]
        cmd += (["--smoothing"] if args.smoothing else []) + (["--zero-operands"] if args.zero_operands else [])
        try:
            child = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=600)
            if child.returncode == 0:
                two_stream_us = json.loads(child.stdout.strip().splitlines()[-1])["two_stream_us"]
            else:
                print(f"bench.py: two-stream child ended with status {child.returncode}", file=sys.stderr)
        except Exception as exc:
            print(f"bench.py: two-stream child failed ({exc})", file=sys.stderr)
    ms_per_step = one_stream_us * 1e-3
    # each kernel alone, its launches back to back (what the rooflines use; includes the ~2.2 us launch-to-launch gap an
    # empty kernel also shows)
    tr = time_region(rotq, eager_only=args.eager)
    tg = time_region(gemm, eager_only=args.eager)
    rotq_us, rotq_eager_us, gemm_us, gemm_eager_us = tr["us"], tr["eager_us"], tg["us"], tg["eager_us"]
    per_linear = None
    if not single:
        per_linear = []
        for li, (nm, k, n, _) in enumerate(linears):
            r1 = time_region(lambda s, li=li: rotq1(s[li]), eager_only=args.eager)["us"]
            g1 = time_region(lambda s, li=li: gemm1(s[li]), eager_only=args.eager)["us"]
            per_linear.append({"name": nm, "K": k, "N": n, "rotq_us": round(r1, 2),
                               "rotq_GB/s": round(rotq_algorithmic_bytes(T, k) / r1 / 1e3, 1),
                               "gemm_us": round(g1, 2), "gemm_TFLOP/s": round(2.0 * T * n * k / g1 / 1e6, 1)})

    flops = sum(2.0 * T * n * k for _, k, n, _ in linears)
    rotq_bytes = sum(rotq_algorithmic_bytes(T, k) for _, k, _, _ in linears)
    weight_bytes = sum(n * k * (0.5 + 1.0 / 32.0) for _, k, n, _ in linears)
    rotq_gbps = rotq_bytes / (rotq_us * 1e-6) / 1e9
    gemm_tflops = flops / (gemm_us * 1e-6) / 1e12
    value = flops / (ms_per_step * 1e-3) / 1e12
    headline = args.config == "c2_8b_down_prefill"

    result = {
        "metric": METRIC,
        "value": round(value, 2),
        "unit": "TFLOP/s (2*T*N*K per whole step: rotate+quantise, then GEMM)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "ms_per_step_eager_launches": round(whole["eager_us"] * 1e-3, 5),
        "ms_per_step_graph_replay": None if whole["graph_us"] is None else round(whole["graph_us"] * 1e-3, 5),
        "ms_per_step_graph_replay_host_clock": round(whole["wall_us"] * 1e-3, 5),
        "ms_per_step_two_stream_graph": None if two_stream_us is None else round(two_stream_us * 1e-3, 5),
        "launch": ("HIP graph replay of the timed steps on one stream, timed by events on that stream (median of "
                   f"{kReps} back-to-back replays that follow {n_warm} untimed steps and {kLeadMs:.0f} ms of untimed replays)"
                   if whole["graph"] else "eager launches on one stream, timed by events on that stream"),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "mxfp4 (E2M1 codes + E8M0 scales; fp32 rotation and accumulation)",
        "data": "synthetic" if not args.zero_operands else "all-zero operands (diagnostic run, not the metric)",
        "config": {"workload": args.config, "T": T,
                   "linears": [{"name": nm, "K": k, "N": n} for nm, k, n, _ in linears],
                   "output": cfg["out"], "buffer_sets": nsets, "operand_layout": "tiled",
                   "rotation_blocks": "packed offline (duqpp_pack_rotation)",
                   "smoothing": bool(args.smoothing)},
        "per_kernel_timing": "each kernel alone, its launches back to back in a replayed graph (median of replays)",
        "components": {
            "rotate_quantize": {"us": round(rotq_us, 2), "us_alone_eager_launches": round(rotq_eager_us, 2),
                                "us_alone_graph_replay": None if tr["graph_us"] is None else round(tr["graph_us"], 2),
                                "launches": len(linears), "GB/s": round(rotq_gbps, 1),
                                "frac_hbm_peak": round(rotq_gbps / HBM_PEAK_GBPS, 4)},
            "mxfp4_gemm": {"us": round(gemm_us, 2), "us_alone_eager_launches": round(gemm_eager_us, 2),
                           "us_alone_graph_replay": None if tg["graph_us"] is None else round(tg["graph_us"], 2),
                           "launches": len(linears), "TFLOP/s": round(gemm_tflops, 1),
                           "frac_mfma_peak": round(gemm_tflops / FP4_PEAK_TFLOPS, 4),
                           # N*K*(1/2 + 1/32) bytes of weights per launch: the decode-shape figure of merit
                           "weight_stream_GB/s": round(weight_bytes / (gemm_us * 1e-6) / 1e9, 1)},
            # one duqpp_rotq_gemm_tiled_packed call per linear (rotate+quantise into the caller's workspace, then the GEMM)
            # beside the two separate calls (ms_per_step): the same two kernels on the same stream either way
            "rotq_gemm_fused_call": {"us": round(fused["us"], 2), "us_eager_launches": round(fused["eager_us"], 2),
                                     "us_graph_replay": None if fused["graph_us"] is None else round(fused["graph_us"], 2),
                                     "separate_calls_us": round(one_stream_us, 2), "launches": len(linears)},
        },
        "roofline": {"kernel": "mxfp4_gemm", "bound": "mfma", "achieved": round(gemm_tflops, 1),
                     "peak": FP4_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(gemm_tflops / FP4_PEAK_TFLOPS, 4),
                     "traffic": MEASURED_TRAFFIC["gemm"] if headline else None,
                     "traffic_source": TRAFFIC_SOURCE if headline else None},
        "roofline_rotate_quantize": {"kernel": "rotq", "bound": "hbm", "achieved": round(rotq_gbps, 1),
                                     "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                                     "frac": round(rotq_gbps / HBM_PEAK_GBPS, 4),
                                     "traffic": MEASURED_TRAFFIC["rotq"] if headline else None,
                                     "traffic_source": TRAFFIC_SOURCE if headline else None},
    }
    if one_kernel is not None:
        # duqpp_rotq_gemm_fused_decode: one launch, no activation operand in memory; every workgroup repeats the rotation
        result["components"]["rotq_gemm_one_kernel"] = {"us": round(one_kernel["us"], 2),
                                                        "us_eager_launches": round(one_kernel["eager_us"], 2),
                                                        "two_launches_us": round(one_stream_us, 2)}
    if per_linear:
        result["components"]["per_linear"] = per_linear
        # each per-linear loop cycles the buffer sets of ONE linear; the aggregate figures above cycle all of them
        result["components"]["per_linear_note"] = (f"each figure cycles one linear's {nsets} buffer sets; with fewer than "
                                                   "4 sets of a 4096-wide linear they fit the 256 MB last-level cache")
    if T <= 32:
        # decode shapes: the product streams the weights once, so HBM bounds it, not the matrix cores
        result["roofline"] = {"kernel": "mxfp4_gemm (decode)", "bound": "hbm",
                              "achieved": round(weight_bytes / (gemm_us * 1e-6) / 1e9, 1), "peak": HBM_PEAK_GBPS,
                              "unit": "GB/s", "frac": round(weight_bytes / (gemm_us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4),
                              "traffic": None}

    # ---- what the machine sustains on a plain copy, measured here, beside the published HBM peak ---------------
    if not args.no_machine_probe:
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(4):
            dst.copy_(src)
        e1.record()
        torch.cuda.synchronize()
        copy_gbps = 4 * 2.0 * src.numel() * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9
        del src, dst
        result["machine"] = {"hbm_copy_GB/s": round(copy_gbps, 1),
                             "hbm_copy_frac_of_peak": round(copy_gbps / HBM_PEAK_GBPS, 4)}
        result["roofline_rotate_quantize"]["frac_of_copy_rate"] = round(rotq_gbps / copy_gbps, 4)

    # ---- the vendor library's block-scaled FP4 matmul on the same operands (context only), in a child process ---------
    if args.library_yardstick and single and T > 128 and not (args.eager or args.zero_operands):
        import subprocess
        cmd = [sys.executable, os.path.abspath(__file__), "--library-yardstick-child", "--config", args.config, "--steps",
               str(args.steps), "--warmup", str(args.warmup), "--sets", str(nsets)]
        cmd += ["--smoothing"] if args.smoothing else []
        try:
            child = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=300)
            if child.returncode == 0:
                r = json.loads(child.stdout.strip().splitlines()[-1])
                if r["library_yardstick"] is not None:
                    result["library_yardstick"] = r["library_yardstick"]
                else:
                    print(f"bench.py: library yardstick not available ({r.get('reason')})", file=sys.stderr)
            else:
                print(f"bench.py: library yardstick child ended with status {child.returncode}", file=sys.stderr)
        except Exception as exc:
            print(f"bench.py: library yardstick child failed ({exc})", file=sys.stderr)

    # ---- the CPU oracle on a bounded sample of the same workload ---------------------------
    if not args.no_cpu_baseline:
        import oracle
        try:
            from threadpoolctl import threadpool_info
            threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            threads = os.cpu_count() or 1
        # a bounded sample: every token (at most 8192) of one linear -- 2 to 10 s of oracle work at the
        # benchmark shapes, most of it the fp64 product
        Ts = min(T, 8192)
        s0 = sets[0][-1]
        bc_rm, bs_rm = duqpp.untile_operand(s0["bc"], s0["bs"], N, K)       # row-major view of the weights for the oracle
        bc_h, bs_h = bc_rm.cpu().numpy(), bs_rm.cpu().numpy()
        c0 = time.perf_counter()
        a_codes, a_scales, _ = oracle.pipeline.rotate_quantize(x0_bits[:Ts], R0, lam=lam0)
        y_ref = oracle.linear.mxfp4_gemm(a_codes, a_scales, bc_h, bs_h)
        c1 = time.perf_counter()
        result["cpu_baseline"] = {
            "value": round(2.0 * Ts * N * K / (c1 - c0) / 1e12, 5), "unit": "TFLOP/s (whole step)",
            "cores": int(threads), "kind": "oracle", "seconds": round(c1 - c0, 2),
            "sample": f"first {Ts} of {T} tokens of linear '{s0['name']}', full K={K} and N={N} "
                      "(rotate+quantise then fp64 product)"}
        # the sampled rows double as a live parity check of what was timed
        rotq1(s0)
        gemm1(s0)
        torch.cuda.synchronize()
        y_dev = s0["y"][:Ts].float().cpu().numpy()
        ac_rm, as_rm = duqpp.untile_operand(s0["ac"], s0["asc"], T, K)
        a_dev = ac_rm[:Ts].cpu().numpy()
        result["parity"] = {
            "codes_equal_fraction": float(np.mean(a_dev == a_codes)),
            "gemm_rel_fro_vs_oracle_on_own_codes": float(
                np.linalg.norm(y_dev - oracle.linear.mxfp4_gemm(a_dev, as_rm[:Ts].cpu().numpy(), bc_h, bs_h))
                / np.linalg.norm(y_ref)),
            "note": "bf16 output rounding (2^-9) bounds the second figure" if cfg["out"] == "bf16" else ""}
    # ---- the other workloads of the metric, in short: child runs of this script (one process per workload keeps their
    # buffers apart), their main figures under one key.  Only the default run of the headline workload does this.
    if headline and not (args.no_other_workloads or args.eager or args.smoothing or args.zero_operands):
        import subprocess
        others = {}
        for cfg_name, extra in (("c3_decode_gateup_T1", []), ("c3_decode_down_T16", []),
                                ("c4_70b_down_prefill", ["--sets", "2", "--steps", "50", "--no-two-stream"]),
                                ("c5_8b_layer_set_T8192", ["--steps", "20", "--no-two-stream"])):
            cmd = [sys.executable, os.path.abspath(__file__), "--config", cfg_name, "--no-cpu-baseline",
                   "--no-machine-probe"] + extra
            try:
                child = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=300)
                if child.returncode != 0:
                    others[cfg_name] = {"error": f"exit status {child.returncode}"}
                    continue
                r = json.loads(child.stdout.strip().splitlines()[-1])
                c = r["components"]
                others[cfg_name] = {
                    "us_per_step": round(r["ms_per_step"] * 1e3, 2), "steps": r["steps"], "buffer_sets": r["config"]["buffer_sets"],
                    "rotate_quantize_us": c["rotate_quantize"]["us"], "rotate_quantize_frac_hbm_peak": c["rotate_quantize"]["frac_hbm_peak"],
                    "mxfp4_gemm_us": c["mxfp4_gemm"]["us"], "mxfp4_gemm_frac_mfma_peak": c["mxfp4_gemm"]["frac_mfma_peak"],
                    "weight_stream_GB/s": c["mxfp4_gemm"]["weight_stream_GB/s"],
                    "rotq_gemm_fused_call_us": c["rotq_gemm_fused_call"]["us"],
                    "rotq_gemm_one_kernel_us": c.get("rotq_gemm_one_kernel", {}).get("us"),
                    "roofline": {k: r["roofline"][k] for k in ("bound", "achieved", "peak", "unit", "frac")}}
                if "library_yardstick" in r:
                    others[cfg_name]["library_yardstick_us"] = r["library_yardstick"]["us"]
            except Exception as exc:
                others[cfg_name] = {"error": str(exc)}
        result["other_workloads"] = others
    print(json.dumps(result))


if __name__ == "__main__":
    main()
