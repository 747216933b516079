"""Benchmark of the bit-serial GEMM hot path on one MI355X.

    python bench.py --gpus 1 --steps K --warmup W

A step is one pass of the hot path over one batch of the W2A2 4096^3 configuration:
bit-plane packing of the int8 activation matrix (K x N, transposing) followed by the
bit-serial GEMM to int32 (weights are packed once, outside the timed region, as they
would be for inference).  All inputs are resident in HBM before timing starts.  One JSON
line is printed: the headline metric (GOPS = 2 M N K / T, Sec. 4.1 of the paper), the
roofline figures of the dominant kernel, the CPU oracle timed on the host's cores, and
per-kernel figures for the other configurations (GEMV chain, lowered convolution, W4A4
sweep) for context.
"""
from __future__ import annotations

import argparse
import json
import sys
import time

import numpy as np

# chip figures used for the rooflines
CUS, SIMDS_PER_CU, LANES, CLOCK_HZ = 256, 4, 64, 2.4e9
# One product of Alg. 1's inner loop = 32 binary MACs per lane = one v_and_b32 + one v_bcnt_u32_b32.  A SIMD executes the
# AND at 32 lanes per clock (the rate behind the chip's 157.3 TFLOP/s fp32 vector figure) and the popcount at 16 lanes
# per clock: 2 + 4 = 6 clocks per wavefront-wide product.
CLOCKS_PER_PRODUCT = 6
BINARY_PEAK_TOPS = CUS * SIMDS_PER_CU * LANES * 32 * 2 / CLOCKS_PER_PRODUCT * CLOCK_HZ / 1e12   # 1677.7
HBM_PEAK_GBS = 8000.0
# HBM bytes per bs_gemm launch on the W2A2 4096^3 workload, from rocprofv3 --pmc FETCH_SIZE and
# WRITE_SIZE scaled by a 256 MiB copy (profiles/bench_w2a2_4096_trace_and_counters.md): 24.5 MiB + 64 MiB.  A counter run
# cannot be made from inside this script; the figure is the one of the committed profile and is labelled as such.
GEMM_TRAFFIC_BYTES = 92_953_222
GEMM_TRAFFIC_SOURCE = "profiles/bench_w2a2_4096_trace_and_counters.md (rocprofv3 --pmc FETCH_SIZE, WRITE_SIZE of an earlier run of this command; not re-measured in this run)"
# untimed GEMM launches before the warm-up steps (see main)
CLOCK_WARMUP_LAUNCHES = 100
# the inner loop's AND / popcount / idle-slot rhythm is worth 4..16 % and rests on how the compiler spaces dependent
# instructions; below this fraction of the in-run probe rate the line says so ("rhythm_ok": false)
RHYTHM_MIN_FRACTION_OF_PROBE = 0.80


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the benchmark line, run the W1A1 size sweep of Sec. 4.1.2 (every dimension "
                         "from 2^6 to 2^12) and print one JSON line per (M, K, N)")
    ap.add_argument("--only", choices=["gemv", "dense", "planes", "chain"], default=None,
                    help="run one kernel family only, with plain launches and a short JSON line: the few-column "
                         "(batch-1) kernels, the matrix-core kernels on unpacked operands, the matrix-core "
                         "kernels on packed planes, or the batch-1 layer chain conv2..fc7 as eight and as six "
                         "launches; meant to be run under rocprofv3")
    ap.add_argument("--case", default=None, help="with --only: run this one case (see the names in the printed line)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run plain 256 MiB device copies, so that rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE "
                         "readings can be scaled by what the same counter reports for a copy of known size")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus %d is not supported (no collectives, no sharding "
              "in this library)" % args.gpus, file=sys.stderr)
        return 2

    import torch
    import paper_1709_04060_amd as bs
    from paper_1709_04060_amd import workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; there is no CPU fallback", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    bs.load_library()

    def dev(a):
        return torch.from_numpy(np.ascontiguousarray(a)).cuda()

    def timed(fn, iters, warm):
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        for _ in range(iters):
            fn()
        e1.record()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) * 1e3 / iters
        return e0.elapsed_time(e1) / iters, wall

    if args.sweep:
        return sweep(bs, torch)
    if args.only:
        print(json.dumps(only(args.only, args.case, bs, torch, timed)))
        return 0

    if args.calibration_copy:
        src = torch.full((256 << 20,), 3, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ------------------------------------------------------------- headline: W2A2 4096^3
    M = N = K = 4096
    w, a = 2, 2
    d = workloads.cfg2_square(M)
    Wd, Ad = dev(d["W"]), dev(d["A"])
    Wp = bs.bs_pack_planes(Wd, w, bs.BS_TWOS_COMPLEMENT)
    Ap = torch.empty((a, N, bs.bs_words_per_row(K)), dtype=torch.int64, device="cuda")
    C = torch.empty((M, N), dtype=torch.int32, device="cuda")

    BSER = bs.BS_ENGINE_BITSERIAL   # the headline is the AND-popcount kernel (Alg. 1, 2), whatever bs_gemm itself would pick

    def step():
        bs.bs_pack_planes(Ad, a, bs.BS_UNSIGNED, depth_is_strided=True, out=Ap)
        bs.bs_gemm(Wp, bs.BS_TWOS_COMPLEMENT, Ap, bs.BS_UNSIGNED, K, out=C, engine=BSER)

    # The device leaves its idle clocks only after tens of milliseconds of work (measured: 0.451 ms per step over 20
    # steps after a 3-step warm-up, 0.410 ms over 200): set-up ends with 100 untimed GEMM launches (about 40 ms), so
    # that the W warm-up steps and the K timed steps run at the clocks of a busy device whatever W and K are.
    for _ in range(CLOCK_WARMUP_LAUNCHES):
        bs.bs_gemm(Wp, bs.BS_TWOS_COMPLEMENT, Ap, bs.BS_UNSIGNED, K, out=C, engine=BSER)
    torch.cuda.synchronize()
    ev_ms, wall_ms = timed(step, args.steps, args.warmup)
    ms_per_step = max(ev_ms, wall_ms)
    gops = 2.0 * M * N * K / (ms_per_step * 1e-3) / 1e9

    # The dominant kernel's launch duration inside the step: the same pack -> GEMM sequence once more, with an
    # event on either side of every GEMM launch (events are recorded on torch's current stream, which is the
    # stream handed to the library).  The clean loop above gives `value`; this one only the kernel's time.
    ev_a = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    ev_b = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    for i in range(args.steps):
        bs.bs_pack_planes(Ad, a, bs.BS_UNSIGNED, depth_is_strided=True, out=Ap)
        ev_a[i].record()
        bs.bs_gemm(Wp, bs.BS_TWOS_COMPLEMENT, Ap, bs.BS_UNSIGNED, K, out=C, engine=BSER)
        ev_b[i].record()
    torch.cuda.synchronize()
    gemm_ms = sum(x.elapsed_time(y) for x, y in zip(ev_a, ev_b)) / args.steps
    # and alone, back to back (no packing kernel in between: warmer caches, steadier clock)
    gemm_alone_ms, _ = timed(lambda: bs.bs_gemm(Wp, bs.BS_TWOS_COMPLEMENT, Ap, bs.BS_UNSIGNED, K, out=C, engine=BSER), args.steps, 2)
    pack_ms, _ = timed(lambda: bs.bs_pack_planes(Ad, a, bs.BS_UNSIGNED, depth_is_strided=True, out=Ap), args.steps, 2)
    binary_tops = w * a * 2.0 * M * N * K / (gemm_ms * 1e-3) / 1e12

    # the chip's measured ceiling for the AND + popcount pair (register operands, all compute units,
    # eight wavefronts per SIMD), next to the theoretical peak
    sink = torch.empty(8 * CUS, dtype=torch.int32, device="cuda")
    probe_passes = 20000
    probe_ms, _ = timed(lambda: bs.bs_probe_popcount_rate(sink, probe_passes), 3, 1)
    probe_lane_ops = sink.numel() * 256 * probe_passes * 32
    measured_peak_tops = probe_lane_ops / 2 * 32 * 2 / (probe_ms * 1e-3) / 1e12

    result = {
        "metric": "bit-serial GEMM GOPS (2*M*N*K/T), W2A2", "value": round(gops, 1), "unit": "GOPS",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "clock_warmup_launches": CLOCK_WARMUP_LAUNCHES,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u32", "dtype_note": "32-bit AND + popcount on bit planes, int32 accumulation",
        "data": "synthetic",
        "config": {"workload": "W2A2 4096x4096x4096: pack int8 activations (K x N) to bit planes + bit-serial "
                               "GEMM (AND-popcount engine) to int32; weights pre-packed", "M": M, "N": N, "K": K,
                   "wbits": w, "abits": a, "engine": "bit-serial (bs_gemm_on); bs_gemm itself picks the fp4 matrix-core "
                                                      "kernel for this shape, see other_configs.engines_on_packed_planes"},
        "roofline": {"bound": "alu", "kernel": "bs_gemm_kernel<2,2,...>", "achieved": round(binary_tops, 1),
                     "peak": round(BINARY_PEAK_TOPS, 1), "unit": "binary TOP/s", "frac": round(binary_tops / BINARY_PEAK_TOPS, 4),
                     "measured_peak": round(measured_peak_tops, 1),
                     "frac_of_measured_peak": round(binary_tops / measured_peak_tops, 4),
                     "rhythm_ok": bool(binary_tops >= RHYTHM_MIN_FRACTION_OF_PROBE * measured_peak_tops),
                     "kernel_ms": round(gemm_ms, 4), "kernel_ms_back_to_back": round(gemm_alone_ms, 4),
                     "traffic": GEMM_TRAFFIC_BYTES, "traffic_source": GEMM_TRAFFIC_SOURCE,
                     "algorithmic_bytes": 2 * (w * M * K // 8) // 1 + 4 * M * N},
        "breakdown_ms": {"pack_activations": round(pack_ms, 4), "bs_gemm": round(gemm_ms, 4)},
    }

    # ------------------------------------------------------------- CPU oracle on the host cores
    if not args.no_cpu_baseline:
        import oracle
        # spot check of the timed result against the oracle (sampled outputs; the full comparison is in tests/)
        Ch = C.cpu().numpy()
        rng = np.random.default_rng(0)
        for _ in range(64):
            m, n = int(rng.integers(M)), int(rng.integers(N))
            assert int(Ch[m, n]) == oracle.dot(d["W"], d["A"], m, n), "GPU result differs from the oracle"
        oracle.gemm(d["W"][:64], d["A"])
        t0 = time.perf_counter()
        reps = 0
        while reps < 3 or time.perf_counter() - t0 < 10.0:
            oracle.gemm(d["W"], d["A"])
            reps += 1
        dt = (time.perf_counter() - t0) / reps
        result["cpu_baseline"] = {"value": round(2.0 * M * N * K / dt / 1e9, 1), "unit": "GOPS",
                                  "cores": oracle.num_threads(), "kind": "oracle",
                                  "compile_flags": "gcc " + " ".join(oracle.COMPILE_FLAGS) + " (built where there is no GPU, "
                                                   "hence no -march=native: the host's widest vectors are not used)",
                                  "sample": "the full 4096^3 integer product (no packing), mean of %d runs, %.2f s each"
                                            % (reps, dt)}
        # the oracle on the small configurations, once each (milliseconds), beside the GPU times below
        def once(fn):
            t = time.perf_counter()
            fn()
            return round((time.perf_counter() - t) * 1e3, 2)
        c3, c4 = workloads.cfg3_fc_chain(), workloads.cfg4_conv2()
        result["cpu_baseline"]["other_configs_ms"] = {
            "fc6_W1A2_4096x9216x1": once(lambda: oracle.threshold(oracle.gemm(c3["W6"], c3["x"]), c3["thr6"])),
            "fc7_W1A2_4096x4096x1": once(lambda: oracle.threshold(
                oracle.gemm(c3["W7"], np.zeros((c3["W7"].shape[1], 1), dtype=np.int8)), c3["thr7"])),
            "conv2_W1A2_direct_convolution_and_thresholds": once(lambda: oracle.threshold(
                oracle.conv_direct(c4["x"], c4["filt"], c4["stride"], c4["pad"]).reshape(-1, c4["filt"].shape[0]).T.copy(),
                c4["thr"]))}
        for n5 in (1, 64, 1024, 8192):   # W4A4 8192 x 8192 x N: integer product + 15 thresholds per row
            c5 = workloads.cfg5_w4a4(n5)
            result["cpu_baseline"]["other_configs_ms"]["W4A4_8192x8192x%d_product_and_thresholds" % n5] = once(
                lambda: oracle.threshold(oracle.gemm(c5["W"], c5["A"]), c5["thr"]))
            del c5

    # ------------------------------------------------------------- other configurations, per kernel
    if not args.no_extras:
        result["other_configs"] = extras(bs, workloads, dev, timed)

    print(json.dumps(result))
    return 0


def sweep(bs, torch):
    """The paper's performance-versus-size experiment (Sec. 4.1.2, Fig. 3): W1A1 (both operands
    bipolar) bit-serial GEMM for every M, K, N in {2^6 .. 2^12}; GOPS = 2 M N K / T with T the
    graph-replayed kernel time.  Also prints the best and worst GOPS per depth."""
    sizes = [1 << e for e in range(6, 13)]
    BP = bs.BS_BIPOLAR
    best = {}
    for K in sizes:
        for M in sizes:
            Wp = torch.randint(-2 ** 62, 2 ** 62, (1, M, bs.bs_words_per_row(K)), dtype=torch.int64, device="cuda")
            for N in sizes:
                Ap = torch.randint(-2 ** 62, 2 ** 62, (1, N, bs.bs_words_per_row(K)), dtype=torch.int64, device="cuda")
                C = torch.empty((M, N), dtype=torch.int32, device="cuda")
                ms = timed_graph([lambda: bs.bs_gemm(Wp, BP, Ap, BP, K, out=C)], 20)
                gops = 2.0 * M * N * K / ms / 1e6
                print(json.dumps({"sweep": "W1A1", "M": M, "K": K, "N": N, "us": round(ms * 1e3, 2), "GOPS": round(gops, 1)}))
                lo, hi = best.get(K, (float("inf"), 0.0))
                best[K] = (min(lo, gops), max(hi, gops))
    print(json.dumps({"sweep_summary_GOPS_min_max_by_depth": {str(k): [round(v[0], 1), round(v[1], 1)] for k, v in best.items()}}))
    return 0


def only(which, case, bs, torch, timed):
    """One kernel family with plain launches (a counter run of rocprofv3 sees one dispatch per launch and the kernel
    names stay apart when a single case is selected with --case).  Times are HIP-event averages over the launches."""
    BP, U, TC = bs.BS_BIPOLAR, bs.BS_UNSIGNED, bs.BS_TWOS_COMPLEMENT
    BSER = bs.BS_ENGINE_BITSERIAL
    res = {"only": which, "cases": {}}

    def planes(bits, rows, K):
        return torch.randint(-2 ** 62, 2 ** 62, (bits, rows, bs.bs_words_per_row(K)), dtype=torch.int64, device="cuda")

    def thr_for(Mrows, obits):
        T = (1 << obits) - 1
        return torch.sort(torch.randint(-1000, 1000, (Mrows, T), dtype=torch.int32, device="cuda"), dim=1)[0].contiguous()

    def run(name, fns, rounds):
        if case and case != name:
            return
        for f in fns[:2]:
            f()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(rounds):
            for f in fns:
                f()
        e1.record()
        torch.cuda.synchronize()
        res["cases"][name] = {"us_per_launch": round(e0.elapsed_time(e1) * 1e3 / (rounds * len(fns)), 2),
                              "launches": rounds * len(fns)}

    if which == "gemv":
        # (name, w, wfmt, a, M, K, obits, weight buffers cycled): cold = more bytes than the 256 MiB last-level cache
        for (name, w, wf, a, M, K, ob, copies) in [
                ("fc6_W1A2_4096x9216x1_cold", 1, BP, 2, 4096, 9216, 2, 96), ("fc6_W1A2_4096x9216x1_warm", 1, BP, 2, 4096, 9216, 2, 1),
                ("fc7_W1A2_4096x4096x1_cold", 1, BP, 2, 4096, 4096, 2, 192), ("fc7_W1A2_4096x4096x1_warm", 1, BP, 2, 4096, 4096, 2, 1),
                ("W4A4_8192x8192x1_cold", 4, TC, 4, 8192, 8192, 4, 12), ("W4A4_8192x8192x1_warm", 4, TC, 4, 8192, 8192, 4, 1),
                ("W1A2_32768x32768x1_cold", 1, BP, 2, 32768, 32768, 2, 3)]:
            if case and not case.startswith(name):
                continue
            Wps = [planes(w, M, K) for _ in range(copies)]
            Ap, th = planes(a, 1, K), thr_for(M, ob)
            Y = torch.empty((ob, 1, bs.bs_words_per_row(M)), dtype=torch.int64, device="cuda")
            sink = torch.zeros(1024, dtype=torch.int32, device="cuda")
            rounds = 100 if copies == 1 else 3
            run(name, [(lambda Wp=Wp: bs.bs_gemm_threshold(Wp, wf, Ap, U, K, th, ob, out=Y, engine=BSER)) for Wp in Wps], rounds)
            run(name + "_stream_read_probe", [(lambda Wp=Wp: bs.bs_probe_stream_read(Wp, sink)) for Wp in Wps], rounds)
            run(name + "_stream_read_probe_nontemporal", [(lambda Wp=Wp: bs.bs_probe_stream_read(Wp, sink, non_temporal=True)) for Wp in Wps], rounds)
            del Wps
    elif which == "dense":
        for (name, fp4, M, N, K, ob) in [("dense_int8_4096", False, 4096, 4096, 4096, 0), ("dense_int8_8192_fused4", False, 8192, 8192, 8192, 4),
                                         ("dense_fp4_4096", True, 4096, 4096, 4096, 0), ("dense_fp4_8192_fused2", True, 8192, 8192, 8192, 2)]:
            if case and case != name:
                continue
            if fp4:
                Wd = torch.randint(0, 256, (M, K // 2), dtype=torch.uint8, device="cuda") & 0x55
                Ad = torch.randint(0, 256, (N, K // 2), dtype=torch.uint8, device="cuda") & 0x55
            else:
                Wd = torch.randint(-8, 8, (M, K), dtype=torch.int8, device="cuda")
                Ad = torch.randint(0, 16, (N, K), dtype=torch.int8, device="cuda")
            if ob:
                th = thr_for(M, ob)
                Y = torch.empty((ob, N, bs.bs_words_per_row(M)), dtype=torch.int64, device="cuda")
                f = (lambda: bs.bs_gemm_fp4_threshold(Wd, Ad, K, th, ob, out=Y)) if fp4 else (lambda: bs.bs_gemm_i8_threshold(Wd, Ad, K, th, ob, out=Y))
            else:
                C = torch.empty((M, N), dtype=torch.int32, device="cuda")
                f = (lambda: bs.bs_gemm_fp4(Wd, Ad, K, out=C)) if fp4 else (lambda: bs.bs_gemm_i8(Wd, Ad, K, out=C))
            for _ in range(30):
                f()                        # clocks
            run(name, [f], 20)
    elif which == "chain":
        # the W1A2 layers of Table 2 at batch 1 on random planes of their shapes: conv2, pool2, conv3, conv4, conv5, pool5,
        # fc6, fc7 as eight launches, then with the pooling layers folded into conv3 and fc6 (six launches)
        def conv_args(C, F, k):
            return planes(1, F, bs.bs_lowered_depth(C, k, k)), thr_for(F, 2)
        x2 = planes(2, 27 * 27, 96)
        (F2, t2), (F3, t3), (F4, t4), (F5, t5) = conv_args(96, 256, 5), conv_args(256, 384, 3), conv_args(384, 384, 3), conv_args(384, 256, 3)
        W6, t6, W7, t7 = planes(1, 4096, 9216), thr_for(4096, 2), planes(1, 4096, 4096), thr_for(4096, 2)
        y2, p2, y3, y4 = planes(2, 729, 256), planes(2, 169, 256), planes(2, 169, 384), planes(2, 169, 384)
        y5, p5, y6, y7 = planes(2, 169, 256), planes(2, 36, 256), planes(2, 1, 4096), planes(2, 1, 4096)
        eight = [lambda: bs.bs_conv_threshold(x2, U, 27, 27, 96, F2, BP, 5, 5, 1, 2, t2, 2, out=y2),
                 lambda: bs.bs_maxpool_packed(y2, 27, 27, 256, 3, 2, out=p2),
                 lambda: bs.bs_conv_threshold(p2, U, 13, 13, 256, F3, BP, 3, 3, 1, 1, t3, 2, out=y3),
                 lambda: bs.bs_conv_threshold(y3, U, 13, 13, 384, F4, BP, 3, 3, 1, 1, t4, 2, out=y4),
                 lambda: bs.bs_conv_threshold(y4, U, 13, 13, 384, F5, BP, 3, 3, 1, 1, t5, 2, out=y5),
                 lambda: bs.bs_maxpool_packed(y5, 13, 13, 256, 3, 2, out=p5),
                 lambda: bs.bs_gemm_threshold(W6, BP, p5.reshape(2, 1, -1), U, 9216, t6, 2, out=y6),
                 lambda: bs.bs_gemm_threshold(W7, BP, y6, U, 4096, t7, 2, out=y7)]
        six = [eight[0],
               lambda: bs.bs_pool_conv_threshold_batch(y2, 1, 27, 27, 256, 3, 2, F3, BP, 3, 3, 1, 1, t3, 2, out=y3),
               eight[3], eight[4],
               lambda: bs.bs_pool_conv_threshold_batch(y5, 1, 13, 13, 256, 3, 2, W6, BP, 6, 6, 1, 0, t6, 2, out=y6),
               eight[7]]
        run("chain_eight_launches", eight, 200)
        run("chain_six_launches", six, 200)
    else:
        for (name, e, w, a, M, N, K, ob) in [("planes_fp4_W2A2_4096", bs.BS_ENGINE_DENSE_FP4, 2, 2, 4096, 4096, 4096, 0),
                                             ("planes_fp4_W1A2_4096_fused2", bs.BS_ENGINE_DENSE_FP4, 1, 2, 4096, 4096, 4096, 2),
                                             ("planes_int8_W4A4_8192_fused4", bs.BS_ENGINE_DENSE_I8, 4, 4, 8192, 8192, 8192, 4),
                                             ("planes_int8_W2A2_4096", bs.BS_ENGINE_DENSE_I8, 2, 2, 4096, 4096, 4096, 0),
                                             ("bitserial_W2A2_4096", BSER, 2, 2, 4096, 4096, 4096, 0)]:
            if case and case != name:
                continue
            wf = BP if w == 1 else TC
            Wq, Aq = planes(w, M, K), planes(a, N, K)
            if ob:
                th = thr_for(M, ob)
                Y = torch.empty((ob, N, bs.bs_words_per_row(M)), dtype=torch.int64, device="cuda")
                f = lambda: bs.bs_gemm_threshold(Wq, wf, Aq, U, K, th, ob, out=Y, engine=e)
            else:
                C = torch.empty((M, N), dtype=torch.int32, device="cuda")
                f = lambda: bs.bs_gemm(Wq, wf, Aq, U, K, out=C, engine=e)
            for _ in range(30):
                f()
            run(name, [f], 20)
    return res


def timed_graph(fn_list, reps):
    """Average time per call with the calls of `fn_list` (distinct closures, run round-robin)
    captured `reps` times into one HIP graph and replayed: this takes the host's launch
    overhead out of the timing of kernels that run for a few microseconds."""
    import torch
    for f in fn_list:
        f()
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(s):
        with torch.cuda.graph(g, stream=s):
            for i in range(reps):
                fn_list[i % len(fn_list)]()
    torch.cuda.synchronize()
    # replay untimed for about 30 ms first: the capture above leaves the device idle long enough for its clocks
    # to drop, and they come back only after tens of milliseconds of work
    t0 = time.perf_counter()
    g.replay()
    torch.cuda.synchronize()
    once = max(time.perf_counter() - t0, 1e-6)
    for _ in range(min(2000, int(0.03 / once))):
        g.replay()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    rounds = max(5, min(200, int(0.005 / once)))
    e0.record()
    for _ in range(rounds):
        g.replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / (rounds * reps)


def extras(bs, workloads, dev, timed):
    import torch
    out = {}

    def planes(bits, rows, K):
        return torch.randint(-2 ** 62, 2 ** 62, (bits, rows, bs.bs_words_per_row(K)), dtype=torch.int64, device="cuda")

    def thr_for(Mrows, obits):
        T = (1 << obits) - 1
        return torch.sort(torch.randint(-1000, 1000, (Mrows, T), dtype=torch.int32, device="cuda"), dim=1)[0].contiguous()

    BSER = bs.BS_ENGINE_BITSERIAL

    def fused(name, w, wf, a, af, M, N, K, obits, copies=1, reps=None, stream_probe=False):
        # `copies` distinct weight buffers are cycled through so that the weights of a small
        # layer do not simply sit in the last-level cache (256 MB) from the previous launch.
        # These rows time the AND-popcount kernels (engine named explicitly).
        Wps = [planes(w, M, K) for _ in range(copies)]
        Ap, th = planes(a, N, K), thr_for(M, obits)
        Y = torch.empty((obits, N, bs.bs_words_per_row(M)), dtype=torch.int64, device="cuda")
        fns = [(lambda Wp=Wp: bs.bs_gemm_threshold(Wp, wf, Ap, af, K, th, obits, out=Y, engine=BSER)) for Wp in Wps]
        work = 2.0 * M * N * K
        if work > 1e12:                       # long kernels: plain back-to-back launches
            ms, _ = timed(fns[0], 10, 2)
        else:
            ms = timed_graph(fns, reps or max(2 * copies, 20))
        byts = (w * M + a * N) * bs.bs_words_per_row(K) * 8 + th.numel() * 4 + Y.numel() * 8
        out[name] = {"us": round(ms * 1e3, 2), "GOPS": round(work / ms / 1e6, 1),
                     "frac_of_valu_popcount_peak": round(w * a * work / (ms * 1e-3) / 1e12 / BINARY_PEAK_TOPS, 4),
                     "GBps": round(byts / ms / 1e6, 1), "frac_of_hbm_peak": round(byts / ms / 1e6 / HBM_PEAK_GBS, 4),
                     "weight_buffers_cycled": copies, "weight_bytes_cycled": copies * Wps[0].numel() * 8}
        if stream_probe:
            # the measured floor: a plain streaming read of the same weight buffers, cycled the same way (the
            # shortest time in which a kernel of this library brings that many bytes in from where they lie)
            sink = torch.zeros(1024, dtype=torch.int32, device="cuda")
            for nt in (False, True):
                pf = [(lambda Wp=Wp: bs.bs_probe_stream_read(Wp, sink, non_temporal=nt)) for Wp in Wps]
                pms = timed_graph(pf, reps or max(2 * copies, 20))
                out[name]["stream_read_of_the_weights_us" + ("_nontemporal" if nt else "")] = round(pms * 1e3, 2)

    BP, U, TC = bs.BS_BIPOLAR, bs.BS_UNSIGNED, bs.BS_TWOS_COMPLEMENT
    # "cold": more weight bytes cycled than the 256 MiB last-level cache holds (432, 384 and 384 MiB)
    fused("fc6_W1A2_4096x9216x1_cold", 1, BP, 2, U, 4096, 1, 9216, 2, copies=96, stream_probe=True)
    fused("fc7_W1A2_4096x4096x1_cold", 1, BP, 2, U, 4096, 1, 4096, 2, copies=192, stream_probe=True)
    fused("fc6_W1A2_4096x9216x1_warm", 1, BP, 2, U, 4096, 1, 9216, 2, copies=1)
    fused("conv2_W1A2_256x2400x729", 1, BP, 2, U, 256, 729, 2400, 2)
    fused("W4A4_8192x8192x1_cold", 4, TC, 4, U, 8192, 1, 8192, 4, copies=12, stream_probe=True)
    fused("W4A4_8192x8192x1_warm", 4, TC, 4, U, 8192, 1, 8192, 4, copies=1, stream_probe=True)
    for n in (64, 1024, 8192):
        fused("W4A4_8192x8192x%d" % n, 4, TC, 4, U, 8192, n, 8192, 4)
    # compute-bound rate against precision (Sec. 4.1.1 of the paper lists W1A1, W1A2, W1A3, W2A2, W2A3): 4096^3,
    # int32 output, unsigned activations, bipolar (1-bit) or two's-complement weights
    sweep_p = {}
    for (w_, a_) in [(1, 1), (1, 2), (1, 3), (2, 2), (2, 3), (3, 3), (4, 4)]:
        Wq, Aq = planes(w_, 4096, 4096), planes(a_, 4096, 4096)
        Cq = torch.empty((4096, 4096), dtype=torch.int32, device="cuda")
        wf_ = BP if w_ == 1 else TC
        ms, _ = timed(lambda: bs.bs_gemm(Wq, wf_, Aq, U, 4096, out=Cq, engine=BSER), 10, 3)
        gops = 2.0 * 4096 ** 3 / ms / 1e6
        sweep_p["W%dA%d" % (w_, a_)] = {"us": round(ms * 1e3, 1), "GOPS": round(gops, 1), "GOPS_x_w_x_a": round(gops * w_ * a_, 1),
                                        "frac_of_valu_popcount_peak": round(gops * w_ * a_ / 1e3 / BINARY_PEAK_TOPS, 4)}
    out["precision_sweep_4096x4096x4096"] = sweep_p
    # a GEMV large enough that launch and first-byte latency stop mattering
    fused("W1A2_32768x32768x1_cold", 1, BP, 2, U, 32768, 1, 32768, 2, copies=3, reps=12, stream_probe=True)
    # The per-layer choice of Sec. 4.1.1 / 4.2 as the library makes it on PACKED PLANES: the same call on the
    # AND-popcount kernels, on the two matrix-core kernels that expand plane bits in their loader, and as bs_gemm /
    # bs_gemm_threshold pick by themselves; beside them the matrix-core kernels on operands unpacked beforehand
    # (bs_gemm_fp4 / bs_gemm_i8: the caller's buffers, unpack time not counted).
    eng = {}
    names = {bs.BS_ENGINE_BITSERIAL: "bitserial", bs.BS_ENGINE_DENSE_I8: "dense_int8", bs.BS_ENGINE_DENSE_FP4: "dense_fp4",
             bs.BS_ENGINE_AUTO: "auto"}
    for (w_, a_, M_, N_, K_, ob_) in [(2, 2, 4096, 4096, 4096, 0), (2, 2, 4096, 4096, 4096, 2), (1, 2, 4096, 4096, 4096, 2),
                                       (1, 1, 4096, 4096, 4096, 0), (4, 4, 8192, 8192, 8192, 4), (4, 4, 8192, 1024, 8192, 4),
                                       (4, 4, 8192, 64, 8192, 4), (1, 2, 384, 10816, 2304, 2), (2, 2, 1024, 1024, 4096, 2)]:
        wf_ = BP if w_ == 1 else TC
        af_ = BP if (w_ == 1 and a_ == 1) else U
        Wq, Aq = planes(w_, M_, K_), planes(a_, N_, K_)
        if ob_:
            th_ = thr_for(M_, ob_)
            Yq = torch.empty((ob_, N_, bs.bs_words_per_row(M_)), dtype=torch.int64, device="cuda")
            call = lambda e: bs.bs_gemm_threshold(Wq, wf_, Aq, af_, K_, th_, ob_, out=Yq, engine=e)
        else:
            Cq = torch.empty((M_, N_), dtype=torch.int32, device="cuda")
            call = lambda e: bs.bs_gemm(Wq, wf_, Aq, af_, K_, out=Cq, engine=e)
        row = {}
        engines = [bs.BS_ENGINE_BITSERIAL, bs.BS_ENGINE_DENSE_I8] + ([bs.BS_ENGINE_DENSE_FP4] if max(w_, a_) <= 2 else []) \
            + [bs.BS_ENGINE_AUTO]
        for e in engines:
            if 2.0 * M_ * N_ * K_ * (w_ * a_ if e == bs.BS_ENGINE_BITSERIAL else 1) > 2e12:
                ms_e, _ = timed(lambda: call(e), 5, 2)
            else:
                ms_e = timed_graph([lambda: call(e)], 10)
            row[names[e] + "_us"] = round(ms_e * 1e3, 2)
        row["auto_picks"] = names[bs.bs_choose_engine(w_, wf_, a_, af_, M_, N_, K_)]
        # reference: the same product from operands unpacked beforehand into the caller's buffers
        if max(w_, a_) <= 2:
            W4q, A4q = bs.bs_unpack_planes_fp4(Wq, wf_, K_), bs.bs_unpack_planes_fp4(Aq, af_, K_)
            ref = (lambda: bs.bs_gemm_fp4_threshold(W4q, A4q, K_, th_, ob_, out=Yq)) if ob_ else (lambda: bs.bs_gemm_fp4(W4q, A4q, K_, out=Cq))
            row["dense_fp4_on_unpacked_operands_us"] = round(timed_graph([ref], 10) * 1e3, 2)
            del W4q, A4q
        else:
            W8q, A8q = bs.bs_unpack_planes(Wq, wf_, K_), bs.bs_unpack_planes(Aq, af_, K_)
            ref = (lambda: bs.bs_gemm_i8_threshold(W8q, A8q, K_, th_, ob_, out=Yq)) if ob_ else (lambda: bs.bs_gemm_i8(W8q, A8q, K_, out=Cq))
            row["dense_int8_on_unpacked_operands_us"] = round((timed(ref, 5, 2)[0] if 2.0 * M_ * N_ * K_ > 2e12 else timed_graph([ref], 10)) * 1e3, 2)
            del W8q, A8q
        best = min((v, k) for k, v in row.items() if k.endswith("_us") and "unpacked" not in k and not k.startswith("auto"))
        row["fastest_on_planes"] = best[1][:-3]
        flops = 2.0 * M_ * N_ * K_
        row["auto_GOPS"] = round(flops / row["auto_us"] / 1e3, 1)
        eng["W%dA%d_%dx%dx%d_%s" % (w_, a_, M_, K_, N_, ("fused_%dbit_out" % ob_) if ob_ else "int32_out")] = row
        del Wq, Aq
    out["engines_on_packed_planes"] = eng
    # the W1A2 layers of the paper's AlexNet (Table 2) as one packed chain, batch 1:
    # conv2 (fused lowering + GEMM + thresholds) -> pool -> conv3 -> conv4 -> conv5 -> pool -> fc6 -> fc7
    xin, layers = workloads.alexnet_inner()
    H0, W0, C0 = xin.shape
    x0 = bs.bs_pack_planes(dev(xin.reshape(H0 * W0, C0)), 2, U)
    prepared = []
    for L in layers:
        if L["kind"] == "conv":
            F = L["geom"][3]
            prepared.append((L, bs.bs_pack_planes(dev(L["filt"].reshape(F, -1)), 1, BP), dev(L["thr"])))
        elif L["kind"] == "fc":
            prepared.append((L, bs.bs_pack_planes(dev(L["W"]), 1, BP), dev(L["thr"])))
        else:
            prepared.append((L, None, None))

    def frame():
        cur = x0
        for L, Wp, th in prepared:
            if L["kind"] == "conv":
                H, W, C, F, k, s, p = L["geom"]
                cur = bs.bs_conv_threshold(cur, U, H, W, C, Wp, BP, k, k, s, p, th, 2, out=L.setdefault(
                    "_out", torch.empty((2, ((H + 2 * p - k) // s + 1) ** 2, bs.bs_words_per_row(F)), dtype=torch.int64, device="cuda")))
            elif L["kind"] == "pool":
                H, W, C, k, s = L["geom"]
                cur = bs.bs_maxpool_packed(cur, H, W, C, k, s, out=L.setdefault(
                    "_out", torch.empty((2, ((H - k) // s + 1) ** 2, bs.bs_words_per_row(C)), dtype=torch.int64, device="cuda")))
            else:
                M, K = L["geom"]
                cur = bs.bs_gemm_threshold(Wp, BP, cur.reshape(2, 1, -1), U, K, th, 2, out=L.setdefault(
                    "_out", torch.empty((2, 1, bs.bs_words_per_row(M)), dtype=torch.int64, device="cuda")))
        return cur
    ms = timed_graph([frame], 20)
    # every layer alone on the input the chain gives it (Table 2's rows; lowering is inside the convolution kernels)
    def one_layer(L, Wp, th, cur):
        if L["kind"] == "conv":
            H, W, C, F, k, s, p = L["geom"]
            return lambda: bs.bs_conv_threshold(cur, U, H, W, C, Wp, BP, k, k, s, p, th, 2, out=L["_out"])
        if L["kind"] == "pool":
            H, W, C, k, s = L["geom"]
            return lambda: bs.bs_maxpool_packed(cur, H, W, C, k, s, out=L["_out"])
        return lambda: bs.bs_gemm_threshold(Wp, BP, cur.reshape(2, 1, -1), U, L["geom"][1], th, 2, out=L["_out"])
    per_layer, cur = {}, x0
    for L, Wp, th in prepared:
        per_layer[L["name"]] = round(timed_graph([one_layer(L, Wp, th, cur)], 20) * 1e3, 2)
        cur = L["_out"]
    # the two pooling layers folded into their consumers' operand fetch: conv3 reads pool2's windows, fc6 (a convolution
    # whose kernel is the whole pooled map) reads pool5's; six launches, same result
    def frame_folded(alone=None):
        cur, pool, calls = x0, None, []
        for L, Wp, th in prepared:
            if L["kind"] == "pool":
                pool = L["geom"]
                continue
            if L["kind"] == "conv":
                H, W, C, F, k, s, p = L["geom"]
                if pool is not None:
                    f = (lambda cur=cur, pool=pool, Wp=Wp, th=th, L=L, k=k, s=s, p=p:
                         bs.bs_pool_conv_threshold_batch(cur, 1, pool[0], pool[1], pool[2], pool[3], pool[4], Wp, BP, k, k, s, p, th, 2, out=L["_out"]))
                else:
                    f = (lambda cur=cur, Wp=Wp, th=th, L=L, H=H, W=W, C=C, k=k, s=s, p=p:
                         bs.bs_conv_threshold(cur, U, H, W, C, Wp, BP, k, k, s, p, th, 2, out=L["_out"]))
            else:
                M, K = L["geom"]
                if pool is not None:
                    PH = (pool[0] - pool[3]) // pool[4] + 1
                    f = (lambda cur=cur, pool=pool, Wp=Wp, th=th, L=L, PH=PH:
                         bs.bs_pool_conv_threshold_batch(cur, 1, pool[0], pool[1], pool[2], pool[3], pool[4], Wp, BP, PH, PH, 1, 0, th, 2, out=L["_out"]))
                else:
                    f = (lambda cur=cur, Wp=Wp, th=th, L=L, K=K:
                         bs.bs_gemm_threshold(Wp, BP, cur.reshape(2, 1, -1), U, K, th, 2, out=L["_out"]))
            calls.append((L["name"] + ("_reading_pooled_input" if pool is not None else ""), f))
            cur, pool = L["_out"], None
        return calls
    want_last = frame().clone()
    folded = frame_folded()
    def run_folded():
        for _, f in folded:
            f()
    run_folded()
    torch.cuda.synchronize()
    folded_same = bool(torch.equal(prepared[-1][0]["_out"], want_last))
    ms_folded = timed_graph([run_folded], 20)
    per_layer_folded = {name: round(timed_graph([f], 20) * 1e3, 2) for name, f in folded if name.endswith("pooled_input")}
    out["alexnet_W1A2_layers_conv2_to_fc7_chain"] = {
        "us_per_frame": round(ms * 1e3, 2), "frames_per_s": round(1e3 / ms, 1), "kernels_per_frame": len(prepared),
        "us_per_layer_alone": per_layer,
        "pooling_folded_into_consumers": {"us_per_frame": round(ms_folded * 1e3, 2), "frames_per_s": round(1e3 / ms_folded, 1),
                                          "kernels_per_frame": len(folded), "same_output": folded_same,
                                          "us_per_fused_layer_alone": per_layer_folded},
        "context": "the same layers (lowering + GEMM rows of Table 2, bsgemm-intl column) sum to 55.1 ms on the "
                   "paper's Cortex-A57 core; synthetic weights here"}
    # the same chain on a batch of images (columns = batch x pixels): throughput instead of latency.  Once with the
    # AND-popcount engine named for every layer, once as the library chooses per layer (Sec. 4.2: "choosing the execution
    # method for each layer"); lowering happens inside the kernels on either engine.
    names = {bs.BS_ENGINE_BITSERIAL: "bitserial", bs.BS_ENGINE_DENSE_I8: "dense_int8", bs.BS_ENGINE_DENSE_FP4: "dense_fp4"}
    for Bn in (16, 64, 256):
        xb = torch.randint(0, 4, (Bn * H0 * W0, C0), dtype=torch.int8, device="cuda")
        xbp = bs.bs_pack_planes(xb, 2, U)
        bufs = {}

        def frame_batch(engine):
            cur = xbp
            for L, Wp, th in prepared:
                key = (L["name"], Bn)
                if L["kind"] == "conv":
                    H, W, C, F, k, s, p = L["geom"]
                    OHW = ((H + 2 * p - k) // s + 1) ** 2
                    cur = bs.bs_conv_threshold_batch(cur, U, Bn, H, W, C, Wp, BP, k, k, s, p, th, 2, engine=engine, out=bufs.setdefault(
                        key, torch.empty((2, Bn * OHW, bs.bs_words_per_row(F)), dtype=torch.int64, device="cuda")))
                elif L["kind"] == "pool":
                    H, W, C, k, s = L["geom"]
                    OHW = ((H - k) // s + 1) ** 2
                    cur = bs.bs_maxpool_packed_batch(cur, Bn, H, W, C, k, s, out=bufs.setdefault(
                        key, torch.empty((2, Bn * OHW, bs.bs_words_per_row(C)), dtype=torch.int64, device="cuda")))
                else:
                    M, K = L["geom"]
                    cur = bs.bs_gemm_threshold(Wp, BP, cur.reshape(2, Bn, -1), U, K, th, 2, engine=engine, out=bufs.setdefault(
                        key, torch.empty((2, Bn, bs.bs_words_per_row(M)), dtype=torch.int64, device="cuda")))
            return cur
        want = frame_batch(BSER).clone()
        same = bool((frame_batch(bs.BS_ENGINE_AUTO) == want).all())
        msb = timed_graph([lambda: frame_batch(BSER)], 10)
        msc = timed_graph([lambda: frame_batch(bs.BS_ENGINE_AUTO)], 10)
        picks = {}
        for L, Wp, th in prepared:
            if L["kind"] == "conv":
                H, W, C, F, k, s, p = L["geom"]
                picks[L["name"]] = names[bs.bs_choose_engine(1, BP, 2, U, F, Bn * ((H + 2 * p - k) // s + 1) ** 2, bs.bs_lowered_depth(C, k, k))]
            elif L["kind"] == "fc":
                picks[L["name"]] = names[bs.bs_choose_engine(1, BP, 2, U, L["geom"][0], Bn, L["geom"][1])]
        out["alexnet_W1A2_layers_conv2_to_fc7_chain_batch_%d" % Bn] = {
            "bitserial_engine": {"us_per_batch": round(msb * 1e3, 2), "frames_per_s": round(Bn * 1e3 / msb, 1)},
            "engine_chosen_per_layer": {"us_per_batch": round(msc * 1e3, 2), "frames_per_s": round(Bn * 1e3 / msc, 1),
                                        "engine": picks, "same_output_as_bitserial_chain": same}}
        del xb, xbp, bufs
    # the dense (int8 MFMA) engine on the compute-bound configurations, beside the bit-serial
    # numbers above: same logical product, operands unpacked to int8
    def dense(name, M, N, K, obits):
        Wd = torch.randint(-8, 8, (M, K), dtype=torch.int8, device="cuda")
        Ad = torch.randint(0, 16, (N, K), dtype=torch.int8, device="cuda")
        th = thr_for(M, obits) if obits else None
        if obits:
            Y = torch.empty((obits, N, bs.bs_words_per_row(M)), dtype=torch.int64, device="cuda")
            f = lambda: bs.bs_gemm_i8_threshold(Wd, Ad, K, th, obits, out=Y)
        else:
            Cd = torch.empty((M, N), dtype=torch.int32, device="cuda")
            f = lambda: bs.bs_gemm_i8(Wd, Ad, K, out=Cd)
        ms, _ = timed(f, 10, 3)
        tops = 2.0 * M * N * K / (ms * 1e-3) / 1e12
        out[name] = {"us": round(ms * 1e3, 2), "GOPS": round(tops * 1e3, 1),
                     "roofline": {"bound": "mfma", "achieved": round(tops, 1), "peak": 5000.0, "unit": "int8 TOP/s",
                                  "frac": round(tops / 5000.0, 4)}}
    dense("dense_engine_4096x4096x4096_int32_out", 4096, 4096, 4096, 0)
    dense("dense_engine_8192x8192x8192_fused_4bit_out", 8192, 8192, 8192, 4)
    dense("dense_engine_8192x8192x1024_fused_4bit_out", 8192, 1024, 8192, 4)
    Wp2 = planes(2, 4096, 4096)
    W8 = torch.empty((4096, 4096), dtype=torch.int8, device="cuda")
    ms = timed_graph([lambda: bs.bs_unpack_planes(Wp2, TC, 4096, out=W8)], 20)
    out["unpack_4096x4096_2_planes_to_i8"] = {"us": round(ms * 1e3, 2),
                                              "GBps": round((Wp2.numel() * 8 + W8.numel()) / ms / 1e6, 1)}
    # the fp4 flavour of the dense engine (operands of at most 2 bits as E2M1 codes, twice the int8 MFMA rate)
    def dense_fp4(name, M, N, K, obits):
        Wd = torch.randint(0, 256, (M, K // 2), dtype=torch.uint8, device="cuda") & 0x55   # nibbles 0, 1, 4, 5: 0, 0.5, 2, 3
        Ad = torch.randint(0, 256, (N, K // 2), dtype=torch.uint8, device="cuda") & 0x55
        if obits:
            th = thr_for(M, obits)
            Y = torch.empty((obits, N, bs.bs_words_per_row(M)), dtype=torch.int64, device="cuda")
            f = lambda: bs.bs_gemm_fp4_threshold(Wd, Ad, K, th, obits, out=Y)
        else:
            Cd = torch.empty((M, N), dtype=torch.int32, device="cuda")
            f = lambda: bs.bs_gemm_fp4(Wd, Ad, K, out=Cd)
        ms, _ = timed(f, 10, 3)
        tops = 2.0 * M * N * K / (ms * 1e-3) / 1e12
        out[name] = {"us": round(ms * 1e3, 2), "GOPS": round(tops * 1e3, 1),
                     "roofline": {"bound": "mfma", "achieved": round(tops, 1), "peak": 10100.0, "unit": "fp4 TFLOP/s",
                                  "frac": round(tops / 10100.0, 4)}}
    dense_fp4("dense_fp4_engine_4096x4096x4096_int32_out", 4096, 4096, 4096, 0)
    dense_fp4("dense_fp4_engine_8192x8192x8192_fused_2bit_out", 8192, 8192, 8192, 2)
    # stand-alone thresholding of a large int32 result (the unfused route of S5)
    Cbig = torch.randint(-40000, -20000, (8192, 8192), dtype=torch.int32, device="cuda")
    thb = thr_for(8192, 4) - 30000
    Yb = torch.empty((4, 8192, bs.bs_words_per_row(8192)), dtype=torch.int64, device="cuda")
    ms = timed_graph([lambda: bs.bs_threshold_activate(Cbig, thb, 4, out=Yb)], 10)
    byts = Cbig.numel() * 4 + Yb.numel() * 8 + thb.numel() * 4
    out["threshold_activate_8192x8192_4bit"] = {"us": round(ms * 1e3, 2), "GBps": round(byts / ms / 1e6, 1),
                                                "frac_of_hbm_peak": round(byts / ms / 1e6 / HBM_PEAK_GBS, 4)}
    del Cbig, Yb
    # interleaved lowering of conv2 alone, and the two pack kernels
    x = planes(2, 27 * 27, 96)
    low = torch.empty((2, 729, bs.bs_words_per_row(2400)), dtype=torch.int64, device="cuda")
    ms = timed_graph([lambda: bs.bs_im2col_interleaved(x, 27, 27, 96, 5, 5, 1, 2, out=low)], 50)
    out["conv2_interleaved_lowering"] = {"us": round(ms * 1e3, 2),
                                         "GBps": round((low.numel() * 8 + x.numel() * 8) / ms / 1e6, 1)}
    X = torch.randint(0, 4, (8192, 8192), dtype=torch.int8, device="cuda")
    P = torch.empty((2, 8192, bs.bs_words_per_row(8192)), dtype=torch.int64, device="cuda")
    for strided in (False, True):
        ms = timed_graph([lambda: bs.bs_pack_planes(X, 2, U, depth_is_strided=strided, out=P)], 20)
        byts = X.numel() + P.numel() * 8
        out["pack_8192x8192_i8_to_2_planes_%s" % ("depth_strided" if strided else "depth_contiguous")] = {
            "us": round(ms * 1e3, 2), "GBps": round(byts / ms / 1e6, 1), "frac_of_hbm_peak": round(byts / ms / 1e6 / HBM_PEAK_GBS, 4)}
    return out


if __name__ == "__main__":
    sys.exit(main())
