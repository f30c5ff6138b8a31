"""Benchmark of the W4A4 DSFQ linear path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 5] [--bits 4] [--matrix-path e2m3] [--no-cpu-baseline]

A step is one pass of the whole online path (rotate + smooth + per-token quantize, int4 x int4 GEMM,
dequant + bias epilogue) over every layer of the chosen synthetic config, inputs resident in HBM.
At 4 bits the default matrix path writes the codes as E2M3 numbers and multiplies them on the 6-bit
floating-point matrix instructions (qvggt_linear_e2m3: the same integer sums and outputs, bit for bit,
as the int8-instruction path qvggt_linear, which --matrix-path int8 times as the headline and the default
run reports beside it as "w4a4_int8_path").  Prints one JSON line.  The default workload is the benchmark's configs[4]
(fc1 and fc2 of the VGGT-1B MLP at 100 frames), the largest single-GPU configuration and the
one the throughput targets are stated on.  --bits 8 / 6 time the same layers in the 8-bit / 6-bit setting (int8
codes in 128-row blocks, qvggt_linear_i8b); the default 4-bit run also reports the 8-bit setting as a side measurement
("w8a8", and "w8a8_row_major" for the same setting on row-major codes).

Beside the headline (exactly K steps after W warm-up steps; by default 200 after 50, about a quarter of a second of work, so
that the figure is a steady-state one) the line carries: the same step repeated back to back for
about two seconds ("sustained": the board settles under its power limit), mean / median / min per kernel from HIP events,
machine ceilings measured in the run ("ceilings": an elementwise copy, register-only loops of the two matrix instructions),
the other single-GPU configurations in short ("other_configs"), and the CPU oracle timed per stage on all cores and on one.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
INT8_PEAK_TOPS = 5000.0      # MI355X dense int8 MFMA, published (5.0 POP/s)
FP6_PEAK_TOPS = 10100.0      # MI355X dense fp6 MFMA, published (10.1 PFLOP/s)
METRIC = "W4A4 GEMM TOPS (% int8 MFMA peak) + rotate-quant GB/s at VGGT-1B shapes"


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--config", type=int, default=5, choices=[2, 3, 4, 5])
    ap.add_argument("--bits", type=int, default=4, choices=[4, 6, 8], help="quantization setting timed as the headline")
    ap.add_argument("--matrix-path", default="e2m3", choices=["e2m3", "int8"],
                    help="4-bit setting: codes as E2M3 numbers on the 6-bit floating-point matrix instructions, or on the int8 ones")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--headline-only", action="store_true",
                    help="skip the side measurements (8-bit setting, calibration reductions, other configs): what the profiles under profiles/ are taken with")
    ap.add_argument("--sustain-seconds", type=float, default=2.0, help="length of the back-to-back leg reported as 'sustained' (0: skip)")
    ap.add_argument("--cpu-rows", type=int, default=16384, help="rows per layer the oracle is timed on with all cores")
    ap.add_argument("--cpu-rows-1thread", type=int, default=1024, help="rows per layer the oracle is timed on with one thread (0: skip)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run plain 1 GiB device copies (reference dispatches for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU; every step of the path is row-independent and would "
              "shard by tokens with no collective, but multi-GPU runs are not part of it (use --gpus 1)",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2509_21302_amd as q
    import synth

    q.load_library()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)
    q.qvggt_init()

    def to_dev(a):
        if a is None:
            return None
        a = np.ascontiguousarray(a)
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)
        return torch.from_numpy(a).to(dev)

    # ------------------------------------------------------------------ set-up (untimed)
    wide_bits = args.bits if args.bits != 4 else 8        # the width the int8-code path runs at (headline, or the side measurement)

    def build_layers(config, bit_settings):
        layers = []
        for name in synth.config_layers(config):
            s = synth.layer_spec(config, name)
            signs = to_dev(synth.make_signs(s))
            a = torch.empty(s.K, dtype=torch.float32, device=dev)
            q.qvggt_rotated_col_absmax(to_dev(synth.make_calibration(s)), signs, a)
            Wd = to_dev(synth.make_weights(s))
            X = to_dev(synth.make_activation_frames(s, workers=16))
            L = dict(spec=s, signs=signs, bias=to_dev(synth.make_bias(s)), X=X,
                     Y=torch.empty(s.M, s.N, dtype=torch.bfloat16, device=dev),
                     ws=torch.empty(max(q.qvggt_workspace_bytes_i8(s.M, s.N, s.K), q.qvggt_workspace_bytes_i8b(s.M, s.N, s.K)),
                                    dtype=torch.uint8, device=dev),
                     Xq=torch.empty(q.qvggt_i8b_bytes(s.M, s.K), dtype=torch.uint8, device=dev),   # sized for int8 blocks; the others use less
                     sx=torch.empty(s.M, dtype=torch.float32, device=dev), prep={})
            L["Xq4"] = L["Xq"].view(-1)[: s.M * s.K // 2].view(s.M, s.K // 2)
            L["Xq8"] = L["Xq"][: s.M * s.K].view(s.M, s.K).view(torch.int8)
            L["Xb"] = L["Xq"].view(torch.int8)                                  # int8 blocks: rows padded to 128
            L["Xf"] = L["Xq"].view(-1)[: q.qvggt_e2m3_bytes(s.M, s.K)]          # E2M3 blocks: 3/4 byte per code, rows padded to 128
            assert L["Xf"].numel() == q.qvggt_e2m3_bytes(s.M, s.K) and L["ws"].numel() >= q.qvggt_workspace_bytes_e2m3(s.M, s.N, s.K)
            for bits in sorted(bit_settings):
                sw = torch.empty(s.N, dtype=torch.float32, device=dev)
                inv = torch.empty(s.K, dtype=torch.float32, device=dev)
                if bits == 4:
                    Wq = torch.empty(s.N, s.K // 2, dtype=torch.uint8, device=dev)
                    q.qvggt_prep_weights(Wd, a, signs, 0.5, Wq, sw, inv)
                else:
                    Wq = torch.empty(s.N, s.K, dtype=torch.int8, device=dev)
                    q.qvggt_prep_weights_i8(Wd, a, signs, 0.5, bits, Wq, sw, inv)
                L["prep"][bits] = dict(Wq=Wq, sw=sw, inv=inv)
                if bits == wide_bits:
                    Wb = torch.empty(q.qvggt_i8b_bytes(s.N, s.K), dtype=torch.int8, device=dev)
                    q.qvggt_int8_to_blocks(Wq, s.N, s.K, Wb)
                    L["prep"]["i8b"] = dict(Wq=Wb, sw=sw, inv=inv)
                if bits == 4:
                    Wf = torch.empty(q.qvggt_e2m3_bytes(s.N, s.K), dtype=torch.uint8, device=dev)
                    lost = torch.zeros(1, dtype=torch.int32, device=dev)
                    q.qvggt_codes_to_e2m3(Wq, s.N, s.K, Wf, lost)
                    assert int(lost.item()) == 0, "weight codes -8 have no E2M3 value"
                    L["prep"]["e2m3"] = dict(Wq=Wf, sw=sw, inv=inv)
            layers.append(L)
        torch.cuda.synchronize()
        return layers

    layers = build_layers(args.config, {args.bits} if args.headline_only else {args.bits, 4, 8})

    def linear(L, bits):
        P = L["prep"][bits]
        if bits == "e2m3":
            q.qvggt_linear_e2m3(L["X"], L["signs"], P["inv"], P["Wq"], P["sw"], L["bias"], L["Y"], L["ws"])
        elif bits == "i8b":
            q.qvggt_linear_i8b(L["X"], L["signs"], P["inv"], wide_bits, P["Wq"], P["sw"], L["bias"], L["Y"], L["ws"])
        elif bits == 4:
            q.qvggt_linear(L["X"], L["signs"], P["inv"], P["Wq"], P["sw"], L["bias"], L["Y"], L["ws"])
        else:
            q.qvggt_linear_i8(L["X"], L["signs"], P["inv"], bits, P["Wq"], P["sw"], L["bias"], L["Y"], L["ws"])

    def rotate_quant(L, bits):
        P = L["prep"][bits]
        if bits == "e2m3":
            q.qvggt_rotate_smooth_quant_e2m3(L["X"], L["signs"], P["inv"], L["Xf"], L["sx"])
        elif bits == "i8b":
            q.qvggt_rotate_smooth_quant_i8b(L["X"], L["signs"], P["inv"], wide_bits, L["Xb"], L["sx"])
        elif bits == 4:
            q.qvggt_rotate_smooth_quant(L["X"], L["signs"], P["inv"], L["Xq4"], L["sx"])
        else:
            q.qvggt_rotate_smooth_quant_i8(L["X"], L["signs"], P["inv"], bits, L["Xq8"], L["sx"])

    def gemm(L, bits):
        P, s = L["prep"][bits], L["spec"]
        if bits == "e2m3":
            q.qvggt_e2m3_gemm(L["Xf"], L["sx"], P["Wq"], P["sw"], L["bias"], s.M, s.N, s.K, L["Y"], None)
        elif bits == "i8b":
            q.qvggt_i8b_gemm(L["Xb"], L["sx"], P["Wq"], P["sw"], L["bias"], s.M, s.N, s.K, L["Y"], None)
        elif bits == 4:
            q.qvggt_w4a4_gemm(L["Xq4"], L["sx"], P["Wq"], P["sw"], L["bias"], s.M, s.N, s.K, L["Y"], None)
        else:
            q.qvggt_i8_gemm(L["Xq8"], L["sx"], P["Wq"], P["sw"], L["bias"], s.M, s.N, s.K, L["Y"], None)

    def blocks_ok_for(ls):
        # the blocked operand formats are defined for the bf16 kernel-1 shapes; elsewhere the int8-code path runs on row-major codes
        return all(L["spec"].x_dtype == "bf16" and L["spec"].K in (1024, 2048, 4096) for L in ls)

    blocks_ok = blocks_ok_for(layers)
    if args.bits == 4:
        headline = "e2m3" if (args.matrix_path == "e2m3" and blocks_ok) else 4
    else:
        headline = "i8b" if blocks_ok else args.bits

    def ops_of(ls):
        return sum(2.0 * L["spec"].M * L["spec"].N * L["spec"].K for L in ls)

    def timed_steps(ls, bits, n):
        """n back-to-back steps, bracketed by synchronisation on both sides: wall seconds"""
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            for L in ls:
                linear(L, bits)
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    # ------------------------------------------------------------------ timed region: whole path, exactly K steps after W warm-up steps
    timed_steps(layers, headline, args.warmup)
    elapsed = timed_steps(layers, headline, args.steps)
    ms_per_step = elapsed * 1e3 / args.steps
    ops_per_step = ops_of(layers)
    value = ops_per_step / (ms_per_step * 1e-3) / 1e12

    # the same step back to back for about sustain-seconds: what the rate is once the board has settled under its power limit
    sustained = None
    if args.sustain_seconds > 0:
        n_sus = max(args.steps, int(args.sustain_seconds / (ms_per_step * 1e-3)) + 1)
        el = timed_steps(layers, headline, n_sus)
        sustained = dict(steps=n_sus, seconds=el, ms_per_step=el * 1e3 / n_sus, value_TOPS=ops_per_step / (el / n_sus) / 1e12,
                         ratio_to_headline=(ms_per_step * 1e-3) / (el / n_sus))

    # ------------------------------------------------------------------ per-kernel durations (HIP events on the launch stream)
    # same kernels, same arguments, launched through the two single-kernel entry points so that events can sit between them
    def per_kernel(ls, bits, steps):
        ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
               for _ in ls] for _ in range(steps)]
        for k in range(steps):
            for L, (e0, e1, e2) in zip(ls, ev[k]):
                e0.record()
                rotate_quant(L, bits)
                e1.record()
                gemm(L, bits)
                e2.record()
        torch.cuda.synchronize()
        per_layer = {}
        rq_ms_all, gemm_ms_all, rq_bytes_all, rq_method_bytes_all, gemm_ops_all = 0.0, 0.0, 0.0, 0.0, 0.0
        for i, L in enumerate(ls):
            s = L["spec"]
            rqs = np.array([ev[k][i][0].elapsed_time(ev[k][i][1]) for k in range(steps)])
            gms = np.array([ev[k][i][1].elapsed_time(ev[k][i][2]) for k in range(steps)])
            rq, gm = float(rqs.mean()), float(gms.mean())
            x_bytes = 2 if s.x_dtype == "bf16" else 4
            code_bytes = {"e2m3": 0.75, 4: 0.5}.get(bits, 1.0)
            rq_bytes = s.M * (x_bytes * s.K + s.K * code_bytes + 4)                           # what this kernel moves: X in, codes out (as stored), step out
            rq_method_bytes = s.M * (x_bytes * s.K + s.K * (0.5 if bits in ("e2m3", 4) else 1.0) + 4)   # the method's bytes: a 4-bit code is half a byte
            gemm_ops = 2.0 * s.M * s.N * s.K
            per_layer[s.name] = dict(M=s.M, K=s.K, N=s.N,
                                     rotate_quant_ms=rq, rotate_quant_ms_median=float(np.median(rqs)), rotate_quant_ms_min=float(rqs.min()),
                                     rotate_quant_GBps=rq_method_bytes / rq / 1e6, rotate_quant_GBps_own_bytes=rq_bytes / rq / 1e6,
                                     gemm_ms=gm, gemm_ms_median=float(np.median(gms)), gemm_ms_min=float(gms.min()),
                                     gemm_TOPS=gemm_ops / gm / 1e9)
            rq_ms_all += rq; gemm_ms_all += gm; rq_bytes_all += rq_bytes; rq_method_bytes_all += rq_method_bytes; gemm_ops_all += gemm_ops
        return per_layer, rq_ms_all, gemm_ms_all, rq_bytes_all, gemm_ops_all, rq_method_bytes_all

    per_layer, rq_ms_all, gemm_ms_all, rq_bytes_all, gemm_ops_all, rq_method_bytes_all = per_kernel(layers, headline, min(args.steps, 50))
    n_layers = len(layers)
    gemm_tops = gemm_ops_all / gemm_ms_all / 1e9
    rq_gbps = rq_bytes_all / rq_ms_all / 1e6
    rq_gbps_method = rq_method_bytes_all / rq_ms_all / 1e6

    # side measurement: another setting on the same layers (whole path, then per kernel), outside the headline's timed region
    def side_run(ls, key, n=None):
        n = n or max(3, min(args.steps // 4, 20))
        timed_steps(ls, key, 2)
        ms8 = timed_steps(ls, key, n) * 1e3 / n
        pl8, rq8, gm8, rqb8, ops8, rqm8 = per_kernel(ls, key, n)
        frac = {"gemm_frac_fp6_peak": ops8 / gm8 / 1e9 / FP6_PEAK_TOPS} if key == "e2m3" else {"gemm_frac_int8_peak": ops8 / gm8 / 1e9 / INT8_PEAK_TOPS}
        return dict(steps=n, ms_per_step=ms8, value_TOPS=ops_of(ls) / (ms8 * 1e-3) / 1e12, gemm_TOPS=ops8 / gm8 / 1e9, **frac,
                    rotate_quant_GBps=rqm8 / rq8 / 1e6, rotate_quant_frac_hbm_peak=rqm8 / rq8 / 1e6 / HBM_PEAK_GBS,
                    rotate_quant_frac_hbm_peak_own_bytes=rqb8 / rq8 / 1e6 / HBM_PEAK_GBS, per_layer=pl8)

    side, side_rows, side_int8_path = None, None, None
    if args.bits == 4 and not args.headline_only:
        side_rows = side_run(layers, 8)
        side = side_run(layers, "i8b") if blocks_ok else side_rows
        if headline == "e2m3":
            side_int8_path = side_run(layers, 4)

    # ------------------------------------------------------------------ machine ceilings, measured in this run
    def event_ms(fn, reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        fn()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    ceilings = None
    if not args.headline_only or args.calibrate_copy:
        # 1 GiB read + 1 GiB written by an elementwise kernel (also what the HBM byte counters are scaled with, see profiles/)
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).fill_(1.0)
        dst = torch.empty_like(src)
        t_copy = event_ms(lambda: torch.add(src, 1.0, out=dst), 3)
        del src, dst
        ceilings = dict(copy_GBps=2.0 * (1 << 30) / t_copy / 1e6, copy_frac_hbm_peak=2.0 * (1 << 30) / t_copy / 1e6 / HBM_PEAK_GBS,
                        copy="elementwise kernel, 1 GiB in + 1 GiB out")
    if not args.headline_only:
        # register-only loops of the two matrix instructions: one wave per SIMD, 16 independent accumulators, tens of milliseconds each
        sink = torch.empty(65536, dtype=torch.float32, device=dev)
        iters = 4000
        for kind, name, kk in ((0, "mfma_int8_register_only_TOPS", 32), (1, "mfma_fp6_register_only_TFLOPS", 64)):
            t = event_ms(lambda: q.qvggt_mfma_ceiling(kind, iters, sink), 3)
            ceilings[name] = 256 * 4 * iters * 16 * (2.0 * 32 * 32 * kk) / (t * 1e-3) / 1e12
        ceilings["mfma_int8_frac_peak"] = ceilings["mfma_int8_register_only_TOPS"] / INT8_PEAK_TOPS
        ceilings["mfma_fp6_frac_peak"] = ceilings["mfma_fp6_register_only_TFLOPS"] / FP6_PEAK_TOPS
        del sink

    # HBM bytes per launch measured with rocprofv3 counters in separate runs of this command (see profiles/); None if that file is absent
    traffic, traffic_rq = None, None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        try:
            t = json.load(open(tpath)).get(f"config{args.config}", {})
            if headline == "e2m3":
                traffic, traffic_rq = t.get("e2m3_gemm_bytes_per_launch"), t.get("rotate_quant_e2m3_bytes_per_launch")
            elif args.bits == 4:
                traffic, traffic_rq = t.get("w4a4_gemm_bytes_per_launch"), t.get("rotate_quant_bytes_per_launch")
        except Exception:
            traffic, traffic_rq = None, None
    # the contraction is priced against the peak of the matrix instructions it runs on
    mfma_peak = FP6_PEAK_TOPS if headline == "e2m3" else INT8_PEAK_TOPS
    roofline = dict(kernel="e2m3_gemm_kernel" if headline == "e2m3" else "w4a4_gemm_kernel", bound="mfma", achieved=gemm_tops,
                    peak=mfma_peak, unit="TFLOP/s" if headline == "e2m3" else "TOP/s",
                    frac=gemm_tops / mfma_peak, traffic=traffic,
                    traffic_source="rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command, profiles/hbm_traffic.json",
                    ops_per_launch=gemm_ops_all / n_layers, avg_launch_ms=gemm_ms_all / n_layers)
    roofline_rq = dict(kernel="rotate_quant_mfma_kernel", bound="hbm", achieved=rq_gbps_method, peak=HBM_PEAK_GBS, unit="GB/s",
                       frac=rq_gbps_method / HBM_PEAK_GBS, traffic=traffic_rq,
                       bytes_per_launch=rq_method_bytes_all / n_layers, bytes="M (2.5 K + 4): bf16 in, 4-bit codes, one fp32 step per token",
                       achieved_own_bytes=rq_gbps, frac_own_bytes=rq_gbps / HBM_PEAK_GBS,
                       own_bytes_per_launch=rq_bytes_all / n_layers, avg_launch_ms=rq_ms_all / n_layers)

    # side measurement: the two HBM-bound reductions of the calibration-set arithmetic (Sec. 3.3) on the first layer's input,
    # taken as one sample of `frames` frames: per-frame mean / variance, and the cosine of every frame with frame 0
    nfds = None
    if args.bits == 4 and not args.headline_only and layers[0]["spec"].frames >= 2:      # a correlation needs two frames
        L0 = layers[0]
        s0_ = L0["spec"]
        fe = s0_.rows_per_frame * s0_.K
        Xf = L0["X"][: s0_.frames * s0_.rows_per_frame].view(s0_.frames, fe)
        code = q.QVGGT_BF16 if Xf.dtype == torch.bfloat16 else q.QVGGT_F32
        ws = torch.empty(q.qvggt_nfds_workspace_bytes(s0_.frames, fe, code), dtype=torch.uint8, device=dev)
        mean = torch.empty(s0_.frames, dtype=torch.float32, device=dev)
        var = torch.empty(s0_.frames, dtype=torch.float32, device=dev)
        corr = torch.empty(1, s0_.frames - 1, dtype=torch.float32, device=dev)
        astat = torch.empty(s0_.K, dtype=torch.float32, device=dev)
        nbytes = Xf.numel() * Xf.element_size()
        t_m = event_ms(lambda: q.qvggt_nfds_moments(Xf, mean, var, ws), 5)
        t_c = event_ms(lambda: q.qvggt_nfds_frame_correlation(Xf.view(1, s0_.frames, fe), corr, ws), 5)
        # the smoothing statistic at scale: max_t |X H|[t, j] over all tokens of the same tensor (Sec. 3.2, numerator of the factor)
        t_a = event_ms(lambda: q.qvggt_rotated_col_absmax(L0["X"], L0["signs"], astat), 5)
        nfds = dict(tensor=f"{s0_.frames} frames x {s0_.rows_per_frame} tokens x {s0_.K} ({Xf.dtype})".replace("torch.", ""),
                    moments_ms=t_m, moments_GBps=nbytes / t_m / 1e6, moments_frac_hbm_peak=nbytes / t_m / 1e6 / HBM_PEAK_GBS,
                    frame_correlation_ms=t_c, frame_correlation_GBps=nbytes / t_c / 1e6,
                    frame_correlation_frac_hbm_peak=nbytes / t_c / 1e6 / HBM_PEAK_GBS,
                    rotated_col_absmax_ms=t_a, rotated_col_absmax_GBps=nbytes / t_a / 1e6,
                    rotated_col_absmax_frac_hbm_peak=nbytes / t_a / 1e6 / HBM_PEAK_GBS)
        del ws, Xf

    # side measurement: fc2's kernel 1 reading fc1's output with the GELU applied on load, beside the plain kernel on the same
    # tensor (the activation pass it replaces reads and writes that tensor once more)
    gelu_side = None
    by_name = {L["spec"].name: L for L in layers}
    if (args.bits == 4 and headline == "e2m3" and not args.headline_only and "fc1" in by_name and "fc2" in by_name
            and by_name["fc2"]["spec"].K == by_name["fc1"]["spec"].N and by_name["fc2"]["spec"].K in (1024, 2048, 4096)):
        L1, L2 = by_name["fc1"], by_name["fc2"]
        linear(L1, "e2m3")                                     # fc1's output of this run: the tensor fc2's kernel 1 would read
        P2 = L2["prep"]["e2m3"]
        gelu_table = torch.empty(q.qvggt_gelu_table_bytes(), dtype=torch.uint8, device=dev)
        q.qvggt_gelu_table(gelu_table)
        fused = lambda: q.qvggt_gelu_rotate_smooth_quant_e2m3(L1["Y"], L2["signs"], P2["inv"], gelu_table, L2["Xf"], L2["sx"])
        plain = lambda: q.qvggt_rotate_smooth_quant_e2m3(L1["Y"], L2["signs"], P2["inv"], L2["Xf"], L2["sx"])
        # the two in turn, twice, 20 launches each after a launch that is not timed: neither gets the colder board
        t_f = t_p = 0.0
        for _ in range(2):
            t_f += event_ms(fused, 20) / 2
            t_p += event_ms(plain, 20) / 2
        s2 = L2["spec"]
        gelu_side = dict(tensor=f"fc1 output {s2.M} x {s2.K} bf16", gelu_rotate_quant_ms=t_f, rotate_quant_ms=t_p,
                         activation_pass_bytes_saved=4.0 * s2.M * s2.K,
                         activation_pass_ms_at_hbm_peak=4.0 * s2.M * s2.K / HBM_PEAK_GBS / 1e6)
    del by_name

    specs = [L["spec"] for L in layers]

    # ------------------------------------------------------------------ the other single-GPU configurations, in short
    other = None
    if args.bits == 4 and not args.headline_only:
        other = {}
        del layers
        torch.cuda.empty_cache()
        for cfg in (2, 3, 4):
            if cfg == args.config:
                continue
            ls = build_layers(cfg, {4})
            key = "e2m3" if (args.matrix_path == "e2m3" and blocks_ok_for(ls)) else 4
            n = 10
            timed_steps(ls, key, 3)
            ms = timed_steps(ls, key, n) * 1e3 / n
            pl, rq_ms, gm_ms, rq_b, g_ops, rq_mb = per_kernel(ls, key, n)
            other[f"config{cfg}"] = dict(
                workload=", ".join(f"{L['spec'].name} {L['spec'].M}x{L['spec'].K}->{L['spec'].N}" for L in ls), matrix_path=str(key),
                steps=n, ms_per_step=ms, value_TOPS=ops_of(ls) / (ms * 1e-3) / 1e12, gemm_TOPS=g_ops / gm_ms / 1e9,
                rotate_quant_GBps=rq_mb / rq_ms / 1e6,
                per_layer={k: dict(rotate_quant_us=v["rotate_quant_ms"] * 1e3, rotate_quant_us_min=v["rotate_quant_ms_min"] * 1e3,
                                   gemm_us=v["gemm_ms"] * 1e3, gemm_us_min=v["gemm_ms_min"] * 1e3, gemm_TOPS=v["gemm_TOPS"],
                                   rotate_quant_GBps=v["rotate_quant_GBps"]) for k, v in pl.items()})
            del ls
            torch.cuda.empty_cache()

    # ------------------------------------------------------------------ CPU oracle beside it (bounded samples)
    cpu = None
    if not args.no_cpu_baseline:
        import ctypes

        import oracle
        gomp = ctypes.CDLL("libgomp.so.1")                  # the OpenMP runtime the oracle's C library runs on: its real team size
        gomp.omp_get_max_threads.restype = ctypes.c_int
        threads_all = int(gomp.omp_get_max_threads())

        def oracle_leg(rows):
            preps = []
            for s in specs:
                sg = synth.make_signs(s)
                a = oracle.rotated_col_absmax(synth.make_calibration(s), pre_signs=sg)
                preps.append((s, sg, oracle.prepare_weights(synth.make_weights(s), a, pre_signs=sg, bits=args.bits), synth.make_bias(s),
                              synth.make_activation_rows(s, list(range(min(rows, s.M))))))
            st = dict(rotate_quant=0.0, int_gemm=0.0, epilogue=0.0)
            t_all0 = time.perf_counter()
            for s, sg, prep, bias, Xs in preps:
                t0 = time.perf_counter()
                dx, qx, _ = oracle.rotate_smooth_quant(Xs, prep.c_hat, sg, None, args.bits)
                t1 = time.perf_counter()
                acc = oracle.int_gemm(qx, prep.qw)
                t2 = time.perf_counter()
                oracle.dequant_bias(acc, dx, prep.dw, None if bias is None else oracle.to_f64(bias))
                t3 = time.perf_counter()
                st["rotate_quant"] += t1 - t0; st["int_gemm"] += t2 - t1; st["epilogue"] += t3 - t2
            total = time.perf_counter() - t_all0
            ops = sum(2.0 * min(rows, s.M) * s.N * s.K for s, *_ in preps)
            return total, ops, st

        total, cpu_ops, stages = oracle_leg(args.cpu_rows)
        cpu = dict(value=cpu_ops / total / 1e12, unit="TOPS", cores=threads_all, kind="oracle", seconds=total, seconds_per_stage=stages,
                   sample=f"first {args.cpu_rows} rows of each layer of config {args.config} through the oracle's three stages "
                          f"(dense fp64 Hadamard + quantize, int GEMM, dequant + bias); weight preparation not timed")
        if args.cpu_rows_1thread > 0:
            gomp.omp_set_num_threads(1)
            total1, ops1, stages1 = oracle_leg(args.cpu_rows_1thread)
            gomp.omp_set_num_threads(threads_all)
            cpu["one_thread"] = dict(value=ops1 / total1 / 1e12, unit="TOPS", cores=1, seconds=total1, seconds_per_stage=stages1,
                                     sample=f"first {args.cpu_rows_1thread} rows of each layer, same stages, OpenMP team of 1")

    s0 = specs[0]
    out = {
        "metric": METRIC if args.bits == 4 else METRIC.replace("W4A4", f"W{args.bits}A{args.bits}"), "value": value, "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": ("int4 codes as fp6 E2M3 (fp6 MFMA, fp32 accumulate: exact integer sums)" if headline == "e2m3" else
                  ("int4" if args.bits == 4 else f"int{args.bits} in int8") + " (int8 MFMA, int32 accumulate)"), "data": "synthetic",
        "config": {"workload": f"BASELINE configs[{args.config - 1}]: " + ", ".join(f"{s.name} {s.M}x{s.K}->{s.N}" for s in specs),
                   "tokens": s0.M, "frames": s0.frames, "layers": [s.name for s in specs], "parallelism": "1 GPU"},
        "gemm_TOPS": gemm_tops,
        **({"gemm_frac_fp6_peak": gemm_tops / FP6_PEAK_TOPS,
            "gemm_work_relative_to_int8_peak": gemm_tops / INT8_PEAK_TOPS} if headline == "e2m3" else {"gemm_frac_int8_peak": gemm_tops / INT8_PEAK_TOPS}),
        "rotate_quant_GBps": rq_gbps_method, "rotate_quant_frac_hbm_peak": rq_gbps_method / HBM_PEAK_GBS,
        "rotate_quant_GBps_own_bytes": rq_gbps, "rotate_quant_frac_hbm_peak_own_bytes": rq_gbps / HBM_PEAK_GBS,
        "sustained": sustained, "ceilings": ceilings,
        "per_layer": per_layer, "roofline": roofline, "roofline_rotate_quant": roofline_rq, "cpu_baseline": cpu,
    }
    if side is not None:
        out["w8a8"] = side
        if side_rows is not side:
            out["w8a8_row_major"] = side_rows
    if side_int8_path is not None:
        out["w4a4_int8_path"] = side_int8_path
    if nfds is not None:
        out["calibration_reductions"] = nfds
    if gelu_side is not None:
        out["gelu_fused_kernel1"] = gelu_side
    if other is not None:
        out["other_configs"] = other
    print(json.dumps(out))


if __name__ == "__main__":
    main()
