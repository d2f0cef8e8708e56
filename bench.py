#!/usr/bin/env python3
"""Benchmark of the quire-exact posit hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--size S] [--no-cpu]

Workload (benchmark config 5, the one the metric is quoted on): posit<8,0> quire
GEMM with M = N = K = 4096, operands N(0,1) rounded to posit<8,0>, all inputs
resident in HBM before timing starts.  One step is one pass over every stage of
the path on that batch:

    float32 -> posit<8,0> rounding of A and B        (posit_round)
    C = round(A @ B), 32-bit quire, one rounding      (posit_gemm)
    C -> posit<16,1> (exact widening)                 (posit_convert)
    W <- round(W - lr * C) in posit<16,1>, plus the
        posit<8,0> copy of the new W                  (posit_axpy)

`value` is M*N*K multiply-accumulates divided by the time of the whole step.
`roofline` is for the posit_gemm call alone (at this size: the pass that writes the operands'
int8 digit planes, then the integer-matrix-core kernel), timed with HIP events on the launch
stream.  The kernel forms every posit product exactly from four int8 x int8 products
(two base-128 digits per operand, int32 sums), so its bound is the int8 MFMA rate:
achieved = 8 int8 operations per posit MAC x M*N*K / time against the published 5.0 POP/s.
The line also carries the posit MAC rate against the integer-VALU peak the metric names
(one packed 16-bit dot-product lane-op = 2 MACs: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz x 2
= 78.6 TMAC/s), which the previous, vector-ALU kernel was bound by.
`cpu_baseline` times the (untuned) C++ oracle on a sample of rows of the same GEMM.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_TMACS = 256 * 4 * 16 * 2.4e9 * 2 / 1e12  # 78.6 TMAC/s: integer vector ALU, packed 16-bit dot products
PEAK_INT8_TOPS = 5000.0                       # dense int8 MFMA, published
INT8_OPS_PER_POSIT_MAC = 8                    # four int8 multiply-accumulates: (128 ah + al)(128 bh + bl)
# HBM-side bytes per posit_gemm call at 4096^3 (digit-plane pass + GEMM kernel), from two rocprofv3 --pmc passes
# (profiles/p8_gemm_4096_hbm_traffic.md): FETCH_SIZE x 2.0 (copy-kernel scale) + WRITE_SIZE, in KiB.
GEMM_4096_TRAFFIC_KIB = (189582, 21375, 16493, 65536)  # (FETCH gemm, WRITE gemm, FETCH digit pass, WRITE digit pass)


def _time_ms(torch, fn, reps, warm=2):
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


HBM_PEAK_TBS = 8.0  # MI355X HBM3E, published


def elementwise_measurements(torch, pn, n=1 << 27):
    """The bandwidth-bound entry points at n = 2^27 elements: algorithmic bytes per element (every input pattern read
    once, every output pattern written once) over the mean launch time, as TB/s and as a fraction of the 8 TB/s HBM
    peak; `copy` is torch's device-to-device copy of the same size class, the rate this machine reaches on a plain copy."""
    out = {}
    gen = torch.Generator(device="cuda")
    gen.manual_seed(2105000535)
    xf = torch.randn(n, dtype=torch.float32, device="cuda", generator=gen)
    p8 = pn.posit_round(xf, "p8")
    p16 = pn.posit_round(xf, "p16")
    g16 = pn.posit_round(xf * 0.01, "p16")
    o8 = torch.empty(n, dtype=torch.uint8, device="cuda")
    o16 = torch.empty(n, dtype=torch.uint16, device="cuda")
    of = torch.empty(n, dtype=torch.float32, device="cuda")
    w16 = p16.clone()
    p12 = pn.posit_round(xf, "p12_2")
    g12 = pn.posit_round(xf * 0.01, "p12_2")
    w12 = p12.clone()
    lr16, lr12 = 0xEB33, int(pn.posit_round(torch.tensor([-0.1], dtype=torch.float32, device="cuda"), "p12_2").cpu().view(torch.int16)[0]) & 0xFFF
    cases = [
        ("copy_f32 (torch, reference)", 8, lambda: of.copy_(xf)),
        ("round_f32_to_p8", 5, lambda: pn.posit_round(xf, "p8", out=o8)),
        ("round_f32_to_p16", 6, lambda: pn.posit_round(xf, "p16", out=o16)),
        ("convert_p8_to_p16", 3, lambda: pn.posit_convert(p8, "p8", "p16", out=o16)),
        ("convert_p16_to_p8", 3, lambda: pn.posit_convert(p16, "p16", "p8", out=o8)),
        ("convert_p16_to_f32", 6, lambda: pn.posit_convert(p16, "p16", "f32", out=of)),
        ("axpy_p16_p16", 6, lambda: pn.posit_axpy(lr16, g16, w16, "p16", "p16")),
        ("axpy_p16_p16_copy_p8", 7, lambda: pn.posit_axpy(lr16, g16, w16, "p16", "p16", fcopy="p8", y_copy=o8)),
        ("axpy_p12_2_p12_2_copy_p8_2", 7, lambda: pn.posit_axpy(lr12, g12, w12, "p12_2", "p12_2", fcopy="p8_2", y_copy=o8)),
    ]
    for name, bytes_per_elem, fn in cases:
        ms = _time_ms(torch, fn, 10, warm=2)
        tbs = n * bytes_per_elem / (ms * 1e-3) / 1e12
        out["elementwise_2^27_" + name] = {"ms": round(ms, 4), "B/elem": bytes_per_elem, "TB/s": round(tbs, 3),
                                           "frac_of_hbm_peak": round(tbs / HBM_PEAK_TBS, 3)}
    return out


def copy_calibration(torch):
    """One 256 MiB device-to-device copy: the kernel of known size that scales rocprofv3's FETCH_SIZE / WRITE_SIZE."""
    src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    src.fill_(1)
    torch.cuda.synchronize()
    dst.copy_(src)  # reads 256 MiB, writes 256 MiB
    torch.cuda.synchronize()
    del src, dst


def issue_rates():
    """Measured instruction-issue rates of this GPU (paper_2105_00053_amd/csrc/issue_rates.hip): the practical ceilings
    the kernels' lane-operation counts are priced against, beside the nominal 256 CU x 64 lanes x 2.4 GHz = 39.3 T/s."""
    import ctypes
    path = os.path.join(ROOT, "paper_2105_00053_amd", "libpositnn_rates.so")
    if not os.path.exists(path):
        raise RuntimeError("libpositnn_rates.so is not built: run python -m paper_2105_00053_amd.build")
    lib = ctypes.CDLL(path)
    rates = (ctypes.c_double * 5)()
    info = (ctypes.c_int * 2)()
    if lib.pnn_issue_rates(rates, info) != 0:
        raise RuntimeError("pnn_issue_rates failed")
    nominal = info[0] * 64 * 2.4e9
    return {"compute_units": info[0], "clock_kHz_reported": info[1], "nominal_lane_ops_per_s_T": round(nominal / 1e12, 2),
            "dot2_i16_lane_ops_per_s_T": round(rates[0] / 1e12, 2), "dot2_i16_TMAC_per_s": round(2 * rates[0] / 1e12, 2),
            "fma_f64_lane_ops_per_s_T": round(rates[1] / 1e12, 2), "int32_lane_ops_per_s_T": round(rates[2] / 1e12, 2),
            "lds_read_b128_TB_per_s": round(rates[3] / 1e12, 2), "mfma_i32_32x32x32_i8_POP_per_s": round(rates[4] / 1e15, 2)}


def extra_measurements(torch, pn, workloads):
    """The other benchmark configs, for the record (not part of `value`): GEMM kernels of configs 2 and 5
    and whole training steps of configs 3 and 4 (device-resident, see paper_2105_00053_amd/train_step.py)."""
    import numpy as np
    from paper_2105_00053_amd import train_step
    out = {}
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    for cfg, fmt, S, sigma, ext in ((5, "p8", 1024, 1.0, False), (5, "p8", 2048, 1.0, False), (2, "p16", 1024, 0.1, True), (5, "p32", 1024, 1.0, False),
                                    (5, "p8_2", 1024, 1.0, False), (5, "p8_2", 4096, 1.0, False)):
        A, B = workloads.gemm_operands(cfg, S, sigma=sigma, extremes=ext)
        Ap, Bp = pn.posit_round(dev(A), fmt), pn.posit_round(dev(B), fmt)
        C = torch.empty((S, S), dtype=Ap.dtype, device="cuda")
        ws = torch.empty(max(16, pn.posit_gemm_workspace(fmt, fmt, False, False, S, S, S)), dtype=torch.uint8, device="cuda")
        ms = _time_ms(torch, lambda: pn.posit_gemm(Ap, Bp, fmt, fmt, out=C, workspace=ws), 10 if fmt != "p32" else 3)
        out["gemm_%s_%d" % (fmt, S)] = {"ms": round(ms, 4), "TMAC/s": round(S ** 3 / ms / 1e9, 3)}
    # posit<8,0> convolutions, the three passes: two layers of the CifarNet-shaped net (batch 128) and a 64-channel
    # 56 x 56 layer at batch 256; 3 x 3 filters, padding 1, whole calls (operand rewriting and merging launches included)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(2105000536)
    for N, C, H, K in ((128, 32, 32, 32), (128, 64, 16, 64), (256, 64, 56, 64)):
        d = pn.ConvDesc(N, C, H, H, K, 3, 3, 1, 1, 1, 1)
        x = pn.posit_round(torch.randn((N, C, H, H), device="cuda", generator=gen), "p8")
        w = pn.posit_round(torch.randn((K, C, 3, 3), device="cuda", generator=gen) * 0.2, "p8")
        dy = pn.posit_round(torch.randn((N, K, H, H), device="cuda", generator=gen), "p8")
        b = pn.posit_round(torch.randn((K,), device="cuda", generator=gen), "p8")
        y, dx = torch.empty_like(dy), torch.empty_like(x)
        dw, db = torch.empty((K, C, 3, 3), dtype=torch.uint16, device="cuda"), torch.empty((K,), dtype=torch.uint16, device="cuda")
        wss = [torch.empty(max(16, pn.posit_conv2d_workspace(i, "p8", "p8" if i < 2 else "p16", d)), dtype=torch.uint8, device="cuda") for i in range(3)]
        gmac = N * H * H * K * C * 9 / 1e9
        entry = {"GMAC": round(gmac, 2)}
        for name, fn in (("fwd", lambda: pn.posit_conv2d_fwd(x, w, d, "p8", "p8", bias=b, out=y, workspace=wss[0])),
                         ("bwd_data", lambda: pn.posit_conv2d_bwd_data(dy, w, d, "p8", "p8", out=dx, workspace=wss[1])),
                         ("bwd_weight", lambda: pn.posit_conv2d_bwd_weight(dy, x, d, "p8", "p16", with_bias=True, out=dw, out_bias=db, workspace=wss[2]))):
            ms = _time_ms(torch, fn, 10, warm=2)
            entry[name] = {"ms": round(ms, 4), "TMAC/s": round(gmac / ms, 2)}
        out["conv_p8_N%d_C%d_%dx%d_K%d_3x3" % (N, C, H, H, K)] = entry
    out.update(elementwise_measurements(torch, pn))
    final = dict(compute="p8_2", master="p12_2", loss="p10_2")  # Sec. 4, Table 4: the configuration the paper ends up with
    for name, net, fmts in (("lenet5_step_batch64", workloads.LENET, {}), ("cifarnet_step_batch128", workloads.CIFARNET, {}),
                            ("lenet5_step_batch64_posit8_2_12_2_10_2", workloads.LENET, final),
                            ("cifarnet_step_batch128_posit8_2_12_2_10_2", workloads.CIFARNET, final)):
        x, params, labels = workloads.network_inputs(net)
        model = train_step.Net(net["layers"], [(dev(w), dev(b)) for w, b in params], **fmts)
        xd, ld = dev(x), torch.from_numpy(labels).cuda()
        ms = _time_ms(torch, lambda: train_step.training_step(model, xd, ld), 10, warm=3)
        runner = train_step.GraphedStep(model, tuple(xd.shape))
        ld32 = ld.to(torch.int32)
        ms_graph = _time_ms(torch, lambda: runner.step(xd, ld32), 10, warm=3)
        out[name] = {"ms": round(ms, 3), "ms_graph_replay": round(ms_graph, 3)}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--size", type=int, default=4096, help="M = N = K")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--cpu-rows", type=int, default=0, help="rows of C the CPU baseline computes (0 = auto)")
    ap.add_argument("--sustained-steps", type=int, default=200, help="steps of the longer run reported as `sustained` (0 = skip)")
    ap.add_argument("--no-extra", action="store_true", help="skip the secondary measurements (other benchmark configs)")
    ap.add_argument("--only-elementwise", action="store_true",
                    help="run only the bandwidth-bound entry points at 2^27 elements and print their rates (the command the elementwise profiles use)")
    ap.add_argument("--issue-rates", action="store_true",
                    help="run only the instruction-issue microbenchmarks (csrc/issue_rates.hip) and print the measured rates")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one 256 MiB device copy before timing (scale reference for rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only (the path is data-parallel over rows of A: "
              "more GPUs would each take a block of rows); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2105_00053_amd as pn
    import workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    pn.load()
    torch.cuda.set_device(0)
    if args.issue_rates:
        print(json.dumps(issue_rates()))
        return
    if args.only_elementwise:
        if args.copy_calibration:
            copy_calibration(torch)
        print(json.dumps(elementwise_measurements(torch, pn)))
        return
    S = args.size
    A32, B32 = workloads.gemm_operands(5, S)
    Af = torch.from_numpy(A32).cuda()
    Bf = torch.from_numpy(B32).cuda()
    W = pn.posit_round(torch.from_numpy(workloads.normal_matrix(5, 7, (S, S))).cuda(), "p16")
    lr_bits = 0xEB33  # -(0x14CD): posit<16,1> pattern of -0.1 (two's complement of the pattern of 0.1)
    A8 = torch.empty((S, S), dtype=torch.uint8, device="cuda")
    B8 = torch.empty((S, S), dtype=torch.uint8, device="cuda")
    C8 = torch.empty((S, S), dtype=torch.uint8, device="cuda")
    C16 = torch.empty((S, S), dtype=torch.uint16, device="cuda")
    W8 = torch.empty((S, S), dtype=torch.uint8, device="cuda")
    need = pn.posit_gemm_workspace("p8", "p8", False, False, S, S, S)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")

    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]

    def step(i=None):
        pn.posit_round(Af, "p8", out=A8)
        pn.posit_round(Bf, "p8", out=B8)
        if i is not None:
            ev[i][0].record()
        pn.posit_gemm(A8, B8, "p8", "p8", out=C8, workspace=ws)
        if i is not None:
            ev[i][1].record()
        pn.posit_convert(C8, "p8", "p16", out=C16)
        pn.posit_axpy(lr_bits, C16, W, "p16", "p16", fcopy="p8", y_copy=W8)

    if args.copy_calibration:
        copy_calibration(torch)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    gemm_ms = sum(a.elapsed_time(b) for a, b in ev) / args.steps
    macs = float(S) ** 3
    value = macs / (ms_per_step * 1e-3) / 1e9  # GMAC/s over the whole step
    achieved = macs / (gemm_ms * 1e-3) / 1e12  # TMAC/s of the GEMM kernel

    # a longer run of the same step, for a sustained figure beside the short timed region (clocks settle under load)
    sustained = None
    if args.sustained_steps > 0:
        torch.cuda.synchronize()
        ts = time.perf_counter()
        for _ in range(args.sustained_steps):
            step()
        torch.cuda.synchronize()
        sustained_ms = (time.perf_counter() - ts) * 1e3 / args.sustained_steps
        sustained = {"steps": args.sustained_steps, "ms_per_step": round(sustained_ms, 4),
                     "GMAC/s": round(macs / (sustained_ms * 1e-3) / 1e9, 1)}

    traffic, traffic_source = None, "not measured for this size"
    if S == 4096 and GEMM_4096_TRAFFIC_KIB:
        fg, wg, fd, wd = GEMM_4096_TRAFFIC_KIB
        traffic = int((2.0 * (fg + fd) + wg + wd) * 1024)
        traffic_source = "stored constant from profiles/p8_gemm_4096_hbm_traffic.md (two rocprofv3 --pmc runs), not measured by this run"
    result = {
        "metric": "quire-exact posit MAC/s (GMAC/s) + % of integer-VALU peak, posit<8,0> GEMM",
        "value": round(value, 1),
        "unit": "GMAC/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int32",  # int8 x int8 digit products summed in int32, combined modulo 2^32: the quire of Table 1
        "data": "synthetic",
        "config": {"workload": "posit<8,0> quire GEMM M=N=K=%d (benchmark config 5), step = round A,B + gemm + convert + axpy" % S,
                   "fin": "posit<8,0>", "fout": "posit<8,0>", "quire_bits": 32},
        "roofline": {
            "bound": "mfma",
            "kernel": "p8_mfma_gemm_kernel (with its digit-plane pass: the posit_gemm call)",
            "achieved": round(achieved * INT8_OPS_PER_POSIT_MAC, 1),
            "peak": PEAK_INT8_TOPS,
            "unit": "TOP/s (int8)",
            "frac": round(achieved * INT8_OPS_PER_POSIT_MAC / PEAK_INT8_TOPS, 4),
            "kernel_ms": round(gemm_ms, 4),
            "int8_ops_per_posit_mac": INT8_OPS_PER_POSIT_MAC,
            "posit_TMAC_per_s": round(achieved, 3),
            "integer_valu_peak_TMAC_per_s": round(PEAK_TMACS, 1),
            "x_integer_valu_peak": round(achieved / PEAK_TMACS, 3),
            "algorithmic_bytes": 3 * S * S,
            "traffic": traffic,
            "traffic_source": traffic_source,
        },
    }

    if sustained:
        result["sustained"] = sustained
    if not args.no_extra:
        result["extra"] = extra_measurements(torch, pn, workloads)

    if not args.no_cpu:
        from oracle import fast
        threads = fast.hw_threads()
        A8n = A8.cpu().numpy()
        B8n = B8.cpu().numpy()
        rows = args.cpu_rows or max(8, min(S, (64 * threads * 4096 * 4096) // (S * S)))  # about 15 s of CPU work
        t0 = time.perf_counter()
        Cn, overflowed = fast.gemm(A8n, B8n, "p8", "p8", rows=(0, rows), threads=threads)
        dt = time.perf_counter() - t0
        mism = int((Cn[:rows] != C8[:rows].cpu().numpy()).sum())
        result["cpu_baseline"] = {
            "value": round(rows * float(S) * S / dt / 1e9, 4),
            "unit": "GMAC/s",
            "cores": threads,
            "kind": "oracle",
            "sample": "first %d rows of C (of %d), full K, C++ oracle with %d threads, %.1f s" % (rows, S, threads, dt),
            "mismatches_vs_gpu": mism,
            "quire_overflows": int(overflowed),
        }
    print(json.dumps(result))


if __name__ == "__main__":
    main()
