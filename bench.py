#!/usr/bin/env python3
"""Benchmark of the GEMM / BRGEMM hot path on one MI355X.

One "step" is one pass of the whole hot path (tile decomposition, operand staging,
MFMA loop, epilogue) over the headline workload: bf16-in / fp32-accumulate /
bf16-out GEMM with M = N = K = 4096, row-major, beta = 0, inputs N(0,1) rounded to
bf16 and already resident in HBM.  Prints ONE JSON line with the whole-job TFLOP/s,
the MFMA roofline of the kernel (HIP-event duration of the same launches) and the
CPU oracle timed on a bounded sample of the same workload.  Other configurations
(fp32 2048^3, MLP shapes, skinny M, batch-reduce) are timed too and reported under
"others" in the same line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "GEMM TFLOP/s and % of MFMA peak (fp32, bf16), 4096^3 and MLP shapes"
PEAK_BF16 = 2516.6      # TFLOP/s, dense bf16 MFMA: 256 CUs x 4096 flop/clk x 2.4 GHz
PEAK_F32 = 157.3        # TFLOP/s, fp32 MFMA
HBM_TBS = 8.0
# Bytes beyond L2 per launch of the headline kernel, from rocprofv3 --pmc FETCH_SIZE and
# WRITE_SIZE passes over this same command (profiles/bf16_pingpong_256x256x64_gemm4096_nn.md):
# (FETCH_SIZE KiB x 2.0 + WRITE_SIZE KiB x 1.0) x 1024; the factors are what the same counters
# read for a plain 1 GiB copy.  The figure belongs to the kernel sources it was taken on:
# "sources" is the SHA-256 (first 16 hex digits) of the files below at that time, and the
# bench line reports null as soon as they have changed.
HEADLINE_TRAFFIC = {"variant": "bf16_pingpong_256x256x64",
                    "bytes": (98430.2 * 2.0 + 32769.4 * 1.0) * 1024.0,
                    "files": ["paper_2511_13764_amd/csrc/bf16_pingpong.hpp", "paper_2511_13764_amd/csrc/bf16_pingpong.hip",
                              "paper_2511_13764_amd/csrc/bf16_tiles.hpp"],
                    "sources": "6ac75e20769fbb4d"}
WARMUP_FLOOR_MS = 100.0  # continuous load before any timed region (clock management settles in ~30 ms)


def kernel_sources_digest(files):
    import hashlib
    h = hashlib.sha256()
    for f in files:
        with open(os.path.join(ROOT, f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def headline_traffic(variant):
    if variant != HEADLINE_TRAFFIC["variant"]:
        return None
    if kernel_sources_digest(HEADLINE_TRAFFIC["files"]) != HEADLINE_TRAFFIC["sources"]:
        return None
    return HEADLINE_TRAFFIC["bytes"]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # The chip's clock management needs ~30 ms of continuous load to settle (the first 50
    # launches of the headline kernel run ~50 % slower than the steady state).  Whatever
    # --warmup says, every timed region is preceded by at least WARMUP_FLOOR_MS of
    # untimed launches of the same call.
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=300)
    ap.add_argument("--settle-ms", type=float, default=WARMUP_FLOOR_MS,
                    help="untimed continuous load before every timed region (profiling passes use 0)")
    ap.add_argument("--print-sources-digest", action="store_true",
                    help="print the digest that ties HEADLINE_TRAFFIC to the kernel sources, and exit")
    ap.add_argument("--no-others", action="store_true", help="time the headline workload only")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run three plain 1 GiB device copies (reference for FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.print_sources_digest:
        print(kernel_sources_digest(HEADLINE_TRAFFIC["files"]))
        return
    if args.gpus != 1:
        print("bench.py: the library runs on one GPU; --gpus must be 1 "
              "(a multi-GPU job would shard M or N across GPUs with no exchange)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2511_13764_amd import binding as B
    from paper_2511_13764_amd import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_each_way": src.numel() * 4, "copies": 3}))
        return
    B.load()

    def dev(x):
        return torch.from_numpy(x.view(np.int16) if x.dtype == np.uint16 else x).cuda()

    def settle(fn, floor_ms=None):
        """Untimed launches for at least floor_ms of GPU work."""
        floor_ms = args.settle_ms if floor_ms is None else min(floor_ms, args.settle_ms)
        if floor_ms <= 0:
            return
        t_w = time.perf_counter()
        while (time.perf_counter() - t_w) * 1e3 < floor_ms:
            for _ in range(20):
                fn()
            torch.cuda.synchronize()

    def time_launches(fn, steps, warmup):
        """Wall time per step (sync on both sides) and HIP-event time per launch."""
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        for _ in range(steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) / steps
        return wall, e0.elapsed_time(e1) * 1e-3 / steps

    def per_launch(fn, n, group=1):
        """Median and minimum HIP-event time of `n` samples of `group` launches each."""
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
        for a, b in evs:
            a.record()
            for _ in range(group):
                fn()
            b.record()
        torch.cuda.synchronize()
        ts = sorted(a.elapsed_time(b) * 1e-3 / group for a, b in evs)
        return ts[len(ts) // 2], ts[0]

    # ------------------------------------------------------------------ headline: bf16 4096^3
    case = W.config3_bf16_square(4096)
    M, N, K = case.M, case.N, case.K
    dA, dB = dev(case.A), dev(case.B)
    dC = torch.empty((M, N), dtype=torch.int16, device="cuda")
    ws_bytes = B.gemm_workspace_bytes(B.DTYPE_BF16, M, N, K)
    ws = torch.empty(min(ws_bytes, 1 << 30), dtype=torch.uint8, device="cuda")

    def step():
        B.gemm_bf16(0, 0, M, N, K, dA, K, dB, N, 0.0, dC, N, 0, workspace=ws)

    settle(step)
    wall, ev = time_launches(step, args.steps, args.warmup)
    variant = B.gemm_variant_name(B.gemm_last_variant())
    split = B.gemm_last_split()
    med, mn = per_launch(step, 50)
    flops = 2.0 * M * N * K
    value = flops / wall / 1e12
    achieved = flops / ev / 1e12

    # Matrix-pipe rate of this device with no LDS or memory traffic, on operands of the
    # workload's distribution and on zeros: the rate is set by the chip's power management
    # and depends on the operand values.  Two bf16 forms: 16x16x32 with 32 accumulators (the
    # instruction and register shape of the headline kernel and of the streaming kernels:
    # the denominator of frac_of_measured_mfma_rate) and 32x32x16 with 8 accumulators (the
    # 4-wave 128 x 128 kernel).
    def mfma_rate(dtype, ops):
        sink = torch.empty(2048 * 512, dtype=torch.float32, device="cuda")
        fl = [0.0]

        def probe():
            fl[0] = B.gemm_mfma_probe(dtype, ops, 256, 2048, sink)
        settle(probe, 30.0)
        _, t = time_launches(probe, 20, 3)
        return fl[0] / t / 1e12

    g = torch.Generator(device="cuda").manual_seed(20251113)
    ops_n = torch.randn(6 * 64 * 8, device="cuda", generator=g).to(torch.bfloat16)
    ops_w = torch.randn(12 * 64 * 8, device="cuda", generator=g).to(torch.bfloat16)
    measured = {"bf16_16x16x32_normal_operands": round(mfma_rate(B.PROBE_BF16_16X16X32, ops_w), 1),
                "bf16_16x16x32_zero_operands": round(mfma_rate(B.PROBE_BF16_16X16X32, torch.zeros_like(ops_w)), 1),
                "bf16_32x32x16_normal_operands": round(mfma_rate(B.DTYPE_BF16, ops_n), 1),
                "bf16_32x32x16_zero_operands": round(mfma_rate(B.DTYPE_BF16, torch.zeros_like(ops_n)), 1),
                "f32_uniform_operands": round(mfma_rate(B.DTYPE_F32, torch.rand(6 * 64, device="cuda", generator=g) * 2 - 1), 1),
                "s8_uniform_operands": round(mfma_rate(B.PROBE_S8, torch.randint(-128, 128, (12 * 64 * 16,), device="cuda",
                                                                               dtype=torch.int8, generator=g)), 1),
                "f8_normal_operands": round(mfma_rate(B.PROBE_F8, torch.randn(12 * 64 * 32, device="cuda", generator=g)
                                                      .to(torch.float8_e4m3fn)), 1),
                "unit": "TFLOP/s (int8: TOP/s)", "what": "register-only MFMA issue loop, 2 waves per SIMD on every CU"}

    out = {
        "metric": METRIC, "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "warmup_floor_ms": args.settle_ms, "ms_per_step": round(wall * 1e3, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "bf16-in/fp32-acc/bf16-out GEMM M=N=K=4096 row-major (NN) beta=0, N(0,1) inputs",
                   "variant": variant, "split": split},
        "roofline": {"bound": "mfma", "achieved": round(achieved, 2), "peak": PEAK_BF16, "unit": "TFLOP/s",
                     "frac": round(achieved / PEAK_BF16, 4), "traffic": headline_traffic(variant),
                     "traffic_unit": "bytes per launch (algorithmic: %d)" % (2 * (M * K + K * N + M * N)),
                     "kernel": variant, "us_per_launch": round(ev * 1e6, 2),
                     "us_median": round(med * 1e6, 2), "us_min": round(mn * 1e6, 2),
                     "frac_of_measured_mfma_rate": round(achieved / measured["bf16_16x16x32_normal_operands"], 4)},
        "measured_mfma_rate": measured,
    }

    # ------------------------------------------------------------------ CPU oracle beside it (bounded sample)
    if not args.no_cpu:
        from oracle import reference as oracle
        rows_probe = list(range(0, M, M // 64))[:64]
        t0 = time.perf_counter()
        oracle.gemm_ref(case.A, K, case.B, N, M, N, K, rows=rows_probe)
        rate = len(rows_probe) * N * K / (time.perf_counter() - t0)          # MAC/s
        n_rows = int(min(M, max(128, 12.0 * rate / (N * K))))
        rows = sorted(set(np.linspace(0, M - 1, n_rows).astype(int).tolist()))
        t0 = time.perf_counter()
        ref = oracle.gemm_ref(case.A, K, case.B, N, M, N, K, rows=rows)
        dt = time.perf_counter() - t0
        got = oracle.bf16_to_f64(dC.cpu().numpy().view(np.uint16)[rows])
        err = float(np.linalg.norm(got - ref) / np.linalg.norm(ref))
        out["cpu_baseline"] = {"value": round(2.0 * len(rows) * N * K / dt / 1e12, 5), "unit": "TFLOP/s",
                               "cores": oracle.num_threads(), "kind": "oracle",
                               "sample": f"{len(rows)} of {M} complete rows of C of the same 4096^3 problem "
                                         f"({dt:.1f} s); GPU rows match them to rel. Frobenius {err:.2e}"}
        assert err <= 2e-3, f"GPU result disagrees with the oracle: {err}"

    # ------------------------------------------------------------------ the other configurations
    if not args.no_others:
        others = {}

        def record(name, flops_, fn, peak, steps=50, warmup=20, bytes_=None):
            settle(fn)
            w_, e_ = time_launches(fn, steps, warmup)
            med_, min_ = per_launch(fn, 20, group=1 if e_ > 50e-6 else 20)
            r = {"us": round(e_ * 1e6, 2), "us_median": round(med_ * 1e6, 2), "us_min": round(min_ * 1e6, 2),
                 "tflops": round(flops_ / e_ / 1e12, 2),
                 "frac_mfma_peak": round(flops_ / e_ / 1e12 / peak, 4),
                 "variant": B.gemm_variant_name(B.gemm_last_variant()), "split": B.gemm_last_split()}
            if bytes_ is not None:
                r["hbm_gbs"] = round(bytes_ / e_ / 1e9, 1)
                r["frac_hbm_peak"] = round(bytes_ / e_ / 1e12 / HBM_TBS, 4)
                # the attainable roofline of an HBM-bound shape: min(MFMA peak, flop/byte x measured copy rate)
                r["frac_of_measured_copy"] = round(bytes_ / e_ / 1e9 / copy_gbs, 4)
            others[name] = r

        # Device copy bandwidth of this machine: a plain 1 GiB copy (read + write counted), the
        # measured stand-in for the 8 TB/s datasheet figure in the HBM-bound rows below.
        src_c = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst_c = torch.empty_like(src_c)
        settle(lambda: dst_c.copy_(src_c), 30.0)
        _, t_copy = time_launches(lambda: dst_c.copy_(src_c), 20, 3)
        copy_gbs = 2.0 * src_c.numel() * 4 / t_copy / 1e9
        out["hbm_copy_gbs"] = round(copy_gbs, 1)
        del src_c, dst_c

        # fp32 2048^3 with beta = 0.5
        c2 = W.config2_f32_2048()
        a2, b2, c2d = dev(c2.A), dev(c2.B), dev(c2.C0.copy())
        record("f32_2048_beta0.5", c2.flops,
               lambda: B.gemm_f32(0, 0, 2048, 2048, 2048, a2, 2048, b2, 2048, 0.5, c2d, 2048, workspace=ws), PEAK_F32)
        del a2, b2, c2d
        # fp32 at the 4096^3 point of the metric (same distribution, device-generated: timing only)
        a4 = torch.rand((4096, 4096), device="cuda") * 2 - 1
        b4 = torch.rand((4096, 4096), device="cuda") * 2 - 1
        c4 = torch.rand((4096, 4096), device="cuda") * 2 - 1
        record("f32_4096_beta0.5", 2.0 * 4096 ** 3,
               lambda: B.gemm_f32(0, 0, 4096, 4096, 4096, a4, 4096, b4, 4096, 0.5, c4, 4096, workspace=ws), PEAK_F32,
               steps=20, warmup=5)
        others["f32_4096_beta0.5"]["frac_of_measured_mfma_rate"] = round(
            others["f32_4096_beta0.5"]["tflops"] / measured["f32_uniform_operands"], 4)
        del a4, b4, c4
        # bf16 squares (random device data of the same distribution: timing only)
        for s in (1024, 2048, 8192):
            a = torch.randn((s, s), device="cuda").to(torch.bfloat16)
            b = torch.randn((s, s), device="cuda").to(torch.bfloat16)
            c = torch.empty((s, s), device="cuda", dtype=torch.bfloat16)
            record(f"bf16_{s}", 2.0 * s ** 3,
                   lambda: B.gemm_bf16(0, 0, s, s, s, a, s, b, s, 0.0, c, s, 0, workspace=ws), PEAK_BF16,
                   steps=20 if s == 8192 else 100)
            del a, b, c
        # binary16 operands and results, same kernels with the f16 matrix instruction
        a = torch.randn((4096, 4096), device="cuda").to(torch.float16)
        b = torch.randn((4096, 4096), device="cuda").to(torch.float16)
        c = torch.empty((4096, 4096), device="cuda", dtype=torch.float16)
        record("f16_4096", 2.0 * 4096 ** 3,
               lambda: B.gemm_f16(0, 0, 4096, 4096, 4096, a, 4096, b, 4096, 0.0, c, 4096, 0, workspace=ws), PEAK_BF16,
               steps=100)
        del a, b, c
        # int8 operands, int32 results (NT: both operands k-contiguous); peak 5.0 POP/s dense int8
        a = torch.randint(-128, 128, (4096, 4096), device="cuda", dtype=torch.int8)
        b = torch.randint(-128, 128, (4096, 4096), device="cuda", dtype=torch.int8)
        c = torch.empty((4096, 4096), device="cuda", dtype=torch.int32)
        record("s8_4096_nt", 2.0 * 4096 ** 3,
               lambda: B.gemm_s8(0, 1, 4096, 4096, 4096, a, 4096, b, 4096, 0, c, 4096), 5033.2, steps=100)
        others["s8_4096_nt"]["unit"] = "TOP/s (tflops / frac_mfma_peak fields), against 5033.2 TOP/s int8 MFMA"
        others["s8_4096_nt"]["frac_of_measured_mfma_rate"] = round(others["s8_4096_nt"]["tflops"] / measured["s8_uniform_operands"], 4)
        # the same with B stored K x N (n-contiguous: re-laid-out by the transposing one-byte LDS read)
        record("s8_4096_nn", 2.0 * 4096 ** 3,
               lambda: B.gemm_s8(0, 0, 4096, 4096, 4096, a, 4096, b, 4096, 0, c, 4096), 5033.2, steps=100)
        others["s8_4096_nn"]["unit"] = others["s8_4096_nt"]["unit"]
        del a, b, c
        # FP8 (E4M3) operands, bf16 results (NT); peak 5.0 PFLOP/s dense fp8
        a = torch.randn((4096, 4096), device="cuda").to(torch.float8_e4m3fn)
        b = torch.randn((4096, 4096), device="cuda").to(torch.float8_e4m3fn)
        c = torch.empty((4096, 4096), device="cuda", dtype=torch.bfloat16)
        record("f8_4096_nt", 2.0 * 4096 ** 3,
               lambda: B.gemm_f8(0, 1, 4096, 4096, 4096, a, 4096, b, 4096, 0.0, c, 4096, 0, workspace=ws), 5033.2,
               steps=100)
        others["f8_4096_nt"]["frac_of_measured_mfma_rate"] = round(others["f8_4096_nt"]["tflops"] / measured["f8_normal_operands"], 4)
        record("f8_4096_nn", 2.0 * 4096 ** 3,
               lambda: B.gemm_f8(0, 0, 4096, 4096, 4096, a, 4096, b, 4096, 0.0, c, 4096, 0, workspace=ws), 5033.2,
               steps=100)
        del a, b, c
        # MLP shapes, weights stored N x K
        # The skinny cases are bound by the stream of the 90 MB weight matrix, which fits
        # the 256 MB last-level cache: "warm" repeats one matrix, "cold" rotates over four
        # (360 MB) so that every launch streams its weights from HBM.
        for which, (Kk, Nn) in (("up", (4096, 11008)), ("down", (11008, 4096))):
            wgts = [(torch.randn((Nn, Kk), device="cuda") * 0.02).to(torch.bfloat16) for _ in range(4)]
            wgt = wgts[0]
            for Mm in (4096, 128, 16):
                a = torch.randn((Mm, Kk), device="cuda").to(torch.bfloat16)
                c = torch.empty((Mm, Nn), device="cuda", dtype=torch.bfloat16)
                bytes_ = 2.0 * (Mm * Kk + Kk * Nn + Mm * Nn)
                record(f"mlp_{which}_M{Mm}" + ("_warm" if Mm <= 128 else ""), 2.0 * Mm * Nn * Kk,
                       lambda: B.gemm_bf16(0, 1, Mm, Nn, Kk, a, Kk, wgt, Kk, 0.0, c, Nn, 0, workspace=ws),
                       PEAK_BF16, steps=30 if Mm == 4096 else 100, bytes_=bytes_ if Mm <= 128 else None)
                if Mm == 4096 and which == "up":
                    # the paper's benchmark kernel (Section 6): GEMM + bias + ReLU in one pass
                    bias = torch.randn(Nn, device="cuda")
                    record("mlp_up_M4096_bias_relu", 2.0 * Mm * Nn * Kk,
                           lambda: B.brgemm_fused(B.DTYPE_BF16, 0, 1, Mm, Nn, Kk, 1, a, None, Kk, wgt, None, Kk, 0.0,
                                                  c, Nn, 0, bias, B.EPI_BIAS | B.EPI_RELU, workspace=ws),
                           PEAK_BF16, steps=30)
                if Mm <= 128:
                    turn = [0]

                    def cold():
                        turn[0] = (turn[0] + 1) & 3
                        B.gemm_bf16(0, 1, Mm, Nn, Kk, a, Kk, wgts[turn[0]], Kk, 0.0, c, Nn, 0, workspace=ws)
                    record(f"mlp_{which}_M{Mm}_cold", 2.0 * Mm * Nn * Kk, cold, PEAK_BF16, steps=100, bytes_=bytes_)
                del a, c
            del wgts, wgt
        # the same GEMMs with B packed once beforehand (Section 2.2; packing is not timed)
        def packed_of(b, tB, Kk, Nn):
            pk = torch.empty(B.gemm_packed_b_bytes(Kk, Nn) // 2, dtype=torch.int16, device="cuda")
            B.gemm_pack_b_bf16(tB, Kk, Nn, b, b.shape[1], pk)
            return pk
        a = torch.randn((4096, 4096), device="cuda").to(torch.bfloat16)
        b = torch.randn((4096, 4096), device="cuda").to(torch.bfloat16)
        c = torch.empty((4096, 4096), device="cuda", dtype=torch.bfloat16)
        pk = packed_of(b, 0, 4096, 4096)
        record("bf16_4096_packedB", 2.0 * 4096 ** 3,
               lambda: B.gemm_bf16_packed(0, 4096, 4096, 4096, a, 4096, pk, 0.0, c, 4096, 0, workspace=ws), PEAK_BF16,
               steps=100)
        del a, b, c, pk
        for Mm in (4096, 16):
            Kk, Nn = 4096, 11008
            pks = [packed_of((torch.randn((Nn, Kk), device="cuda") * 0.02).to(torch.bfloat16), 1, Kk, Nn)
                   for _ in range(4 if Mm == 16 else 1)]
            a = torch.randn((Mm, Kk), device="cuda").to(torch.bfloat16)
            c = torch.empty((Mm, Nn), device="cuda", dtype=torch.bfloat16)
            turn = [0]

            def packed_step():
                turn[0] = (turn[0] + 1) % len(pks)
                B.gemm_bf16_packed(0, Mm, Nn, Kk, a, Kk, pks[turn[0]], 0.0, c, Nn, 0, workspace=ws)
            record(f"mlp_up_M{Mm}_packedB" + ("_cold" if Mm == 16 else ""), 2.0 * Mm * Nn * Kk, packed_step, PEAK_BF16,
                   steps=30 if Mm == 4096 else 100, bytes_=2.0 * (Mm * Kk + Kk * Nn + Mm * Nn) if Mm == 16 else None)
            del a, c, pks
        # batch-reduce over scattered tiles
        c5 = W.config5_brgemm()
        pool = dev(c5.pool)
        ao, bo = torch.from_numpy(c5.A_off).cuda(), torch.from_numpy(c5.B_off).cuda()
        cc = torch.zeros((c5.M, c5.N), dtype=torch.float32, device="cuda")
        record("brgemm_512x512x64x64", c5.flops,
               lambda: B.brgemm_bf16(0, 0, c5.M, c5.N, c5.K, c5.batch, pool, ao, c5.lda, pool, bo, c5.ldb, 1.0,
                                     cc, c5.N, workspace=ws), PEAK_BF16, steps=200, warmup=20)
        del pool, ao, bo, cc
        # Context only, not a path of this library: the vendor GEMM library as PyTorch calls it
        # (torch.matmul), same box, same clock state, same shapes and value distributions.
        vendor = {}

        def vendor_time(name, flops_, fn):
            settle(fn)
            _, e_ = time_launches(fn, 50, 20)
            vendor[name] = {"us": round(e_ * 1e6, 2), "tflops": round(flops_ / e_ / 1e12, 2)}

        try:
            for s_ in (2048, 4096):
                a = torch.randn((s_, s_), device="cuda").to(torch.bfloat16)
                b = torch.randn((s_, s_), device="cuda").to(torch.bfloat16)
                c = torch.empty((s_, s_), device="cuda", dtype=torch.bfloat16)
                vendor_time(f"bf16_{s_}", 2.0 * s_ ** 3, lambda: torch.matmul(a, b, out=c))
                del a, b, c
            a = torch.randn((4096, 4096), device="cuda").to(torch.bfloat16)
            w = (torch.randn((11008, 4096), device="cuda") * 0.02).to(torch.bfloat16)
            c = torch.empty((4096, 11008), device="cuda", dtype=torch.bfloat16)
            vendor_time("mlp_up_M4096", 2.0 * 4096 * 11008 * 4096, lambda: torch.matmul(a, w.t(), out=c))
            del a, w, c
            a = torch.rand((2048, 2048), device="cuda") * 2 - 1
            b = torch.rand((2048, 2048), device="cuda") * 2 - 1
            c = torch.empty((2048, 2048), device="cuda")
            vendor_time("f32_2048", 2.0 * 2048 ** 3, lambda: torch.matmul(a, b, out=c))
            del a, b, c
        except Exception as exc:        # context only: never let it take the line down
            vendor["error"] = repr(exc)
        out["others"] = others
        out["vendor_library_via_torch_matmul"] = vendor

    print(json.dumps(out))


if __name__ == "__main__":
    main()
