#!/usr/bin/env python3
"""Benchmark of the QNN hot path on one MI355X.

Primary line (the driver's contract): binary-GEMM throughput at 8192^3 on packed +-1 operands (1 +-1 MAC = 2 ops),
inputs resident in HBM, one step = one qnn_binary_gemm call.  The same JSON line carries the MNIST-shaped MLP forward
(samples/s) and the other configurations as secondary figures, the roofline of the dominant kernel measured with HIP
events on the launch stream, and the CPU oracle timed on this machine's host cores on a bounded sample.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--engine auto|valu|mfma] [--only c3|c2|c1|c4|c5]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
for _p in (ROOT, os.path.join(ROOT, "tests")):
    if _p not in sys.path:
        sys.path.insert(0, _p)

import numpy as np  # noqa: E402

VALU_PEAK_TOPS = 256 * 64 * 32 * 2.4e9 / 1e12  # 256 CUs x 64 lanes/clk x (32 MAC per xor+bcnt pair = 32 ops/lane/clk) x 2.4 GHz
MFMA_I8_PEAK_TOPS = 5000.0                     # dense int8 matrix-core peak, 2 ops per MAC
MFMA_FP4_PEAK_TOPS = 10100.0                   # dense FP4 matrix-core peak
HBM_PEAK_GBS = 8000.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def time_steps(fn, steps, warmup):
    """K calls of fn between two HIP events on the launch stream, after W untimed calls; returns ms per call."""
    import torch

    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    return e0.elapsed_time(e1) / steps, wall_ms


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=200,
                    help="untimed calls first; the card needs some hundred launches to raise its shader clock from idle")
    ap.add_argument("--engine", default="auto", choices=["auto", "valu", "mfma", "fp4"])
    ap.add_argument("--only", default="", help="comma list of c1,c2,c3,c4,c5 (default: all)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="target CPU time of the oracle sample")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="also run a plain 256 MiB device copy (known size) so that rocprofv3 --pmc FETCH_SIZE / "
                         "WRITE_SIZE readings of the GEMM can be scaled by what the same counter reads for the copy")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (every configuration is measured whole on one MI355X); "
              "run it with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_1609_07061_amd as q
    import qnn_inputs as qi
    from qnn_testlib import dev, np_pack_bits, np_pack_pm1

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    engine = {"auto": q.ENGINE_AUTO, "valu": q.ENGINE_VALU, "mfma": q.ENGINE_MFMA, "fp4": q.ENGINE_MFMA_FP4}[args.engine]
    only = set(filter(None, args.only.split(","))) or {"c1", "c2", "c3", "c4", "c5"}
    seed = qi.SEED_BASE
    steps, warmup = args.steps, args.warmup
    sec_steps = max(5, steps // 5)
    sec_warm = max(3, warmup // 10)
    extra = {}

    # ---------------------------------------------------------------- C3: 8192^3 binary GEMM (primary)
    n = 8192
    log("[bench] generating C3 operands")
    a3 = qi.pm1(seed, 30, (n, n))
    w3 = qi.pm1(seed, 31, (n, n))
    A3, W3 = dev(np_pack_pm1(a3)), dev(np_pack_pm1(w3))
    C3 = torch.empty((n, n), dtype=torch.int32, device="cuda")
    ops3 = 2.0 * n * n * n
    ms3, wall3 = time_steps(lambda: q.qnn_binary_gemm(A3, W3, n, out=C3, engine=engine), steps, warmup)
    tops3 = ops3 / (ms3 * 1e-3) / 1e12
    log(f"[bench] C3 8192^3: {ms3:.4f} ms/step, {tops3:.1f} binary TOPS")
    # spot check of the timed output against the oracle (a few complete rows)
    import oracle

    rows = np.array([0, 4095, 8191])
    assert np.array_equal(C3[rows].cpu().numpy(), oracle.gemm_pm1(a3[rows], w3)), "C3 output differs from the oracle"
    used = q.qnn_last_engine()
    used_name = {q.ENGINE_VALU: "valu", q.ENGINE_MFMA: "mfma", q.ENGINE_MFMA_FP4: "fp4"}[used]
    if used == q.ENGINE_MFMA_FP4:
        roof = {"bound": "mfma", "achieved": tops3, "peak": MFMA_FP4_PEAK_TOPS, "unit": "TOP/s",
                "frac": tops3 / MFMA_FP4_PEAK_TOPS, "traffic": None, "kernel": "gemm_mfma_kernel<fp4>",
                "peak_dtype": "fp4 (E2M1) dense MFMA, fp32 accumulate"}
    elif used == q.ENGINE_MFMA:
        roof = {"bound": "mfma", "achieved": tops3, "peak": MFMA_I8_PEAK_TOPS, "unit": "TOP/s",
                "frac": tops3 / MFMA_I8_PEAK_TOPS, "traffic": None, "kernel": "gemm_mfma_kernel",
                "peak_dtype": "int8 dense MFMA, int32 accumulate"}
    else:
        roof = {"bound": "alu", "achieved": tops3, "peak": VALU_PEAK_TOPS, "unit": "TOP/s",
                "frac": tops3 / VALU_PEAK_TOPS, "traffic": None, "kernel": "gemm_valu_kernel",
                "peak_dtype": "integer vector ALU: one xor and one popcount-accumulate per 32 MACs"}
    roof["frac_of_int8_mfma_peak"] = tops3 / MFMA_I8_PEAK_TOPS
    roof["frac_of_valu_xor_popcount_peak"] = tops3 / VALU_PEAK_TOPS
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        try:
            t = json.load(open(tpath)).get(roof["kernel"] + "@c3")
            if t:
                roof["traffic"] = t["fetch_bytes"] + t["write_bytes"]  # HBM bytes per launch, measured (profiles/)
                roof["traffic_detail"] = t
        except Exception:
            pass

    if args.traffic_probe:
        D3 = torch.empty_like(C3)
        for _ in range(3):
            D3.copy_(C3)  # 268 435 456 bytes read + the same written per call
        # two more kernels of known size, with the plain loads / stores the GEMM itself uses: a fill (268 435 456 bytes
        # written, nothing read) and the sign+pack kernel (268 435 456 bytes read, 8 388 608 written)
        xf = torch.randn((n, n), dtype=torch.float32, device="cuda")
        pk = torch.empty((n, n // 32), dtype=torch.int32, device="cuda")
        for _ in range(3):
            D3.zero_()
            q.qnn_pack_sign(xf, out=pk)
        torch.cuda.synchronize()
        del D3, xf, pk

    # ---------------------------------------------------------------- C3 with sign+pack from fp32 included
    if "c3" in only:
        xf = torch.randn((n, n), dtype=torch.float32, device="cuda")  # values are irrelevant to the cost
        pk = torch.empty((n, n // 32), dtype=torch.int32, device="cuda")
        msp, _ = time_steps(lambda: q.qnn_pack_sign(xf, out=pk), sec_steps, sec_warm)
        extra["pack_sign_8192x8192"] = {"ms": msp, "GBps": (n * n * 4 + n * n / 8) / (msp * 1e-3) / 1e9,
                                        "frac_of_hbm_peak": (n * n * 4 + n * n / 8) / (msp * 1e-3) / 1e9 / HBM_PEAK_GBS}
        extra["c3_tops_including_pack_of_both_operands_from_fp32"] = ops3 / ((ms3 + 2 * msp) * 1e-3) / 1e12
        del xf, pk
        # the two other bandwidth-bound kernels of the path at the same size: the stand-alone threshold + repack over
        # the 8192^2 int32 product, and the bit-plane split of 8-bit codes
        thr = torch.zeros((n,), dtype=torch.int32, device="cuda")
        tb = torch.empty((n, n // 32), dtype=torch.int32, device="cuda")
        mst, _ = time_steps(lambda: q.qnn_threshold_sign(C3, thr, None, out=tb), sec_steps, sec_warm)
        gb = (n * n * 4 + n * n / 8 + n * 4) / (mst * 1e-3) / 1e9
        extra["threshold_sign_8192x8192"] = {"ms": mst, "GBps": gb, "frac_of_hbm_peak": gb / HBM_PEAK_GBS}
        codes = torch.randint(0, 256, (n, n), dtype=torch.uint8, device="cuda")
        pl = torch.empty((8, n, n // 32), dtype=torch.int32, device="cuda")
        msb, _ = time_steps(lambda: q.qnn_pack_bitplanes(codes, 8, out=pl), sec_steps, sec_warm)
        gb = (n * n + n * n) / (msb * 1e-3) / 1e9
        extra["pack_bitplanes_8192x8192_8bit"] = {"ms": msb, "GBps": gb, "frac_of_hbm_peak": gb / HBM_PEAK_GBS}
        del thr, tb, codes, pl

    # ---------------------------------------------------------------- C2: MNIST-shaped MLP forward
    if "c2" in only:
        dims = [784, 4096, 4096, 4096, 10]
        batch = 10000
        x2 = dev(qi.uniform_int(seed, 20, (batch, 784), 0, 255, dtype=np.uint8))
        W2 = [dev(np_pack_pm1(qi.pm1(seed, 21 + l, (dims[l + 1], dims[l])))) for l in range(4)]
        T2 = [dev(qi.uniform_int(seed, 25 + l, (dims[l + 1],), -64, 64)) for l in range(3)]
        ws = torch.empty(q.qnn_binary_mlp_workspace_bytes(batch, 8, dims), dtype=torch.uint8, device="cuda")
        lg = torch.empty((batch, 10), dtype=torch.int32, device="cuda")
        ms2, _ = time_steps(lambda: q.qnn_binary_mlp_forward(x2, 8, dims, W2, T2, logits=lg, workspace=ws, engine=engine),
                            sec_steps, sec_warm)
        bin_mac = batch * (8 * 784 * 4096 + 2 * 4096 * 4096 + 4096 * 10)
        int_mac = batch * (784 * 4096 + 2 * 4096 * 4096 + 4096 * 10)
        extra["c2_mlp_forward"] = {"ms": ms2, "samples_per_s": batch / (ms2 * 1e-3),
                                   "binary_tops_bitplane_accounting": 2.0 * bin_mac / (ms2 * 1e-3) / 1e12,
                                   "effective_integer_tmacs": int_mac / (ms2 * 1e-3) / 1e12}
        log(f"[bench] C2 MLP: {ms2:.4f} ms, {batch / (ms2 * 1e-3):.0f} samples/s")

    # ---------------------------------------------------------------- C1: small GEMM + sign-binarize (latency)
    if "c1" in only:
        xa, xw = dev(qi.normal_f32(seed, 10, (128, 1024))), dev(qi.normal_f32(seed, 11, (1024, 1024)))
        A1 = torch.empty((128, 32), dtype=torch.int32, device="cuda")
        W1 = torch.empty((1024, 32), dtype=torch.int32, device="cuda")
        C1 = torch.empty((128, 1024), dtype=torch.int32, device="cuda")

        def c1():
            q.qnn_pack_sign(xa, out=A1)
            q.qnn_pack_sign(xw, out=W1)
            q.qnn_binary_gemm(A1, W1, 1024, out=C1, engine=engine)

        ms1, wall1 = time_steps(c1, max(steps, 50), 10)
        ms1g, _ = time_steps(lambda: q.qnn_binary_gemm(A1, W1, 1024, out=C1, engine=engine), max(steps, 50), 10)
        extra["c1_pack_pack_gemm_128x1024x1024"] = {"us_gpu": ms1 * 1e3, "us_wall": wall1 * 1e3, "us_gemm_only": ms1g * 1e3}

    # ---------------------------------------------------------------- C4: AlexNet-shaped conv, 1-bit W x 2-bit A
    if "c4" in only:
        B, H, Wd, Cin, Cout = 256, 13, 13, 384, 256
        u = qi.uniform_int(seed, 40, (B, H, Wd, Cin), 0, 3)
        up = dev(np.stack([np_pack_bits((u >> p) & 1) for p in range(2)]))
        wp = dev(np_pack_pm1(qi.pm1(seed, 41, (Cout, 3, 3, Cin)))[None])
        o4 = torch.empty((B, H, Wd, Cout), dtype=torch.int32, device="cuda")
        ms4, _ = time_steps(lambda: q.qnn_bitplane_conv2d(up, [1, 2], q.PLANE_BIT, Cin, wp, [1], q.PLANE_SIGN, 1, 1,
                                                          out=o4, engine=engine), sec_steps, sec_warm)
        imac = B * H * Wd * 9 * Cin * Cout
        extra["c4_conv_alexnet"] = {"ms": ms4, "binary_tops_bitplane_accounting": 2.0 * 2 * imac / (ms4 * 1e-3) / 1e12,
                                    "effective_integer_tmacs": imac / (ms4 * 1e-3) / 1e12}

    # ---------------------------------------------------------------- C5: 4-bit x 4-bit LSTM gate GEMM
    if "c5" in only:
        M, K, N = 2240, 2048, 4096
        a5 = qi.uniform_int(seed, 50, (M, K), -8, 7)
        w5 = qi.uniform_int(seed, 51, (N, K), -8, 7)
        ap5 = dev(np.stack([np_pack_bits((a5 >> p) & 1) for p in range(4)]))
        wp5 = dev(np.stack([np_pack_bits((w5 >> p) & 1) for p in range(4)]))
        o5 = torch.empty((M, N), dtype=torch.int32, device="cuda")
        coef = [1, 2, 4, -8]
        ms5, _ = time_steps(lambda: q.qnn_bitplane_gemm(ap5, coef, q.PLANE_BIT, wp5, coef, q.PLANE_BIT, K, out=o5,
                                                        engine=engine), sec_steps, sec_warm)
        extra["c5_lstm_int4"] = {"ms": ms5, "binary_tops_bitplane_accounting": 2.0 * 16 * M * N * K / (ms5 * 1e-3) / 1e12,
                                 "effective_integer_tmacs": M * N * K / (ms5 * 1e-3) / 1e12}

    # ---------------------------------------------------------------- CPU baseline: the oracle, as it stands
    cpu = None
    if not args.no_cpu_baseline:
        log("[bench] timing the CPU oracle on a sample of C3")
        t0 = time.perf_counter()
        oracle.gemm_pm1(a3[:128], w3)
        probe = time.perf_counter() - t0
        nrows = int(min(n, max(128, 128 * args.cpu_seconds / max(probe, 1e-3))))
        nrows = (nrows // 128) * 128
        reps = 1
        if nrows == n:  # the whole product is cheaper than the target: repeat it
            reps = int(max(1, min(20, round(args.cpu_seconds / max(probe * n / 128, 1e-3)))))
        t0 = time.perf_counter()
        for _ in range(reps):
            oracle.gemm_pm1(a3[:nrows], w3)
        dt = time.perf_counter() - t0
        cpu = {"value": 2.0 * reps * nrows * n * n / dt / 1e12, "unit": "TOPS", "cores": oracle.num_threads(),
               "kind": "oracle",
               "sample": f"{reps} x the first {nrows} of 8192 rows of the C3 product (plain int8 multiply-accumulate, {dt:.1f} s)"}

    out = {
        "metric": "binary GEMM TOPS (1 +-1 MAC = 2 ops) at 8192^3",
        "value": tops3,
        "unit": "TOPS",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": ms3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": {"fp4": "bit-packed +-1 operands expanded on chip to fp4 (E2M1), fp32 accumulate (exact), int32 out",
                  "mfma": "bit-packed +-1 operands expanded on chip to int8, int32 accumulate",
                  "valu": "u32 bit-packed +-1 operands, xor + popcount, int32 accumulate"}[used_name],
        "data": "synthetic (seeded Bernoulli(0.5) +-1 operands; stands in for the paper's 8192^3 benchmark matrices)",
        "config": {"workload": "C3: 8192x8192x8192 binary GEMM on packed +-1 operands, int32 output",
                   "engine": used_name, "M": n, "N": n, "K": n},
        "mlp_forward_samples_per_s": extra.get("c2_mlp_forward", {}).get("samples_per_s"),
        "roofline": roof,
        "cpu_baseline": cpu,
        "secondary": extra,
        "paper_context": "paper reports only ratios on a GTX750: XNOR kernel 23x its baseline kernel, 3.4x cuBLAS at 8192^3; MLP 7x",
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
