#!/usr/bin/env python3
"""Benchmark of the QNN hot path on one MI355X.

Primary line (the driver's contract): binary-GEMM throughput at 8192^3 on packed +-1 operands (1 +-1 MAC = 2 ops),
inputs resident in HBM, one step = one qnn_binary_gemm call: W untimed calls, then exactly K calls between two HIP
events on the launch stream.  The same JSON line carries the second half of the metric (MNIST-shaped MLP forward,
samples/s, with its own roofline fraction), the other configurations as secondary figures (each at least 50 timed calls
after at least 10 warm-up calls, whatever --steps says, and each reported only if a sample of its output equals the
oracle's), the shader clock observed before and after the timed region, per-call durations (median, minimum), the
roofline of the dominant kernel, and the CPU oracle timed on this machine's host cores on a bounded sample.

Order of work: all host-side preparation first (inputs, oracle expectations), then the GPU work back to back -
secondary configurations, then the primary one - so that the primary's few warm-up calls do not have to bring the card up
from idle clocks by themselves; the clock actually seen is in the line (`sclk_mhz`).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--engine auto|valu|mfma|fp4] [--only c3,c2,c1,c4,c5]
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
for _p in (ROOT, os.path.join(ROOT, "tests")):
    if _p not in sys.path:
        sys.path.insert(0, _p)

import numpy as np  # noqa: E402

NOMINAL_MHZ = 2400.0
VALU_PEAK_TOPS = 256 * 64 * 32 * 2.4e9 / 1e12  # 256 CUs x 64 lanes/clk x (32 MAC per xor+bcnt pair = 32 ops/lane/clk) x 2.4 GHz
MFMA_I8_PEAK_TOPS = 5000.0                     # dense int8 matrix-core peak, 2 ops per MAC
MFMA_FP4_PEAK_TOPS = 10100.0                   # dense FP4 matrix-core peak
HBM_PEAK_GBS = 8000.0
ENGINE_NAMES = {1: "valu", 2: "mfma", 3: "fp4", 4: "mfma_lds"}
ENGINE_PEAK = {1: VALU_PEAK_TOPS, 2: MFMA_I8_PEAK_TOPS, 3: MFMA_FP4_PEAK_TOPS, 4: MFMA_I8_PEAK_TOPS}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def time_steps(fn, steps, warmup):
    """K calls of fn between two HIP events on the launch stream, after W untimed calls; returns ms per call."""
    import torch

    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def time_secondary(fn, steps, warmup, min_ms=40.0):
    """time_steps for the secondary figures: a pass shorter than min_ms of GPU time is repeated with as many calls as
    fill it, so that every figure rests on a sustained run and the card is under load from one job to the next."""
    ms = time_steps(fn, steps, warmup)
    if ms * steps < min_ms:
        ms = time_steps(fn, int(min_ms / max(ms, 1e-4)) + 1, 0)
    return ms


def per_call_ms(fn, calls):
    """One event pair per call (all on the launch stream, no host synchronization in between)."""
    import torch

    ev = [torch.cuda.Event(enable_timing=True) for _ in range(calls + 1)]
    ev[0].record()
    for i in range(calls):
        fn()
        ev[i + 1].record()
    torch.cuda.synchronize()
    return [ev[i].elapsed_time(ev[i + 1]) for i in range(calls)]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--engine", default="auto", choices=["auto", "valu", "mfma", "fp4"])
    ap.add_argument("--only", default="", help="comma list of c1,c2,c3,c4,c5 (default: all; c3 always runs)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="target CPU time of the oracle sample")
    ap.add_argument("--primary-first", action="store_true",
                    help="time the primary configuration before the secondary ones (from idle clocks)")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="also run kernels of known size (a 256 MiB device copy, a fill, the sign+pack kernel) so that "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings of the GEMM can be scaled by them")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (every configuration is measured whole on one MI355X); "
              "run it with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    import oracle
    import paper_1609_07061_amd as q
    import qnn_inputs as qi
    from qnn_testlib import dev, np_pack_bits, np_pack_pm1

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    engine = {"auto": None, "valu": q.ENGINE_VALU, "mfma": q.ENGINE_MFMA, "fp4": q.ENGINE_MFMA_FP4}[args.engine]
    only = set(filter(None, args.only.split(","))) or {"c1", "c2", "c3", "c4", "c5"}
    seed = qi.SEED_BASE
    steps, warmup = args.steps, args.warmup
    sec_steps, sec_warm = max(50, steps // 5), max(10, warmup // 10)
    extra = {}
    jobs = []  # (rank in the GPU phase, closure)

    def frac_fields(ops, ms, eng):
        tops = ops / (ms * 1e-3) / 1e12
        return {"engine": ENGINE_NAMES[eng], "integer_tops": tops, "frac_of_engine_peak": tops / ENGINE_PEAK[eng]}

    # ================================================================ host-side preparation (no GPU timing yet)
    n = 8192
    log("[bench] preparing inputs and oracle expectations")
    a3 = qi.pm1(seed, 30, (n, n))
    w3 = qi.pm1(seed, 31, (n, n))
    A3, W3 = dev(np_pack_pm1(a3)), dev(np_pack_pm1(w3))
    C3 = torch.empty((n, n), dtype=torch.int32, device="cuda")
    rows3 = np.unique(np.concatenate([[0, 255, 256, 4095, 4096, n - 1], (qi.raw_u64(seed, 32, 10) % np.uint64(n)).astype(np.int64)]))
    want3 = oracle.gemm_pm1(a3[rows3], w3)
    ops3 = 2.0 * n * n * n

    def run_c3():
        if engine is None:
            q.qnn_binary_gemm(A3, W3, n, out=C3)  # the plain entry point, as a user calls it
        else:
            q.qnn_binary_gemm(A3, W3, n, out=C3, engine=engine)

    if "c2" in only:
        dims = [784, 4096, 4096, 4096, 10]
        batch = 10000
        x2h = qi.uniform_int(seed, 20, (batch, 784), 0, 255, dtype=np.uint8)
        W2h = [qi.pm1(seed, 21 + l, (dims[l + 1], dims[l])) for l in range(4)]
        T2h = [qi.uniform_int(seed, 25 + l, (dims[l + 1],), -64, 64) for l in range(3)]
        idx2 = np.unique(np.concatenate([[0, 255, 256, 9999], (qi.raw_u64(seed, 29, 60) % np.uint64(batch)).astype(np.int64)]))
        want2 = oracle.mlp(x2h[idx2], W2h, T2h)
        x2 = dev(x2h)
        W2 = [dev(np_pack_pm1(w)) for w in W2h]
        T2 = [dev(t) for t in T2h]
        ws2 = torch.empty(q.qnn_binary_mlp_workspace_bytes(batch, 8, dims), dtype=torch.uint8, device="cuda")
        lg2 = torch.empty((batch, 10), dtype=torch.int32, device="cuda")

        def run_c2():
            q.qnn_binary_mlp_forward(x2, 8, dims, W2, T2, logits=lg2, workspace=ws2, engine=engine)

        def job_c2():
            ms2 = time_secondary(run_c2, sec_steps, sec_warm)
            engines = q.qnn_last_engines()
            ok = np.array_equal(lg2[idx2].cpu().numpy(), want2)
            int_mac = [batch * dims[l] * dims[l + 1] for l in range(4)]
            # per-layer time at the peak of the engine that ran it (output layer: its HBM bytes at the HBM peak)
            t_roof = 0.0
            for l in range(3):
                t_roof += 2.0 * int_mac[l] / (ENGINE_PEAK[engines[l]] * 1e12)
            out_bytes = batch * 128 * 4 + 10 * 128 * 4 + batch * 10 * 4
            t_roof += out_bytes / (HBM_PEAK_GBS * 1e9)
            # the output layer alone (10 neurons: bound by reading the 5 MB of packed activations)
            act = torch.zeros((batch, 128), dtype=torch.int32, device="cuda")
            ms_out = time_secondary(lambda: q.qnn_binary_gemm(act, W2[3], 4096, out=lg2), sec_steps, sec_warm)
            extra["c2_mlp_forward"] = {
                "parity_sample_ok": bool(ok), "ms": ms2 if ok else None,
                "samples_per_s": batch / (ms2 * 1e-3) if ok else None,
                "engines_per_layer": [ENGINE_NAMES[e] for e in engines],
                "effective_integer_tmacs": sum(int_mac) / (ms2 * 1e-3) / 1e12 if ok else None,
                "binary_tops_bitplane_accounting": 2.0 * (int_mac[0] * 8 + sum(int_mac[1:])) / (ms2 * 1e-3) / 1e12 if ok else None,
                "output_layer": {"ms": ms_out, "GBps": out_bytes / (ms_out * 1e-3) / 1e9,
                                 "frac_of_hbm_peak": out_bytes / (ms_out * 1e-3) / 1e9 / HBM_PEAK_GBS},
            }
            extra["roofline_c2"] = {
                "bound": "mfma", "unit": "ms", "sum_of_layer_times_at_peak_ms": t_roof * 1e3, "measured_ms": ms2,
                "frac": t_roof * 1e3 / ms2 if ok else None,
                "peaks": "layer 1 int8 MFMA 5000 TOP/s, hidden layers FP4 MFMA 10100 TOP/s (as run), output layer HBM 8 TB/s",
            }
            log(f"[bench] C2 MLP: {ms2:.4f} ms, {batch / (ms2 * 1e-3):.0f} samples/s, parity sample {'ok' if ok else 'FAILED'}")

        jobs.append((3, job_c2))

    if "c4" in only:
        B, H, Wd, Cin, Cout = 256, 13, 13, 384, 256
        u4 = qi.uniform_int(seed, 40, (B, H, Wd, Cin), 0, 3)
        w4 = qi.pm1(seed, 41, (Cout, 3, 3, Cin))
        idx4 = np.array([0, 100, B - 1])
        want4 = oracle.conv2d(u4[idx4], w4.astype(np.int32), 1, 1)
        up4 = dev(np.stack([np_pack_bits((u4 >> p) & 1) for p in range(2)]))
        wp4 = dev(np_pack_pm1(w4)[None])
        o4 = torch.empty((B, H, Wd, Cout), dtype=torch.int32, device="cuda")

        def job_c4():
            ms4 = time_secondary(lambda: q.qnn_bitplane_conv2d(up4, [1, 2], q.PLANE_BIT, Cin, wp4, [1], q.PLANE_SIGN, 1, 1,
                                                           out=o4, engine=engine), sec_steps, sec_warm)
            eng = q.qnn_last_engine()
            ok = np.array_equal(o4[idx4].cpu().numpy(), want4)
            imac = B * H * Wd * 9 * Cin * Cout
            extra["c4_conv_alexnet"] = {"parity_sample_ok": bool(ok), "ms": ms4 if ok else None,
                                        "effective_integer_tmacs": imac / (ms4 * 1e-3) / 1e12 if ok else None,
                                        "binary_tops_bitplane_accounting": 2.0 * 2 * imac / (ms4 * 1e-3) / 1e12 if ok else None,
                                        **(frac_fields(2.0 * imac, ms4, eng) if ok else {})}

        jobs.append((2, job_c4))

    if "c5" in only:
        M5, K5, N5 = 2240, 2048, 4096
        a5 = qi.uniform_int(seed, 50, (M5, K5), -8, 7)
        w5 = qi.uniform_int(seed, 51, (N5, K5), -8, 7)
        idx5 = np.unique(np.concatenate([[0, 255, 256, M5 - 1], (qi.raw_u64(seed, 52, 28) % np.uint64(M5)).astype(np.int64)]))
        want5 = oracle.gemm_int(a5[idx5], w5)
        ap5 = dev(np.stack([np_pack_bits((a5 >> p) & 1) for p in range(4)]))
        wp5 = dev(np.stack([np_pack_bits((w5 >> p) & 1) for p in range(4)]))
        o5 = torch.empty((M5, N5), dtype=torch.int32, device="cuda")
        coef = [1, 2, 4, -8]

        def job_c5():
            ms5 = time_secondary(lambda: q.qnn_bitplane_gemm(ap5, coef, q.PLANE_BIT, wp5, coef, q.PLANE_BIT, K5, out=o5,
                                                         engine=engine), sec_steps, sec_warm)
            eng = q.qnn_last_engine()
            ok = np.array_equal(o5[idx5].cpu().numpy(), want5)
            imac = M5 * N5 * K5
            extra["c5_lstm_int4"] = {"parity_sample_ok": bool(ok), "ms": ms5 if ok else None,
                                     "effective_integer_tmacs": imac / (ms5 * 1e-3) / 1e12 if ok else None,
                                     "binary_tops_bitplane_accounting": 2.0 * 16 * imac / (ms5 * 1e-3) / 1e12 if ok else None,
                                     **(frac_fields(2.0 * imac, ms5, eng) if ok else {})}

        jobs.append((2, job_c5))

    if "c2" in only:
        # backward products of Alg. 1 for a hidden layer of the MLP (10000 x 4096 -> 4096) with gradients quantized to
        # eight-plane fixed-point values: g_a = g W and g_W = g^T a, transposes included
        Mb, Nb, Kb = 10000, 4096, 4096
        gb_h = qi.normal_f32(seed, 60, (Mb, Nb)) * np.float32(0.2)
        wb_h = qi.pm1(seed, 61, (Nb, Kb))
        ab_h = qi.pm1(seed, 62, (Mb, Kb))
        gq_h = oracle.log_code_value(oracle.log_quant(gb_h, -6, 0))
        idxb = np.array([0, 255, 256, 4095])
        want_ga = oracle.gemm_int(gq_h[idxb], np.ascontiguousarray(wb_h.T).astype(np.int32))          # rows of g W
        want_gw = oracle.gemm_int(np.ascontiguousarray(gq_h.T[idxb]), np.ascontiguousarray(ab_h.T).astype(np.int32))  # rows of g^T a
        Gb, Wb, Ab = dev(gb_h), dev(np_pack_pm1(wb_h)), dev(np_pack_pm1(ab_h))
        wsb = torch.empty(q.qnn_binary_backward_workspace_bytes(Mb, Nb, Kb, 8), dtype=torch.uint8, device="cuda")
        Gp = torch.empty((8, Mb, Nb // 32), dtype=torch.int32, device="cuda")
        coefb = [1, 2, 4, 8, 16, 32, 64, -128]
        outb = {}

        def run_bwd():
            q.qnn_log_quant_planes(Gb, -6, 0, 8, as_value=True, out=Gp)
            outb["ga"], outb["gw"] = q.qnn_binary_backward(Gp, coefb, q.PLANE_BIT, Nb, Wb, Ab, Kb, workspace=wsb)

        def job_bwd():
            msb = time_secondary(run_bwd, sec_steps, sec_warm)
            ok = (np.array_equal(outb["ga"][idxb].cpu().numpy(), want_ga)
                  and np.array_equal(outb["gw"][idxb].cpu().numpy(), want_gw))
            imac = 2.0 * Mb * Nb * Kb
            extra["backward_hidden_layer_8bit_gradients"] = {
                "parity_sample_ok": bool(ok), "ms": msb if ok else None,
                "effective_integer_tmacs": imac / (msb * 1e-3) / 1e12 if ok else None,
                "note": "LogQuant of the fp32 gradient to 8 planes, three bit transposes, two 8-plane x 1-plane products"}

        jobs.append((2, job_bwd))

    if "c4" in only:
        # Binarized ConvNet forward (Alg. 4) on the CIFAR-10 architecture of App. A: 2 x 128C3 - MP2 - 2 x 256C3 - MP2 -
        # 2 x 512C3 - MP2 - 1024FC - 1024FC - 10, 32 x 32 RGB images (8-bit), batch 256; logits of sampled images
        # against the oracle (images of a batch are independent)
        Bn, Hn = 256, 32
        couts, pools, fcs = [128, 128, 256, 256, 512, 512], [0, 1, 0, 1, 0, 1], [1024, 1024, 10]
        xn = qi.uniform_int(seed, 80, (Bn, Hn, Hn, 3), 0, 255, dtype=np.uint8)
        conv_w, cin = [], 3
        for l, co in enumerate(couts):
            conv_w.append(qi.pm1(seed, 81 + l, (co, 3, 3, cin)))
            cin = co
        fc_w, fin = [], (Hn // 8) * (Hn // 8) * cin
        for j, fo in enumerate(fcs):
            fc_w.append(qi.pm1(seed, 90 + j, (fo, fin)))
            fin = fo
        widths = couts + fcs[:-1]
        Tn = [qi.uniform_int(seed, 100 + l, (wd,), -(3000 if l == 0 else 40), 3000 if l == 0 else 40) for l, wd in enumerate(widths)]
        Fn = [qi.bernoulli_bits(seed, 110 + l, (wd,)) for l, wd in enumerate(widths)]
        idxn = np.array([0, 100, Bn - 1])
        wantn = oracle.convnet(xn[idxn], conv_w, pools, fc_w, Tn, Fn)
        Xn = dev(xn)
        Wn = [dev(np_pack_pm1(w)) for w in conv_w] + [dev(np_pack_pm1(w)) for w in fc_w]
        Tnd, Fnd = [dev(t) for t in Tn], [dev(f) for f in Fn]
        wsn = torch.empty(q.qnn_binary_convnet_workspace_bytes(Bn, Hn, Hn, 3, 8, couts, pools, fcs), dtype=torch.uint8, device="cuda")
        lgn = torch.empty((Bn, 10), dtype=torch.int32, device="cuda")
        # multiply-accumulates of the network per image
        macs, hh, cc = 0, Hn, 3
        for co, pl in zip(couts, pools):
            macs += hh * hh * 9 * cc * co
            cc = co
            hh = hh // 2 if pl else hh
        fin = hh * hh * cc
        for fo in fcs:
            macs += fin * fo
            fin = fo

        def job_convnet():
            msn = time_secondary(lambda: q.qnn_binary_convnet_forward(Xn, 8, couts, pools, fcs, Wn, Tnd, Fnd, logits=lgn, workspace=wsn,
                                                                      engine=engine or 0), 20, 5)
            engs = q.qnn_last_engines()
            ok = np.array_equal(lgn[idxn].cpu().numpy(), wantn)
            extra["convnet_cifar10_forward_batch256"] = {
                "parity_sample_ok": bool(ok), "ms": msn if ok else None, "images_per_s": Bn / (msn * 1e-3) if ok else None,
                "engines_per_layer": [ENGINE_NAMES.get(e, str(e)) for e in engs],
                "effective_integer_tmacs": Bn * macs / (msn * 1e-3) / 1e12 if ok else None,
                "macs_per_image": macs}

        jobs.append((2, job_convnet))

    if "c4" in only:
        # Sec. 5, repetition of binary 2-D filters, on a layer of the CIFAR-10 ConvNet of App. A (128 -> 128 channels,
        # 3 x 3, 32 x 32 maps, batch 16, +-1 activations held as 2-bit codes so that zero padding is exact): the
        # convolution through the distinct filters against the direct one, and the fraction of filter applications left
        Bd, Hd, Cd = 16, 32, 128
        ud = qi.uniform_int(seed, 70, (Bd, Hd, Hd, Cd), 0, 1) * 2 + 1     # codes 1 (-1) and 3 (+1) of value = code - 2
        wd_h = qi.pm1(seed, 71, (Cd, 3, 3, Cd))
        wantd = oracle.conv2d(ud[:1], wd_h.astype(np.int32), 1)
        Ad = dev(np.stack([np_pack_bits((ud >> p) & 1) for p in range(2)]))
        Wd_ = dev(np_pack_pm1(wd_h))
        wsd = torch.empty(q._lib.qnn_conv2d_dedup_workspace_bytes(Bd, Hd, Hd, Cd, Cd, 1) * Bd, dtype=torch.uint8, device="cuda")
        od = torch.empty((Bd, Hd, Hd, Cd), dtype=torch.int32, device="cuda")
        resd = {}

        def run_dedup():
            resd["out"], resd["counts"] = q.qnn_conv2d_dedup(Ad, [1, 2], Cd, Wd_, 1, workspace=wsd)

        def job_dedup():
            msd = time_secondary(run_dedup, 20, 5)
            msdir = time_secondary(lambda: q.qnn_bitplane_conv2d(Ad, [1, 2], q.PLANE_BIT, Cd, Wd_[None], [1], q.PLANE_SIGN, 1, 1,
                                                             out=od, engine=engine), sec_steps, sec_warm)
            ok = (np.array_equal(resd["out"][:1].cpu().numpy(), wantd) and np.array_equal(od[:1].cpu().numpy(), wantd))
            uniq = int(resd["counts"].sum().item())
            extra["filter_dedup_cifar_layer_128x128"] = {
                "parity_sample_ok": bool(ok), "distinct_2d_filters": uniq, "of": Cd * Cd,
                "fraction_of_filter_applications_left": uniq / (Cd * Cd),
                "ms_through_distinct_filters": msd if ok else None, "ms_direct": msdir if ok else None,
                "note": "random +-1 weights (the paper's 42 % is for trained ones); the direct product is the fast path"}

        jobs.append((1, job_dedup))

    if "c1" in only:
        xa_h, xw_h = qi.normal_f32(seed, 10, (128, 1024)), qi.normal_f32(seed, 11, (1024, 1024))
        want1 = oracle.gemm_pm1(oracle.sign(xa_h), oracle.sign(xw_h))
        xa, xw = dev(xa_h), dev(xw_h)
        A1 = torch.empty((128, 32), dtype=torch.int32, device="cuda")
        W1 = torch.empty((1024, 32), dtype=torch.int32, device="cuda")
        C1 = torch.empty((128, 1024), dtype=torch.int32, device="cuda")

        def c1():
            q.qnn_pack_sign(xa, out=A1)
            q.qnn_pack_sign(xw, out=W1)
            q.qnn_binary_gemm(A1, W1, 1024, out=C1, engine=engine)

        def job_c1():
            ms1 = time_secondary(c1, max(sec_steps, 100), sec_warm)
            ok = np.array_equal(C1.cpu().numpy(), want1)
            ms1g = time_secondary(lambda: q.qnn_binary_gemm(A1, W1, 1024, out=C1, engine=engine), max(sec_steps, 100), sec_warm)
            # cold: 72 rotating copies of the fp32 inputs (325 MB > the 256 MB last-level cache), one event pair per call
            nset = 72
            xas = [xa.clone() for _ in range(nset)]
            xws = [xw.clone() for _ in range(nset)]
            state = {"i": 0}

            def c1_cold():
                i = state["i"] % nset
                state["i"] += 1
                q.qnn_pack_sign(xas[i], out=A1)
                q.qnn_pack_sign(xws[i], out=W1)
                q.qnn_binary_gemm(A1, W1, 1024, out=C1, engine=engine)

            for _ in range(nset):
                c1_cold()
            cold = per_call_ms(c1_cold, 2 * nset)
            extra["c1_pack_pack_gemm_128x1024x1024"] = {
                "parity_ok": bool(ok), "us_warm": ms1 * 1e3 if ok else None, "us_gemm_only_warm": ms1g * 1e3,
                "us_cold_inputs_median": statistics.median(cold) * 1e3, "us_cold_inputs_min": min(cold) * 1e3,
                "note": "three launches (two sign+pack, one product); cold = fp32 inputs rotated over 325 MB"}

        jobs.append((1, job_c1))

    if "c3" in only:
        def job_bw():
            # the bandwidth-bound kernels of the path at 8192 x 8192: sign+pack from fp32, threshold+repack of the int32
            # product, bit-plane split of 8-bit codes
            xf = torch.randn((n, n), dtype=torch.float32, device="cuda")  # values are irrelevant to the cost
            pk = torch.empty((n, n // 32), dtype=torch.int32, device="cuda")
            msp = time_secondary(lambda: q.qnn_pack_sign(xf, out=pk), sec_steps, sec_warm)
            gb = (n * n * 4 + n * n / 8) / (msp * 1e-3) / 1e9
            extra["pack_sign_8192x8192"] = {"ms": msp, "GBps": gb, "frac_of_hbm_peak": gb / HBM_PEAK_GBS}
            del xf, pk
            thr = torch.zeros((n,), dtype=torch.int32, device="cuda")
            tb = torch.empty((n, n // 32), dtype=torch.int32, device="cuda")
            mst = time_secondary(lambda: q.qnn_threshold_sign(C3, thr, None, out=tb), sec_steps, sec_warm)
            gb = (n * n * 4 + n * n / 8 + n * 4) / (mst * 1e-3) / 1e9
            extra["threshold_sign_8192x8192"] = {"ms": mst, "GBps": gb, "frac_of_hbm_peak": gb / HBM_PEAK_GBS}
            codes = torch.randint(0, 256, (n, n), dtype=torch.uint8, device="cuda")
            pl = torch.empty((8, n, n // 32), dtype=torch.int32, device="cuda")
            msb = time_secondary(lambda: q.qnn_pack_bitplanes(codes, 8, out=pl), sec_steps, sec_warm)
            gb = (n * n + n * n) / (msb * 1e-3) / 1e9
            extra["pack_bitplanes_8192x8192_8bit"] = {"ms": msb, "GBps": gb, "frac_of_hbm_peak": gb / HBM_PEAK_GBS}
            del codes, pl
            # quantizer front ends of Sec. 3 from fp32: 2-bit linear codes; 8-bit fixed-point log values with the
            # straight-through gate (two fp32 arrays read); transpose of an 8192 x 8192 bit matrix
            xq = torch.randn((n, n), dtype=torch.float32, device="cuda")
            pl2 = torch.empty((2, n, n // 32), dtype=torch.int32, device="cuda")
            msq = time_secondary(lambda: q.qnn_linear_quant_planes(xq, 0.5, 0, 3, 2, out=pl2), sec_steps, sec_warm)
            gb = (n * n * 4 + 2 * n * n / 8) / (msq * 1e-3) / 1e9
            extra["linear_quant_planes_8192x8192_2bit"] = {"ms": msq, "GBps": gb, "frac_of_hbm_peak": gb / HBM_PEAK_GBS}
            gate = torch.randn((n, n), dtype=torch.float32, device="cuda")
            pl8 = torch.empty((8, n, n // 32), dtype=torch.int32, device="cuda")
            msl = time_secondary(lambda: q.qnn_log_quant_planes(xq, -6, 0, 8, as_value=True, gate=gate, out=pl8), sec_steps, sec_warm)
            gb = (2 * n * n * 4 + 8 * n * n / 8) / (msl * 1e-3) / 1e9
            extra["log_quant_planes_8192x8192_8bit_gated"] = {"ms": msl, "GBps": gb, "frac_of_hbm_peak": gb / HBM_PEAK_GBS}
            del xq, gate, pl8
            tb2 = torch.empty((1, n, n // 32), dtype=torch.int32, device="cuda")
            mstr = time_secondary(lambda: q.qnn_transpose_bits(pl2[:1], n, out=tb2), sec_steps, sec_warm)
            gb = (2 * n * n / 8) / (mstr * 1e-3) / 1e9
            extra["transpose_bits_8192x8192"] = {"ms": mstr, "GBps": gb, "frac_of_hbm_peak": gb / HBM_PEAK_GBS}

        jobs.append((4, job_bw))

    def job_valu_probe():
        # the vector-ALU rate that the 1258 TOP/s peak of the xor + popcount engine assumes, measured: sixteen
        # register-resident {xor, popcount-accumulate} pairs per lane and iteration on every SIMD of the chip
        blocks, iters = 256 * 32, 4096
        sink = torch.empty((blocks * 256,), dtype=torch.int32, device="cuda")
        ms = time_secondary(lambda: q.qnn_probe_valu_peak(sink, blocks, iters), 10, 3)
        tops = 2.0 * blocks * 256 * iters * 16 * 32 / (ms * 1e-3) / 1e12
        extra["valu_xor_popcount_probe"] = {"ms": ms, "TOPS": tops, "assumed_peak_TOPS": VALU_PEAK_TOPS,
                                            "frac_of_assumed_peak": tops / VALU_PEAK_TOPS}

    def job_mfma_probe():
        # the rate the matrix cores sustain on the FP4 instruction alone (operands in registers, one wave per SIMD on
        # every CU, about 0.1 s per pattern): what the 10.1 POP/s peak becomes under this card's power management
        blocks, iters = 256, 200000
        sink = torch.empty((blocks * 256,), dtype=torch.float32, device="cuda")
        res = {}
        for name, bits, vary in (("zero_operands", 0, False), ("all_ones", 0x22222222, False),
                                 ("zeros_and_ones_at_random", 0x22222222, True), ("random_nibbles", 0xFFFFFFFF, True)):
            s0 = torch.zeros(3, dtype=torch.int64, device="cuda")
            s1 = torch.zeros(3, dtype=torch.int64, device="cuda")

            def run(bits=bits, vary=vary):
                q.qnn_probe_mfma_fp4_peak(sink, blocks, iters, bits, vary)

            run()
            q.qnn_stamp_clocks(s0)
            ms = time_steps(run, 2, 0)
            q.qnn_stamp_clocks(s1)
            torch.cuda.synchronize()
            tops = 2.0 * blocks * 4 * iters * 16 * 65536 / (ms * 1e-3) / 1e12
            res[name] = {"ms": ms, "TOPS": tops, "frac_of_fp4_peak": tops / MFMA_FP4_PEAK_TOPS,
                         "avg_sclk_mhz": q.average_shader_clock_mhz(s0, s1)}
        extra["mfma_fp4_probe"] = res

    if "c1" in only:
        jobs.append((0, job_valu_probe))
        jobs.append((0, job_mfma_probe))

    # ================================================================ GPU work, back to back
    primary = {}

    def job_primary():
        # Per-call pass first: a train of these launches that starts on a card which has been idle, or busy with other
        # kinds of kernels, for a few milliseconds runs 15 - 30 % slower between its 10th and 100th call (the power
        # management first boosts, then throttles, then settles) whatever came before; the pass records that ramp
        # call by call, and the timed region that follows it (W warm-up calls, then exactly K timed ones) measures
        # the settled state a production loop runs in.
        primary["sclk_start"] = q.qnn_probe_shader_clock()
        primary["per_call"] = per_call_ms(run_c3, 300)
        primary["sclk_before"] = q.qnn_probe_shader_clock()
        primary["ms"] = time_steps(run_c3, steps, warmup)
        primary["sclk_after"] = q.qnn_probe_shader_clock()
        primary["engine"] = q.qnn_last_engine()
        primary["parity"] = bool(np.array_equal(C3[rows3].cpu().numpy(), want3))

    log("[bench] GPU phase")
    # small and latency-bound workloads first, then the matrix-core ones, the kernels that stream 8192 x 8192 arrays
    # through HBM last: the card reaches the primary configuration from sustained load on both its matrix cores and
    # its memory system
    jobs = [j for _, j in sorted(jobs, key=lambda pj: pj[0])]
    order = [job_primary] + jobs if args.primary_first else jobs + [job_primary]
    for job in order:
        job()
    ms3 = primary["ms"]
    assert primary["parity"], "C3 output differs from the oracle: no throughput is reported"
    tops3 = ops3 / (ms3 * 1e-3) / 1e12
    used = primary["engine"]
    used_name = ENGINE_NAMES[used]
    sclk = 0.5 * (primary["sclk_before"] + primary["sclk_after"])
    log(f"[bench] C3 8192^3: {ms3:.4f} ms/step, {tops3:.1f} binary TOPS, shader clock {primary['sclk_before']:.0f} -> "
        f"{primary['sclk_after']:.0f} MHz")
    extra["c3_tops_including_pack_of_both_operands_from_fp32"] = (
        ops3 / ((ms3 + 2 * extra["pack_sign_8192x8192"]["ms"]) * 1e-3) / 1e12 if "pack_sign_8192x8192" in extra else None)

    peak = ENGINE_PEAK[used]
    roof = {"bound": "alu" if used == 1 else "mfma", "achieved": tops3, "peak": peak, "unit": "TOP/s", "frac": tops3 / peak,
            "traffic": None,
            "kernel": {1: "gemm_valu_kernel", 2: "gemm_mfma_kernel", 3: "gemm_panel_kernel<false, 4, false, false>"}[used],
            "peak_dtype": {1: "integer vector ALU: one xor and one popcount-accumulate per 32 MACs",
                           2: "int8 dense MFMA, int32 accumulate",
                           3: "fp4 (E2M1) dense MFMA, fp32 accumulate"}[used],
            "frac_at_observed_clock": tops3 / (peak * sclk / NOMINAL_MHZ) if sclk == sclk and sclk > 0 else None,
            "frac_of_int8_mfma_peak": tops3 / MFMA_I8_PEAK_TOPS,
            "frac_of_valu_xor_popcount_peak": tops3 / VALU_PEAK_TOPS}
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        try:
            t = json.load(open(tpath)).get(roof["kernel"] + "@c3")
            if t:
                roof["traffic"] = t["fetch_bytes"] + t["write_bytes"]  # HBM bytes per launch from the committed rocprofv3 runs
                roof["traffic_detail"] = t
        except Exception:
            pass

    if args.traffic_probe:
        D3 = torch.empty_like(C3)
        xf = torch.randn((n, n), dtype=torch.float32, device="cuda")
        pk = torch.empty((n, n // 32), dtype=torch.int32, device="cuda")
        for _ in range(3):
            D3.copy_(C3)  # 268 435 456 bytes read + the same written per call
            D3.zero_()    # 268 435 456 bytes written, nothing read
            q.qnn_pack_sign(xf, out=pk)  # 268 435 456 bytes read, 8 388 608 written
        torch.cuda.synchronize()
        del D3, xf, pk

    # ================================================================ CPU baseline: the oracle, as it stands
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

    calls = primary["per_call"]
    out = {
        "metric": "binary GEMM TOPS (1 +-1 MAC = 2 ops) at 8192^3 + MLP forward samples/sec",
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
                   "engine": used_name, "M": n, "N": n, "K": n,
                   "order": "primary first" if args.primary_first else "primary after the secondary configurations"},
        "mlp_forward_samples_per_s": extra.get("c2_mlp_forward", {}).get("samples_per_s"),
        "sclk_mhz": {"before_per_call_pass": primary["sclk_start"], "before_timed_region": primary["sclk_before"],
                     "after_timed_region": primary["sclk_after"], "nominal": NOMINAL_MHZ},
        "per_call_ms": {"calls": len(calls), "median": statistics.median(calls), "min": min(calls),
                        "first5": calls[:5], "calls_10_to_30_mean": sum(calls[10:30]) / 20.0, "last5": calls[-5:],
                        "note": "a separate pass right before the warm-up of the timed region, one event pair per call: it "
                                "shows the ramp of a train of launches that starts on a card not under this load"},
        "roofline": roof,
        "roofline_c2": extra.pop("roofline_c2", None),
        "cpu_baseline": cpu,
        "secondary": extra,
        "paper_context": "paper reports only ratios on a GTX750: XNOR kernel 23x its baseline kernel, 3.4x cuBLAS at 8192^3; MLP 7x",
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
