#!/usr/bin/env python3
"""Benchmark of the QLESS hot path on one MI355X.

A step streams one batch of 64 training examples through the whole path at the 7B-class LoRA
shape: for each of C = 4 checkpoints the [64, 2^27] bf16 gradient batch is projected to
k = 8192 (Rademacher) and quantised to 1 bit into the datastore; the 64 new rows are scored
against the resident validation datastore (M = 512, 4 checkpoints, max over validation) and
the top 5 % of the N = 65536 running score vector is selected.  Inputs are synthetic and
resident in HBM before the timed region.

value = projected+quantised gradient vectors per second over the whole step.  The same run also
times the scoring-only workload (N = 270000, M = 1024, k = 8192, C = 4, 1-bit) and the CPU oracle
on a bounded sample; both are reported on the same JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "projected+quantised grads/sec (d=134M,k=8192) and train×val scores/sec, 1-bit"
PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA, published
PEAK_HBM_GBS = 8000.0


def log(msg):
    print("[bench] " + msg, file=sys.stderr, flush=True)


def _time_ms(torch, fn, reps=3, warm=1):
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


def _store(torch, Q, dev, rows, k, C, seed, sbits):
    codes, rnorm = [], []
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    for c in range(C):
        cc = torch.empty(rows, Q.code_bytes(k, sbits), dtype=torch.uint8, device=dev)
        rr = torch.empty(rows, dtype=torch.float32, device=dev)
        ss = torch.empty(rows, dtype=torch.float32, device=dev)
        for r0 in range(0, rows, 16384):
            r1 = min(rows, r0 + 16384)
            Q.quantize(torch.randn(r1 - r0, k, generator=gen, device=dev), sbits, codes=cc[r0:r1], S=ss[r0:r1], rnorm=rr[r0:r1])
        codes.append(cc)
        rnorm.append(rr)
    return codes, rnorm


def leg_sliced(torch, Q, synth, dev, G, eta, log):
    out, C = {}, 4
    # ---- sliced datastore build (Sec. 3.1): the 7B-class gradient as 128 per-matrix slices of 2^20 columns
    n, d, k = G[0].shape[0], G[0].shape[1], 8192
    if d >= 1 << 24:
        nsl, sl = 128, d // 128
        Pa = torch.empty(n, k, dtype=torch.float32, device=dev)
        Pb = torch.empty(n, k, dtype=torch.float32, device=dev)
        ws_a = torch.empty(max(Q.project_workspace(n, sl, k), 16), dtype=torch.uint8, device=dev)
        ws_b = torch.empty_like(ws_a)
        ws_w = torch.empty(max(Q.project_workspace(n, d, k), 16), dtype=torch.uint8, device=dev)
        codes = torch.empty(n, Q.code_bytes(k, 1), dtype=torch.uint8, device=dev)
        S = torch.empty(n, dtype=torch.float32, device=dev)
        rn = torch.empty(n, dtype=torch.float32, device=dev)
        g = G[0]

        def whole():
            Q.project_quantize_slice(g, k, 0, Pa, True, True, bits=1, codes=codes, S=S, rnorm=rn, ws=ws_w)

        def one_stream():
            for i in range(nsl):
                Q.project_quantize_slice(g[:, i * sl:(i + 1) * sl], k, i * sl, Pa, i == 0, i == nsl - 1, bits=1,
                                         codes=codes, S=S, rnorm=rn, ws=ws_a)

        s2 = torch.cuda.Stream()

        def two_streams():
            main = torch.cuda.current_stream()
            s2.wait_stream(main)
            for i in range(nsl - 1):                          # even slices here, odd ones on the second stream
                piece = g[:, i * sl:(i + 1) * sl]
                if i % 2 == 0:
                    Q.project_quantize_slice(piece, k, i * sl, Pa, i == 0, False, ws=ws_a)
                else:
                    with torch.cuda.stream(s2):
                        Q.project_quantize_slice(piece, k, i * sl, Pb, i == 1, False, ws=ws_b)
            i = nsl - 1                                       # odd: the last slice joins both sums on the second stream
            s2.wait_stream(main)
            with torch.cuda.stream(s2):
                Q.project_quantize_slice(g[:, i * sl:], k, i * sl, Pb, False, True, bits=1, P_other=Pa,
                                         codes=codes, S=S, rnorm=rn, ws=ws_b)
            main.wait_stream(s2)

        tw = _time_ms(torch, whole, reps=2)
        t1 = _time_ms(torch, one_stream, reps=2)
        t2 = _time_ms(torch, two_streams, reps=2)
        out["sliced_build_1bit"] = {"workload": "one checkpoint's [64, 2^%d] bf16 batch -> k=8192, 1-bit, as %d slices of %d columns"
                                                % (d.bit_length() - 1, nsl, sl),
                                    "whole_ms": round(tw, 3), "slices_one_stream_ms": round(t1, 3),
                                    "slices_two_streams_ms": round(t2, 3)}
        log("sliced build: whole %.2f ms, %d slices on one stream %.2f ms, alternating on two streams %.2f ms" % (tw, nsl, t1, t2))
        del Pa, Pb, ws_a, ws_b, ws_w
    return out


def leg_config5(torch, Q, synth, dev, eta, log):
    out, C = {}, 4
    # ---- config 5: Gaussian projection d = 2^28 -> 16384, a batch of 128; 2-bit scoring 8192 x 256 x 4; top-409
    n5, d5, k5 = 128, 1 << 28, 16384
    g5, _ = synth.student_t_gradients(n5, d5, seed=5100, device=dev, dtype=torch.bfloat16)
    ws5 = torch.empty(max(Q.project_workspace(n5, d5, k5), 16), dtype=torch.uint8, device=dev)
    P5 = torch.empty(n5, k5, dtype=torch.float32, device=dev)
    t5 = _time_ms(torch, lambda: Q.project(g5, k5, kind=Q.GAUSSIAN, seed=1, out=P5, ws=ws5), reps=2)
    fl5 = 2.0 * n5 * d5 * k5
    out["config5_project_gaussian"] = {"workload": "[128, 2^28] bf16 -> k=16384, Gaussian table entries", "ms": round(t5, 2),
                                       "grads_per_s": round(n5 / (t5 * 1e-3), 2), "TFLOPs": round(fl5 / (t5 * 1e-3) / 1e12, 1),
                                       "bf16_mfma_frac": round(fl5 / (t5 * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)}
    log("config 5 Gaussian projection [128, 2^28] -> 16384: %.1f ms = %.0f TFLOP/s" % (t5, fl5 / (t5 * 1e-3) / 1e12))
    del g5, ws5, P5
    torch.cuda.empty_cache()
    N5, M5 = 8192, 256
    tc5, tr5 = _store(torch, Q, dev, N5, k5, C, 510, 2)
    vc5, vr5 = _store(torch, Q, dev, M5, k5, C, 520, 2)
    sc5 = torch.empty(N5, dtype=torch.float32, device=dev)
    wss = torch.empty(max(Q.score_workspace(N5, M5, k5, 2, C), 16), dtype=torch.uint8, device=dev)
    wst = torch.empty(max(Q.topk_workspace(N5, 409), 16), dtype=torch.uint8, device=dev)
    ts = _time_ms(torch, lambda: Q.score(tc5, tr5, vc5, vr5, eta, k5, 2, score_out=sc5, ws=wss))
    tt = _time_ms(torch, lambda: Q.topk(sc5, 409, ws=wst))
    macs = float(N5) * M5 * C * k5
    out["config5_score_2bit"] = {"workload": "N=8192 M=256 k=16384 C=4, 2-bit; top-409", "ms": round(ts, 4),
                                 "pair_scores_per_s": round(N5 * M5 / (ts * 1e-3), 1),
                                 "mfma_frac": round(macs / (ts * 1e-3) / 5.05e15, 4), "mfma_peak": "fp4 10.1 POP/s",
                                 "hbm_frac": round(C * (N5 + M5) * (k5 // 4) / (ts * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                                 "topk_409_ms": round(tt, 4)}
    log("config 5 score 2-bit 8192x256x4 k=16384: %.3f ms; top-409 %.3f ms" % (ts, tt))
    del tc5, tr5, vc5, vr5

    return out


def leg_config2(torch, Q, synth, dev, eta, log):
    out, C = {}, 4
    # ---- config 2: N = 16384, M = 256, k = 2048, C = 4, all four widths; top-819
    N2, M2, k2 = 16384, 256, 2048
    for sb in (8, 4, 2, 1):
        tc2, tr2 = _store(torch, Q, dev, N2, k2, C, 210 + sb, sb)
        vc2, vr2 = _store(torch, Q, dev, M2, k2, C, 220 + sb, sb)
        sc2 = torch.empty(N2, dtype=torch.float32, device=dev)
        wss = torch.empty(max(Q.score_workspace(N2, M2, k2, sb, C), 16), dtype=torch.uint8, device=dev)
        wst = torch.empty(max(Q.topk_workspace(N2, 819), 16), dtype=torch.uint8, device=dev)
        ts = _time_ms(torch, lambda: Q.score(tc2, tr2, vc2, vr2, eta, k2, sb, score_out=sc2, ws=wss), reps=5)
        tt = _time_ms(torch, lambda: Q.topk(sc2, 819, ws=wst), reps=5)
        out["config2_score_%dbit" % sb] = {"workload": "N=16384 M=256 k=2048 C=4; top-819", "ms": round(ts, 4),
                                           "pair_scores_per_s": round(N2 * M2 / (ts * 1e-3), 1),
                                           "hbm_frac": round(C * (N2 + M2) * Q.code_bytes(k2, sb) / (ts * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                                           "mfma_frac": round(float(N2) * M2 * C * k2 / (ts * 1e-3) / (5.05e15 if sb <= 2 else 2.5e15), 4),
                                           "topk_819_ms": round(tt, 4)}
        log("config 2 score %d-bit 16384x256x4 k=2048: %.3f ms; top-819 %.3f ms" % (sb, ts, tt))
    n2, d2 = 2048, 1 << 20
    g2, _ = synth.student_t_gradients(n2, d2, seed=2100, device=dev, dtype=torch.bfloat16)
    ws2 = torch.empty(max(Q.project_workspace(n2, d2, k2), 16), dtype=torch.uint8, device=dev)
    P2 = torch.empty(n2, k2, dtype=torch.float32, device=dev)
    t2p = _time_ms(torch, lambda: Q.project(g2, k2, seed=11, out=P2, ws=ws2), reps=3)
    fl2 = 2.0 * n2 * d2 * k2
    out["config2_project"] = {"workload": "[2048, 2^20] bf16 -> k=2048, Rademacher", "ms": round(t2p, 3),
                              "grads_per_s": round(n2 / (t2p * 1e-3), 1),
                              "bf16_mfma_frac": round(fl2 / (t2p * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)}
    log("config 2 projection [2048, 2^20] -> 2048: %.2f ms = %.0f TFLOP/s" % (t2p, fl2 / (t2p * 1e-3) / 1e12))
    del g2, ws2, P2

    return out


def leg_variants(torch, Q, synth, dev, eta, log):
    out, C = {}, 4
    # ---- variants at the large-datastore shape: mixed precision and fused group aggregation (1-bit train codes)
    N4, M4, k = 270000, 1024, 8192
    tc4, tr4 = _store(torch, Q, dev, N4, k, C, 40, 1)
    vc4, vr4 = _store(torch, Q, dev, M4, k, C, 50, 1)
    gen = torch.Generator(device=dev)
    gen.manual_seed(61)
    v16 = []
    for _ in range(C):
        t16 = torch.empty(M4, k, dtype=torch.bfloat16, device=dev)
        Q.normalize16(torch.randn(M4, k, generator=gen, device=dev), out=t16)
        v16.append(t16)
    wsm = torch.empty(max(Q.score_mixed_workspace(N4, M4, k, 1, C), 16), dtype=torch.uint8, device=dev)

    def mixed():
        Q.score_mixed(tc4, tr4, v16, eta, k, 1, ws=wsm)
    tm = _time_ms(torch, mixed, reps=2)
    out["score_mixed_1bit_M1024"] = {"workload": "N=270000 1-bit train codes x M=1024 bfloat16 validation rows, k=8192 C=4",
                                     "ms": round(tm, 3), "pair_scores_per_s": round(N4 * M4 / (tm * 1e-3), 1),
                                     "bf16_mfma_frac": round(2.0 * N4 * M4 * C * k / (tm * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)}
    log("mixed-precision score (1-bit train x bf16 val) 270000x1024x4: %.2f ms" % tm)
    del wsm, v16
    ends = [128 * (t + 1) for t in range(8)]
    wsg = torch.empty(max(Q.score_groups_workspace(N4, M4, k, 1, C), 16), dtype=torch.uint8, device=dev)
    og = torch.empty(N4, 8, dtype=torch.float32, device=dev)
    tg = _time_ms(torch, lambda: Q.score_groups(tc4, tr4, vc4, vr4, eta, k, 1, ends, Q.AGG_MEAN, out=og, ws=wsg), reps=2)
    full = torch.empty(N4, M4, dtype=torch.float32, device=dev)
    wsf = torch.empty(max(Q.score_workspace(N4, M4, k, 1, C), 16), dtype=torch.uint8, device=dev)

    def unfused():
        Q.score(tc4, tr4, vc4, vr4, eta, k, 1, want_score=False, want_full=True, full_out=full, ws=wsf)
        Q.aggregate(full, ends, Q.AGG_MEAN, out=og)
    tu = _time_ms(torch, unfused, reps=2)
    out["score_groups_1bit_M1024"] = {"workload": "N=270000 M=1024 k=8192 C=4 1-bit, mean over 8 groups of 128 validation vectors",
                                      "fused_ms": round(tg, 3), "score_full_then_aggregate_ms": round(tu, 3),
                                      "matrix_bytes_avoided": N4 * M4 * 4}
    log("group means 270000x1024 -> 8 groups: fused %.2f ms, full matrix + aggregate %.2f ms" % (tg, tu))
    return out


def extra_legs(torch, Q, synth, dev, G, eta, log):
    """Legs beside the headline step: the sliced datastore build on one and two streams, the other benchmark
    configurations at their own shapes, and the variants of the path (mixed precision, fused group aggregation)."""
    out = leg_sliced(torch, Q, synth, dev, G, eta, log)
    G.clear()
    torch.cuda.empty_cache()
    out.update(leg_config5(torch, Q, synth, dev, eta, log))
    out.update(leg_config2(torch, Q, synth, dev, eta, log))
    out.update(leg_variants(torch, Q, synth, dev, eta, log))
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--bits", type=int, default=1, choices=[1, 2, 4, 8])
    ap.add_argument("--d-log2", type=int, default=27, help="gradient dimension 2^x (27 = the metric's shape)")
    ap.add_argument("--skip-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--skip-scoring", action="store_true", help="skip the scoring-only leg")
    ap.add_argument("--sweep", action="store_true",
                    help="scoring leg over all four code widths and the validation-set sizes 8 ... 1024")
    ap.add_argument("--only", choices=["config5", "config2", "variants"], default=None,
                    help="run one of the extra legs alone and print its figures (short runs for the profiler)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (reference for profiler byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (no collectives on the path); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2502_01703_amd import binding as Q
    from paper_2502_01703_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    Q.lib()
    if args.only:
        leg = {"config5": leg_config5, "config2": leg_config2, "variants": leg_variants}[args.only]
        if args.calibrate_copy:
            src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
            src.clone()
            torch.cuda.synchronize()
            del src
        print(json.dumps({"only": args.only, "legs": leg(torch, Q, synth, dev, [1.0, 0.75, 0.5, 0.25], log)}), flush=True)
        return

    n, d, k, C, M, N, bits = 64, 1 << args.d_log2, 8192, 4, 512, 65536, args.bits
    k_sel = int(0.05 * N)
    eta = [1.0, 0.75, 0.5, 0.25]

    # ---------------------------------------------------------------- resident synthetic inputs
    t0 = time.time()
    G = []
    for c in range(C):
        g, _ = synth.student_t_gradients(n, d, seed=3000 + c, device=dev, dtype=torch.bfloat16)
        G.append(g)
    torch.cuda.synchronize()
    log("gradients: %d x [%d, 2^%d] bf16 = %.1f GiB resident (%.1f s)" %
        (C, n, args.d_log2, C * n * d * 2 / 2 ** 30, time.time() - t0))

    def synthetic_store(rows, seed, sbits):
        codes, rnorm = [], []
        for c in range(C):
            cc = torch.empty(rows, Q.code_bytes(k, sbits), dtype=torch.uint8, device=dev)
            rr = torch.empty(rows, dtype=torch.float32, device=dev)
            ss = torch.empty(rows, dtype=torch.float32, device=dev)
            gen = torch.Generator(device=dev)
            gen.manual_seed(seed + c)
            for r0 in range(0, rows, 16384):
                r1 = min(rows, r0 + 16384)
                P = torch.randn(r1 - r0, k, generator=gen, device=dev)
                Q.quantize(P, sbits, codes=cc[r0:r1], S=ss[r0:r1], rnorm=rr[r0:r1])
            codes.append(cc)
            rnorm.append(rr)
        return codes, rnorm

    train_codes, train_rnorm = synthetic_store(N, 10, bits)
    val_codes, val_rnorm = synthetic_store(M, 20, bits)
    train_S = [torch.empty(N, dtype=torch.float32, device=dev) for _ in range(C)]
    score = torch.zeros(N, dtype=torch.float32, device=dev)
    ws_score = torch.empty(max(Q.score_workspace(N, M, k, bits, C), 16), dtype=torch.uint8, device=dev)
    Q.score(train_codes, train_rnorm, val_codes, val_rnorm, eta, k, bits, score_out=score, ws=ws_score)
    P = torch.empty(n, k, dtype=torch.float32, device=dev)
    ws_proj = torch.empty(max(Q.project_workspace(n, d, k), 16), dtype=torch.uint8, device=dev)
    ws_topk = torch.empty(max(Q.topk_workspace(N, k_sel), 16), dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)       # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    proj_events = []

    def step(i, timed):
        b = (i * n) % N
        for c in range(C):
            if timed:
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
            Q.project(G[c], k, kind=Q.RADEMACHER, seed=0, out=P, ws=ws_proj)
            if timed:
                e1.record()
                proj_events.append((e0, e1))
            Q.quantize(P, bits, codes=train_codes[c][b:b + n], S=train_S[c][b:b + n],
                       rnorm=train_rnorm[c][b:b + n])
        Q.score([t[b:b + n] for t in train_codes], [t[b:b + n] for t in train_rnorm], val_codes,
                val_rnorm, eta, k, bits, score_out=score[b:b + n], ws=ws_score)
        return Q.topk(score, k_sel, ws=ws_topk)

    for i in range(args.warmup):
        step(i, False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i, True)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / max(args.steps, 1)
    grads_per_s = n * C / (ms_per_step * 1e-3)
    proj_ms = sum(a.elapsed_time(b) for a, b in proj_events) / max(len(proj_events), 1)
    flops = 2.0 * n * d * k
    achieved = flops / (proj_ms * 1e-3) / 1e12 if proj_ms > 0 else 0.0
    log("step %.2f ms; projection launch %.3f ms = %.1f TFLOP/s" % (ms_per_step, proj_ms, achieved))

    traffic = None      # HBM bytes per launch from the committed rocprofv3 --pmc summary
    tp = os.path.join(ROOT, "profiles", "project_kernel_c3_hbm_traffic.txt")
    if os.path.exists(tp) and args.d_log2 == 27:
        for line in open(tp):
            if line.startswith("hbm_bytes_per_launch"):
                traffic = int(line.split("=")[1])
    roofline = {"kernel": "project_kernel", "bound": "mfma", "achieved": round(achieved, 2),
                "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                "traffic": traffic,
                "traffic_source": ("profiles/project_kernel_c3_hbm_traffic.txt: rocprofv3 --pmc FETCH_SIZE, then "
                                   "WRITE_SIZE, of this kernel at this shape, each scaled by the same counter of a "
                                   "plain copy (a stored counter figure, not measured in this run)") if traffic else None,
                "flops_per_launch": flops, "avg_launch_ms": round(proj_ms, 4)}

    # ------------------------------------------------------------- scoring-only leg (1-bit, 270K x 1024)
    extra = {}
    if not args.skip_scoring:
        del train_codes, train_rnorm
        N4 = 270000
        oracle_sample = None
        for sb in ((1, 2, 4, 8) if args.sweep else (1, 8)):
            cbb = Q.code_bytes(k, sb)
            tc4, tr4 = synthetic_store(N4, 40, sb)
            vc4f, vr4f = synthetic_store(1024, 50, sb)
            sc4 = torch.empty(N4, dtype=torch.float32, device=dev)
            ws4 = torch.empty(max(Q.topk_workspace(N4, 13500), 16), dtype=torch.uint8, device=dev)
            # M = 1024: matrix-core bound; M = 8: HBM bound; 9 / 81 / 285: few-shot validation sets (Sec. 4.1)
            for M4 in ((1024, 285, 81, 64, 32, 16, 9, 8) if args.sweep else ((1024, 285, 81, 64, 8) if sb == 1 else (1024, 64, 8))):
                vc4, vr4 = [v[:M4] for v in vc4f], [v[:M4] for v in vr4f]
                wss = torch.empty(max(Q.score_workspace(N4, M4, k, sb, C), 16), dtype=torch.uint8, device=dev)
                Q.score(tc4, tr4, vc4, vr4, eta, k, sb, score_out=sc4, ws=wss)
                torch.cuda.synchronize()
                # enough back-to-back launches that the host's launch latency before the first one (tens of
                # microseconds with an idle GPU) does not weigh on kernels of a fraction of a millisecond
                reps = 3 if M4 > 285 else 20
                e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
                e[0].record()
                for _ in range(reps):
                    Q.score(tc4, tr4, vc4, vr4, eta, k, sb, score_out=sc4, ws=wss)
                e[1].record()
                for _ in range(reps):
                    Q.topk(sc4, 13500, ws=ws4)
                e[2].record()
                torch.cuda.synchronize()
                ts = e[0].elapsed_time(e[1]) / reps
                tt = e[1].elapsed_time(e[2]) / reps
                bytes_alg = C * (N4 + M4) * cbb + 4 * (N4 + M4) * C + 4 * N4
                macs = float(N4) * M4 * C * k
                # matrix-core peak of the path used: 1-bit codes run as FP4 (10.1 POP/s dense), 8-bit as int8 (5.0)
                mac_peak = 5.05e15 if sb <= 2 else 2.5e15
                mfma_frac = macs / (ts * 1e-3) / mac_peak
                hbm_frac = bytes_alg / (ts * 1e-3) / 1e9 / PEAK_HBM_GBS
                extra["score_%dbit_M%d" % (sb, M4)] = {
                    "workload": "N=270000 M=%d k=8192 C=4" % M4, "ms": round(ts, 3),
                    "pair_scores_per_s": round(N4 * M4 / (ts * 1e-3), 1),
                    "dots_per_s": round(N4 * M4 * C / (ts * 1e-3), 1),
                    "mfma_frac": round(mfma_frac, 4), "mfma_peak": "fp4 10.1 POP/s" if sb <= 2 else "int8 5.0 POP/s",
                    "hbm_frac": round(hbm_frac, 4), "binding": "mfma" if mfma_frac > hbm_frac else "hbm",
                    "topk_13500_ms": round(tt, 3)}
                log("score %d-bit 270000x%dx4: %.2f ms (%.3g pair scores/s, %.0f%% of %s MFMA peak, %.0f%% of HBM peak), topk %.3f ms" %
                    (sb, M4, ts, N4 * M4 / (ts * 1e-3), 100 * mfma_frac, "fp4" if sb <= 2 else "int8", 100 * hbm_frac, tt))
            if sb == 1 and not args.skip_cpu:      # rows for the oracle's scoring sample
                oracle_sample = ([t[:2048].cpu().numpy() for t in tc4], [t[:2048].cpu().numpy() for t in tr4],
                                 [v.cpu().numpy() for v in vc4f], [v.cpu().numpy() for v in vr4f])
            del tc4, tr4, vc4f, vr4f, vc4, vr4
        # the un-quantised 16-bit LESS store (Table 1 baseline) scored on the same machine, for comparison
        gen = torch.Generator(device=dev)
        gen.manual_seed(60)
        def store16(rows):
            out = []
            for _ in range(C):
                st16 = torch.empty(rows, k, dtype=torch.bfloat16, device=dev)
                for r0 in range(0, rows, 16384):
                    r1 = min(rows, r0 + 16384)
                    Q.normalize16(torch.randn(r1 - r0, k, generator=gen, device=dev), out=st16[r0:r1])
                out.append(st16)
            return out
        t16, v16 = store16(N4), store16(1024)
        ws16 = torch.empty(max(Q.score16_workspace(N4, 1024, k, C), 16), dtype=torch.uint8, device=dev)
        Q.score16(t16, v16, eta, ws=ws16)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(3):
            Q.score16(t16, v16, eta, ws=ws16)
        e1.record()
        torch.cuda.synchronize()
        t16ms = e0.elapsed_time(e1) / 3
        macs16 = float(N4) * 1024 * C * k
        extra["less16_M1024"] = {"workload": "N=270000 M=1024 k=8192 C=4, bfloat16 store (16-bit LESS comparator)",
                                 "ms": round(t16ms, 3), "pair_scores_per_s": round(N4 * 1024 / (t16ms * 1e-3), 1),
                                 "bf16_mfma_frac": round(2 * macs16 / (t16ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
                                 "store_bytes": C * N4 * k * 2, "store_bytes_1bit": C * N4 * (k // 8 + 8)}
        log("score 16-bit LESS store 270000x1024x4: %.2f ms (%.0f%% of bf16 MFMA peak), store %.2f GB vs %.2f GB at 1 bit" %
            (t16ms, 100 * 2 * macs16 / (t16ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, C * N4 * k * 2 / 1e9, C * N4 * (k // 8 + 8) / 1e9))
        del t16, v16, ws16
        # quantise throughput at the datastore size (HBM-bound kernel)
        Pq = torch.randn(N4, k, device=dev)
        cq = torch.empty(N4, Q.code_bytes(k, 1), dtype=torch.uint8, device=dev)
        sq = torch.empty(N4, dtype=torch.float32, device=dev)
        rq = torch.empty(N4, dtype=torch.float32, device=dev)
        Q.quantize(Pq, 1, codes=cq, S=sq, rnorm=rq)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            Q.quantize(Pq, 1, codes=cq, S=sq, rnorm=rq)
        e1.record()
        torch.cuda.synchronize()
        tq = e0.elapsed_time(e1) / 5
        qbytes = N4 * (4 * k + k // 8 + 8)
        extra["quantize_1bit"] = {"workload": "n=270000 k=8192", "ms": round(tq, 3),
                                  "vectors_per_s": round(N4 / (tq * 1e-3), 1),
                                  "GBps": round(qbytes / (tq * 1e-3) / 1e9, 1),
                                  "hbm_frac": round(qbytes / (tq * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)}
        log("quantize 1-bit 270000x8192: %.3f ms = %.0f GB/s" % (tq, qbytes / (tq * 1e-3) / 1e9))
        del Pq, cq

    g0_host = G[0][0:1].cpu()
    if not args.skip_scoring:
        extra.update(extra_legs(torch, Q, synth, dev, G, eta, log))
    del G

    # ----------------------------------------------------------------- CPU oracle on a bounded sample
    cpu = None
    if not args.skip_cpu:
        import numpy as np
        import oracle
        rows = list(range(0, k, 32))                       # 256 of the 8192 output coordinates
        g0 = g0_host
        t0 = time.perf_counter()
        oracle.project_rows(g0, rows, seed=0)
        t_proj = (time.perf_counter() - t0) * (k / len(rows))     # one gradient, all k coordinates
        Ps = np.random.default_rng(0).standard_normal((n, k)).astype(np.float32)
        t0 = time.perf_counter()
        oc, _, orn = oracle.quantize(Ps, bits)
        t_quant = time.perf_counter() - t0
        vcs = [v.cpu().numpy() for v in val_codes]
        vrs = [v.cpu().numpy() for v in val_rnorm]
        t0 = time.perf_counter()
        oracle.score([oc] * C, [orn] * C, vcs, vrs, eta, k, bits)
        t_score = time.perf_counter() - t0
        t0 = time.perf_counter()
        oracle.topk(score.cpu().numpy(), k_sel)
        t_topk = time.perf_counter() - t0
        t_step_cpu = n * C * t_proj + C * t_quant + t_score + t_topk
        cpu = {"value": round(n * C / t_step_cpu, 6), "unit": "grads/s", "cores": oracle.num_threads(),
               "kind": "oracle",
               "sample": "projection: 1 gradient (d=2^%d) x 256 of 8192 output coordinates, scaled x32; "
                         "quantise 64x8192; score 64x512x4; top-k over 65536" % args.d_log2,
               "seconds": {"project_per_gradient": round(t_proj, 3), "quantize_64": round(t_quant, 4),
                           "score_64x512x4": round(t_score, 4), "topk": round(t_topk, 4)}}
        log("oracle: %.1f s per projected gradient on %d threads" % (t_proj, cpu["cores"]))
        if not args.skip_scoring and oracle_sample is not None:
            t0 = time.perf_counter()
            oracle.score(*oracle_sample, eta, k, 1)
            t_sc = time.perf_counter() - t0
            cpu["scores"] = {"value": round(2048 * 1024 / t_sc, 1), "unit": "pair scores/s",
                             "sample": "2048 of the 270000 train rows x 1024 val x 4 checkpoints, 1-bit, k=8192",
                             "seconds": round(t_sc, 3)}
            log("oracle: %.3g pair scores/s (1-bit, 2048x1024x4 sample, %.2f s)" % (2048 * 1024 / t_sc, t_sc))

    out = {"metric": METRIC, "value": round(grads_per_s, 2), "unit": "grads/s", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
           "data": "synthetic",
           "config": {"workload": "7B-class LoRA shape: d=2^%d bf16, batch n=64, k=8192 Rademacher, C=4 "
                                  "checkpoints, %d-bit datastore, N=65536, M=512, top 5%%" % (args.d_log2, bits),
                      "step": "4 x (project+quantize 64 gradients) + score 64x512x4 + top-3276 of 65536"},
           "roofline": roofline, "cpu_baseline": cpu, "extra": extra}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
