#!/usr/bin/env python3
"""Benchmark of the W6A16 fp6_linear hot path on one MI355X.

Workload (configuration 5 of the benchmark definition): a 34B-class decoder stack - 48 layers, hidden 8192, MLP
22016, grouped-query attention (k/v projections 1024 x 8192) - with every linear layer
(q, k, v, o, gate, up, down) run as fp6_linear on its own packed FP6 weight.  One "step"
is one pass over all 336 linears (24.9 GB of packed weight, so the pass is cold in HBM
by construction).  Two legs are timed: M=1 (decode, HBM-bound: GB/s counting 0.75 byte
per weight) and M=512 (prefill, MFMA-bound: TFLOP/s counting 2*M*N*K).  `value` is the
M=1 leg; the M=512 leg is reported in the same JSON line under "m512".

Inputs are seeded synthetic tensors (paper_2312_08583_amd/inputs.py), resident in HBM
before the timed region.  A pass is captured once into a HIP graph and replayed, so the
timed region holds the kernels and nothing else.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_FP16_PEAK_TFLOPS = 2500.0
WORKLOAD = "cfg5_34b_stack"


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--layers", type=int, default=0, help="layers of the stack (0 = all 48)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-fp16-baseline", action="store_true")
    ap.add_argument("--legs", default="1,512", help="comma-separated M values to time")
    ap.add_argument("--no-fused", action="store_true",
                    help="skip the extra leg with q,k,v and gate,up concatenated along N (4 launches per layer)")
    ap.add_argument("--no-layout2", action="store_true",
                    help="skip the extra leg with the planes in layout 2 (hardware E3M2 -> fp16 conversion)")
    ap.add_argument("--no-ablation", action="store_true",
                    help="skip the bias-shift ablation on the paper's kernel-table shapes")
    ap.add_argument("--no-per-shape", action="store_true",
                    help="skip the per-shape breakdown (a profiler run then sees only the launches of the timed legs)")
    ap.add_argument("--no-ceilings", action="store_true",
                    help="skip the measured ceilings (plain read kernel, MFMA-only kernel) reported beside the nominal peaks")
    ap.add_argument("--no-mha", action="store_true",
                    help="skip the extra leg with full-size k,v projections (the stack without grouped-query attention)")
    ap.add_argument("--no-configs", action="store_true",
                    help="skip the table of the other benchmark configurations (1-4: every shape at every M, cold weights)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run a plain 1 GiB device copy (calibrates the HBM byte counters of a profiler run)")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2312_08583_amd as P
    from paper_2312_08583_amd import inputs

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    cfg = inputs.WORKLOADS[WORKLOAD]
    shapes = cfg["shapes"]
    layers = args.layers or cfg["layers"]

    # ---- build the stack: seeded weights -> packed planes (offline step, untimed)
    t0 = time.time()
    stack = []            # per layer: list of (N, K, hi, lo, scales)
    for layer in range(layers):
        mats = []
        for si, (_, N, K) in enumerate(shapes):
            W = inputs.workload_weight(WORKLOAD, si, layer=layer, device=dev)
            hi, lo, sc = P.fp6_quantize_pack(W)
            mats.append((N, K, hi, lo, sc))
            del W
        stack.append(mats)
    torch.cuda.synchronize()
    build_s = time.time() - t0
    weights_per_pass = sum(N * K for mats in stack for (N, K, *_) in mats)
    launches = sum(len(m) for m in stack)

    def make_leg(M):
        xs = {K: inputs.activation(M, K, seed=inputs.workload_seed(WORKLOAD, 9000 + M + K), device=dev)
              for K in sorted({K for (_, _, K) in shapes})}
        ys = {N: torch.empty((M, N), dtype=torch.float16, device=dev) for N in sorted({N for (_, N, _) in shapes})}
        need = max(P.fp6_linear_workspace_bytes(M, N, K) for (_, N, K) in shapes)
        ws = P.new_workspace(max(need, 16), dev)

        def one_pass():
            for mats in stack:
                for (N, K, hi, lo, sc) in mats:
                    P.fp6_linear(xs[K], hi, lo, sc, N, K, out=ys[N], workspace=ws)
        return one_pass, ys

    def time_passes(one_pass, steps, warmup):
        # capture one pass in a graph (eager pass first: module load, workspace touch)
        one_pass()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            one_pass()
        for _ in range(warmup):
            g.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / steps      # ms per pass

    if args.copy_probe:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)      # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    legs = [int(m) for m in args.legs.split(",")]
    res = {}
    for M in legs:
        one_pass, _ = make_leg(M)
        ms = time_passes(one_pass, args.steps, args.warmup)
        res[M] = dict(ms_per_step=ms,
                      gbs=0.75 * weights_per_pass / (ms * 1e-3) / 1e9,
                      tflops=2.0 * M * weights_per_pass / (ms * 1e-3) / 1e12)

    # ---- per-shape breakdown: the same launches grouped by shape (each shape over its `layers` distinct weights,
    # so every launch is cold), to show which kernel instance sits where against its roofline
    per_shape = {}
    for M in ([] if args.no_per_shape else legs):
        xs = {K: inputs.activation(M, K, seed=inputs.workload_seed(WORKLOAD, 9000 + M + K), device=dev)
              for K in sorted({K for (_, _, K) in shapes})}
        need = max(P.fp6_linear_workspace_bytes(M, N, K) for (_, N, K) in shapes)
        ws = P.new_workspace(max(need, 16), dev)
        rows = []
        for si, (name, N, K) in enumerate(shapes):
            y = torch.empty((M, N), dtype=torch.float16, device=dev)

            def sweep():
                for mats in stack:
                    _, _, hi, lo, sc = mats[si]
                    P.fp6_linear(xs[K], hi, lo, sc, N, K, out=y, workspace=ws)
            us = time_passes(sweep, max(3, args.steps // 4), 1) * 1e3 / len(stack)
            row = {"shape": "%s %dx%d" % (name, N, K), "us": round(us, 2)}
            if M <= 118:
                row["GB/s"] = round(0.75 * N * K / us / 1e3, 1)
                row["frac"] = round(0.75 * N * K / us / 1e3 / HBM_PEAK_GBS, 3)
            else:
                row["TFLOP/s"] = round(2.0 * M * N * K / us / 1e6, 1)
                row["frac"] = round(2.0 * M * N * K / us / 1e6 / MFMA_FP16_PEAK_TFLOPS, 3)
            rows.append(row)
        per_shape["M%d" % M] = rows

    # ---- measured ceilings: what kernels that do nothing else sustain on this machine, for reading the two
    # roofline fractions against (the nominal peaks stay the denominators of `frac`).  Each figure is
    # taken over about a second of back-to-back graph replays after half a second of the same work:
    # the shader clock takes some hundred milliseconds to settle under a new load.
    ceilings = None
    if not args.no_ceilings:
        def sustained(one_pass, warm_s=0.5, run_s=1.0):
            one_pass()
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                one_pass()
            t0 = time.time()
            while time.time() - t0 < warm_s:
                g.replay()
                torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            n, t0 = 0, time.time()
            e0.record()
            while time.time() - t0 < run_s:
                g.replay()
                n += 1
                torch.cuda.synchronize()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / n      # ms per pass

        ceilings = {}
        # (a) plain read of the same bytes in the same launch sizes: one launch per 4-bit plane of the
        # gate projections (90 MB each, a distinct buffer per layer, so every launch is cold)
        gate = [mats[4][2] for mats in stack]
        best = None
        for wgs in (1024, 2048, 4096):
            sink = torch.zeros(wgs * 4, dtype=torch.int32, device=dev)

            def read_pass():
                for hi in gate:
                    P.fp6_probe_read(hi, wgs, sink)
            ms = sustained(read_pass, 0.3, 0.5)
            gbs = sum(h.numel() for h in gate) / (ms * 1e-3) / 1e9
            if best is None or gbs > best[0]:
                best = (gbs, wgs, ms * 1e3 / len(gate))
        ceilings["plain_read_per_launch"] = {"GB/s": round(best[0], 1), "workgroups": best[1], "us_per_launch": round(best[2], 2),
                                             "what": "read-only kernel, one launch per 90 MB buffer, cold, graph replay"}
        big = torch.empty(1 << 31, dtype=torch.uint8, device=dev)
        sink = torch.zeros(4096 * 4, dtype=torch.int32, device=dev)
        big.random_(0, 256)
        ms = sustained(lambda: P.fp6_probe_read(big, 4096, sink), 0.3, 0.5)
        ceilings["plain_read_2GiB"] = {"GB/s": round(big.numel() / (ms * 1e-3) / 1e9, 1),
                                       "what": "read-only kernel, one launch over 2 GiB"}
        del big
        # (b) MFMA-only kernel (8 wavefronts per SIMD), with pseudo-random and with zero operands: the
        # clock the chip holds depends on the operand data
        wgs, iters, reps = 2048, 2000, 20
        sink = torch.zeros(wgs * 256, dtype=torch.float32, device=dev)
        for name, rnd in (("random_operands", True), ("zero_operands", False)):
            flop = P.fp6_probe_mfma(wgs, iters, rnd, sink) * reps

            def mfma_pass():
                for _ in range(reps):
                    P.fp6_probe_mfma(wgs, iters, rnd, sink)
            ms = sustained(mfma_pass)
            ceilings["mfma_only_" + name] = {"TFLOP/s": round(flop / (ms * 1e-3) / 1e12, 1), "us_per_launch": round(ms * 1e3 / reps, 1),
                                             "what": "v_mfma_f32_16x16x32_f16 on register operands, %d workgroups x 4 wavefronts, "
                                                     "sustained for a second" % wgs}

    # ---- extra leg: the stack without grouped-query attention (k and v projections 8192 x 8192 like q):
    # 38.9 G weights per step; the other five projections are those of the main legs
    mha = None
    if not args.no_mha:
        kv = []
        for layer in range(layers):
            pair = []
            for which in (1, 2):
                W = inputs.mha_kv_weight(WORKLOAD, which, layer=layer, device=dev)
                pair.append((W.shape[0], W.shape[1]) + tuple(P.fp6_quantize_pack(W)))
                del W
            kv.append(pair)
        mha = {"what": "k,v projections 8192x8192 (no grouped-query attention), %.2f G weights per step"
                       % ((weights_per_pass + sum(N * K - shapes[1][1] * shapes[1][2] for p_ in kv for (N, K, *_) in p_)) / 1e9)}
        wpp = weights_per_pass + sum(N * K - shapes[1][1] * shapes[1][2] for p_ in kv for (N, K, *_) in p_)
        for M in legs:
            xs = {K: inputs.activation(M, K, seed=inputs.workload_seed(WORKLOAD, 9000 + M + K), device=dev)
                  for K in sorted({K for (_, _, K) in shapes})}
            ys = {N: torch.empty((M, N), dtype=torch.float16, device=dev) for N in sorted({N for (_, N, _) in shapes})}
            need = max(P.fp6_linear_workspace_bytes(M, N, K) for (_, N, K) in shapes)
            ws = P.new_workspace(max(need, 16), dev)

            def mha_pass():
                for mats, pair in zip(stack, kv):
                    for si, (N, K, hi, lo, sc) in enumerate(mats):
                        if si in (1, 2):
                            N, K, hi, lo, sc = pair[si - 1]
                        P.fp6_linear(xs[K], hi, lo, sc, N, K, out=ys[N], workspace=ws)
            ms = time_passes(mha_pass, max(3, args.steps // 2), args.warmup)
            mha["M%d" % M] = ({"ms_per_step": ms, "value": 0.75 * wpp / (ms * 1e-3) / 1e9, "unit": "GB/s",
                               "frac": 0.75 * wpp / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
                              if M <= 118 else
                              {"ms_per_step": ms, "value": 2.0 * M * wpp / (ms * 1e-3) / 1e12, "unit": "TFLOP/s",
                               "frac": 2.0 * M * wpp / (ms * 1e-3) / 1e12 / MFMA_FP16_PEAK_TFLOPS})
        del kv

    # ---- extra leg: projections that read the same input concatenated along N, as inference engines
    # store them (q,k,v -> one [10240, 8192] weight; gate,up -> one [44032, 8192]).  Row scales are per
    # output channel and tiles are ordered by channel block, so the concatenated planes and scales ARE the
    # concatenation of the separate ones: same bytes, same results, 4 launches per layer instead of 7.
    fused = None
    if not args.no_fused:
        names = [n for (n, _, _) in shapes]
        groups = [[names.index(n) for n in g] for g in (("q", "k", "v"), ("o",), ("gate", "up"), ("down",))]
        fstack = []
        for mats in stack:
            fm = []
            for g in groups:
                Ks = {mats[i][1] for i in g}
                assert len(Ks) == 1
                fm.append((sum(mats[i][0] for i in g), Ks.pop(), torch.cat([mats[i][2] for i in g]),
                           torch.cat([mats[i][3] for i in g]), torch.cat([mats[i][4] for i in g])))
            fstack.append(fm)
        fused = {"launches_per_step": sum(len(m) for m in fstack),
                 "what": "q,k,v and gate,up concatenated along N (same planes, same scales, same results)"}
        for M in legs:
            xs = {K: inputs.activation(M, K, seed=inputs.workload_seed(WORKLOAD, 9000 + M + K), device=dev)
                  for K in sorted({K for (_, _, K) in shapes})}
            ys = {N: torch.empty((M, N), dtype=torch.float16, device=dev) for N in sorted({m[0] for m in fstack[0]})}
            ws = P.new_workspace(max(max(P.fp6_linear_workspace_bytes(M, m[0], m[1]) for m in fstack[0]), 16), dev)

            def fused_pass():
                for fm in fstack:
                    for (N, K, hi, lo, sc) in fm:
                        P.fp6_linear(xs[K], hi, lo, sc, N, K, out=ys[N], workspace=ws)
            ms = time_passes(fused_pass, args.steps, args.warmup)
            fused["M%d" % M] = ({"ms_per_step": ms, "value": 0.75 * weights_per_pass / (ms * 1e-3) / 1e9, "unit": "GB/s",
                                 "frac": 0.75 * weights_per_pass / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS} if M <= 118 else
                                {"ms_per_step": ms, "value": 2.0 * M * weights_per_pass / (ms * 1e-3) / 1e12,
                                 "unit": "TFLOP/s",
                                 "frac": 2.0 * M * weights_per_pass / (ms * 1e-3) / 1e12 / MFMA_FP16_PEAK_TFLOPS})
        del fstack

    # ---- extra leg: the same stack with the planes in layout 2 (4+2 planes arranged so that they merge into
    # the operand of gfx950's packed E3M2 -> fp16 conversion; same codes, scales and bytes)
    layout2 = None
    if not args.no_layout2:
        stack2 = []
        for layer in range(layers):
            mats = []
            for si, (_, N, K) in enumerate(shapes):
                W = inputs.workload_weight(WORKLOAD, si, layer=layer, device=dev)
                hi, lo, sc = P.fp6_quantize_pack_v2(W)
                mats.append((N, K, hi, lo, sc))
                del W
            stack2.append(mats)
        layout2 = {"what": "planes in layout 2: merged in registers and converted by v_cvt_scalef32_pk32_f16_bf6"}
        for M in legs:
            xs = {K: inputs.activation(M, K, seed=inputs.workload_seed(WORKLOAD, 9000 + M + K), device=dev)
                  for K in sorted({K for (_, _, K) in shapes})}
            ys = {N: torch.empty((M, N), dtype=torch.float16, device=dev) for N in sorted({N for (_, N, _) in shapes})}
            ws = P.new_workspace(max(max(P.fp6_linear_v2_workspace_bytes(M, N, K) for (_, N, K) in shapes), 16), dev)

            def pass2():
                for mats in stack2:
                    for (N, K, hi, lo, sc) in mats:
                        P.fp6_linear_v2(xs[K], hi, lo, sc, N, K, out=ys[N], workspace=ws)
            ms = time_passes(pass2, args.steps, args.warmup)
            layout2["M%d" % M] = ({"ms_per_step": ms, "value": 0.75 * weights_per_pass / (ms * 1e-3) / 1e9, "unit": "GB/s"}
                                  if M <= 118 else
                                  {"ms_per_step": ms, "value": 2.0 * M * weights_per_pass / (ms * 1e-3) / 1e12,
                                   "unit": "TFLOP/s"})
            # the same planes against bf16 activations (bf16 form of the conversion, bf16 MFMA, bf16 output)
            xb = {K: inputs.activation_bf16(M, K, seed=inputs.workload_seed(WORKLOAD, 9000 + M + K), device=dev)
                  for K in sorted({K for (_, _, K) in shapes})}
            yb = {N: torch.empty((M, N), dtype=torch.bfloat16, device=dev) for N in sorted({N for (_, N, _) in shapes})}

            def pass2b():
                for mats in stack2:
                    for (N, K, hi, lo, sc) in mats:
                        P.fp6_linear_v2_bf16(xb[K], hi, lo, sc, N, K, out=yb[N], workspace=ws)
            layout2["M%d" % M]["bf16_activations_ms_per_step"] = time_passes(pass2b, args.steps, args.warmup)
        del stack2

    # ---- fp16 dense GEMM on the same GPU, same stack (context, not the target)
    fp16 = None
    if not args.no_fp16_baseline:
        dense = [[P.fp6_dequantize(hi, lo, sc, N, K) for (N, K, hi, lo, sc) in mats] for mats in stack]
        fp16 = {}
        for M in legs:
            xs = {K: inputs.activation(M, K, seed=inputs.workload_seed(WORKLOAD, 9000 + M + K), device=dev)
                  for K in sorted({K for (_, _, K) in shapes})}

            def dense_pass():
                for mats, ws_ in zip(stack, dense):
                    for (N, K, *_), Wd in zip(mats, ws_):
                        torch.matmul(xs[K], Wd.t())
            for _ in range(2):
                dense_pass()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            n = max(3, args.steps // 4)
            e0.record()
            for _ in range(n):
                dense_pass()
            e1.record()
            torch.cuda.synchronize()
            fp16[str(M)] = dict(ms_per_step=e0.elapsed_time(e1) / n)
        del dense

    # ---- bias-shift ablation (Section 5.3: the same kernel without bias shift) on the six
    # feed-forward shapes of the paper's kernel table (Appendix B), batch 8, cold weights
    ablation = None
    if not args.no_ablation:
        B = P.binding
        modes = {"bias_shift": 0, "integer_rebias": B.FP6_HINT_DEQUANT(1), "fp16_multiply": B.FP6_HINT_DEQUANT(2)}
        tcfg = inputs.WORKLOADS["paper_table_b1"]
        M = tcfg["Ms"][0]
        ablation = {"M": M, "unit": "us", "shapes": {}}
        for si, (name, N, K) in enumerate(tcfg["shapes"]):
            W = inputs.workload_weight("paper_table_b1", si, device=dev)
            hi, lo, sc = P.fp6_quantize_pack(W)
            del W
            copies = max(2, min(64, int(1.0e9 / (0.75 * N * K))))
            pool = [(hi.clone(), lo.clone()) for _ in range(copies)]
            X = inputs.activation(M, K, seed=inputs.workload_seed("paper_table_b1", 500 + si), device=dev)
            Y = torch.empty((M, N), dtype=torch.float16, device=dev)
            row = {}
            for mode, hint in modes.items():
                ws = P.new_workspace(max(P.fp6_linear_variant_workspace_bytes(M, N, K, hint, 0), 16), dev)

                def sweep():
                    for (h, l) in pool:
                        P.fp6_linear_variant(X, h, l, sc, N, K, hint, 0, out=Y, workspace=ws)
                row[mode] = round(time_passes(sweep, 5, 2) * 1e3 / copies, 2)
            ablation["shapes"]["%s %dx%d" % (name, N, K)] = row
            del pool
        for mode in ("integer_rebias", "fp16_multiply"):
            r = [v[mode] / v["bias_shift"] for v in ablation["shapes"].values()]
            ablation["mean_slowdown_" + mode] = round(sum(r) / len(r), 3)

    # ---- fine-grained scales (Section 3: FGQ, one scale per 128 elements of a row) and FP5 E3M1 "4+1"
    # (Section 4, Section 6) against row-wise FP6 on the same six shapes, batch 8, cold weights
    fgq = None
    if not args.no_ablation:
        tcfg = inputs.WORKLOADS["paper_table_b1"]
        M, block = tcfg["Ms"][0], 128
        fgq = {"M": M, "block": block, "unit": "us", "shapes": {}}
        for si, (name, N, K) in enumerate(tcfg["shapes"]):
            W = inputs.workload_weight("paper_table_b1", si, device=dev)
            X = inputs.activation(M, K, seed=inputs.workload_seed("paper_table_b1", 500 + si), device=dev)
            Y = torch.empty((M, N), dtype=torch.float16, device=dev)
            copies = max(2, min(64, int(1.0e9 / (0.75 * N * K))))
            row = {}
            for mode in ("row_wise", "fgq", "fp5"):
                hi, lo, sc = (P.fp6_quantize_pack(W) if mode == "row_wise" else
                              P.fp6_quantize_pack_fgq(W, block) if mode == "fgq" else P.fp5_quantize_pack(W))
                pool = [(hi.clone(), lo.clone(), sc.clone()) for _ in range(copies)]
                need = (P.fp6_linear_workspace_bytes(M, N, K) if mode == "row_wise" else
                        P.fp6_linear_fgq_workspace_bytes(M, N, K, block) if mode == "fgq" else
                        P.fp5_linear_workspace_bytes(M, N, K))
                ws = P.new_workspace(max(need, 16), dev)

                def sweep():
                    for (h, l, s_) in pool:
                        if mode == "row_wise":
                            P.fp6_linear(X, h, l, s_, N, K, out=Y, workspace=ws)
                        elif mode == "fgq":
                            P.fp6_linear_fgq(X, h, l, s_, N, K, block, out=Y, workspace=ws)
                        else:
                            P.fp5_linear(X, h, l, s_, N, K, out=Y, workspace=ws)
                row[mode] = round(time_passes(sweep, 5, 2) * 1e3 / copies, 2)
                del pool
            fgq["shapes"]["%s %dx%d" % (name, N, K)] = row
            del W
        r = [v["fgq"] / v["row_wise"] for v in fgq["shapes"].values()]
        fgq["mean_slowdown_fgq"] = round(sum(r) / len(r), 3)
        r = [v["fp5"] / v["row_wise"] for v in fgq["shapes"].values()]
        fgq["mean_time_ratio_fp5"] = round(sum(r) / len(r), 3)       # bytes ratio: 0.625 / 0.75 = 0.833

    # ---- the other benchmark configurations (1-4): every shape at every M of the configuration, each timed
    # over a pool of distinct packed copies of at least 1 GB in turn, so every launch reads cold weights
    configs = None
    if not args.no_configs:
        configs = {}
        for wl in ("cfg1_single", "cfg2_llama7b", "cfg3_llama13b", "cfg4_llama70b_mlp"):
            c = inputs.WORKLOADS[wl]
            rows = []
            for si, (name, N, K) in enumerate(c["shapes"]):
                W = inputs.workload_weight(wl, si, device=dev)
                hi, lo, sc = P.fp6_quantize_pack(W)
                del W
                copies = max(2, min(64, int(1.0e9 / (0.75 * N * K)) + 1))
                pool = [(hi.clone(), lo.clone(), sc.clone()) for _ in range(copies)]
                for M in c["Ms"]:
                    X = inputs.activation(M, K, seed=inputs.workload_seed(wl, 500 + si) + M, device=dev)
                    Y = torch.empty((M, N), dtype=torch.float16, device=dev)
                    ws = P.new_workspace(max(P.fp6_linear_workspace_bytes(M, N, K), 16), dev)

                    def sweep():
                        for (h, l, s_) in pool:
                            P.fp6_linear(X, h, l, s_, N, K, out=Y, workspace=ws)
                    us = time_passes(sweep, 5, 2) * 1e3 / copies
                    t_hbm = 0.75 * N * K / (HBM_PEAK_GBS * 1e9) * 1e6
                    t_mfma = 2.0 * M * N * K / (MFMA_FP16_PEAK_TFLOPS * 1e12) * 1e6
                    rows.append({"shape": "%s %dx%d" % (name, N, K), "M": M, "us": round(us, 2),
                                 "GB/s": round(0.75 * N * K / us / 1e3, 1), "TFLOP/s": round(2.0 * M * N * K / us / 1e6, 1),
                                 "bound": "hbm" if t_hbm >= t_mfma else "mfma",
                                 "frac": round(max(t_hbm, t_mfma) / us, 3)})
                del pool
            configs[wl] = rows

    # ---- CPU oracle on a bounded sample of the same workload (reported baseline)
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import fp6_oracle as O
        sample = []
        for si, (_, N, K) in enumerate(shapes):
            W = inputs.workload_weight(WORKLOAD, si, layer=0, device=dev).cpu()
            codes, scales = O.quantize(W.view(torch.int16).numpy().view(np.uint16))     # untimed set-up
            sample.append((N, K, codes, scales))
        xs = {K: inputs.activation(1, K, seed=inputs.workload_seed(WORKLOAD, 9001 + K), device="cpu")
              .view(torch.int16).numpy().view(np.uint16) for K in sorted({K for (_, _, K) in shapes})}
        best = None
        for _ in range(3):
            t0 = time.time()
            for (N, K, codes, scales) in sample:
                O.linear(xs[K], codes, scales)
            dt = time.time() - t0
            best = dt if best is None else min(best, dt)
        wsample = sum(N * K for (N, K, *_) in sample)
        cpu = dict(value=0.75 * wsample / best / 1e9, unit="GB/s", cores=O.threads(), kind="oracle",
                   sample="layer 0 of the stack (7 linears, %.0f M weights) at M=1, oracle fp6o_linear, best of 3; "
                          "oracle quantization of the sample not timed" % (wsample / 1e6))

    # HBM bytes per step from the committed counter summary (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs)
    traffic = {}
    try:
        for line in open(os.path.join(ROOT, "profiles", "bench_cfg5_hbm_traffic.txt")):
            if line.startswith("TRAFFIC_BYTES_PER_STEP_M"):
                k, v = line.strip().split("=")
                traffic[int(k.rsplit("M", 1)[1])] = int(v) * layers // 48
    except OSError:
        pass

    lead = res[legs[0]]
    out = {
        "metric": "fp6_linear achieved HBM GB/s (M=1) and TFLOP/s (M=512) vs roofline, 1 MI355X",
        "value": lead["gbs"] if legs[0] <= 118 else lead["tflops"],
        "unit": "GB/s" if legs[0] <= 118 else "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": lead["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": "%s: %d layers x 7 fp6_linear (q,k,v,o,gate,up,down; hidden 8192, MLP 22016, GQA kv 1024), "
                               "M=%d, %.2f G weights per step" % (WORKLOAD, layers, legs[0], weights_per_pass / 1e9),
                   "launches_per_step": launches, "build_seconds": round(build_s, 1)},
        "roofline": ({"bound": "hbm", "achieved": lead["gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                      "frac": lead["gbs"] / HBM_PEAK_GBS, "traffic": traffic.get(legs[0]),
                      "kernel": "decode_kernel (M<=16), all %d launches of a step" % launches}
                     if legs[0] <= 118 else
                     {"bound": "mfma", "achieved": lead["tflops"], "peak": MFMA_FP16_PEAK_TFLOPS, "unit": "TFLOP/s",
                      "frac": lead["tflops"] / MFMA_FP16_PEAK_TFLOPS, "traffic": traffic.get(legs[0]),
                      "kernel": "gemm_kernel, all %d launches of a step" % launches}),
        "cpu_baseline": cpu,
    }
    if 512 in res and legs[0] != 512:
        r = res[512]
        out["m512"] = {"value": r["tflops"], "unit": "TFLOP/s", "ms_per_step": r["ms_per_step"],
                       "roofline": {"bound": "mfma", "achieved": r["tflops"], "peak": MFMA_FP16_PEAK_TFLOPS,
                                    "unit": "TFLOP/s", "frac": r["tflops"] / MFMA_FP16_PEAK_TFLOPS, "traffic": traffic.get(512),
                                    "kernel": "gemm_kernel (block_m 128), all %d launches of a step" % launches}}
    out["per_shape"] = per_shape
    if ceilings is not None:
        out["measured_ceilings"] = ceilings
        rd = ceilings["plain_read_per_launch"]["GB/s"]
        mf = ceilings["mfma_only_random_operands"]["TFLOP/s"]
        for rf in [out["roofline"]] + ([out["m512"]["roofline"]] if "m512" in out else []):
            rf["measured_ceiling"] = rd if rf["bound"] == "hbm" else mf
            rf["frac_of_measured_ceiling"] = rf["achieved"] / rf["measured_ceiling"]
    if mha is not None:
        out["mha_variant"] = mha
    if configs is not None:
        out["other_configs"] = configs
    if fused is not None:
        out["fused_projections"] = fused
    if layout2 is not None:
        out["layout2_hardware_convert"] = layout2
    if ablation is not None:
        out["bias_shift_ablation"] = ablation
    if fgq is not None:
        out["fgq_and_fp5_vs_row_wise_fp6"] = fgq
    if fp16 is not None:
        out["fp16_dense_baseline"] = {"kind": "torch.matmul (hipBLASLt) on the dequantized fp16 weights, same stack",
                                      "ms_per_step": {m: v["ms_per_step"] for m, v in fp16.items()}}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
