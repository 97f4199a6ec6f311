#!/usr/bin/env python3
"""Benchmark of the W6A16 fp6_linear hot path on one MI355X.

Workload (configuration 5 of the benchmark definition): a 34B-class decoder stack - 48 layers, hidden 8192, MLP
22016, grouped-query attention (k/v projections 1024 x 8192) - with every linear layer
(q, k, v, o, gate, up, down) run as fp6_linear on its own packed FP6 weight.  One "step"
is one pass over all 336 linears (24.9 GB of packed weight, so the pass is cold in HBM
by construction).  Two legs are timed: M=1 (decode, HBM-bound: GB/s counting 0.75 byte
per weight) and M=512 (prefill, MFMA-bound: TFLOP/s counting 2*M*N*K).  `value` is the
M=1 leg with seven fp6_linear calls (seven launches) per layer on one stream; the M=512 leg and the same
stack run through fp6_linear_group (q,k,v in one call, gate,up in one call: four calls per layer) are
reported inside `roofline` and `config` of the same JSON line.

Inputs are seeded synthetic tensors (paper_2312_08583_amd/inputs.py), resident in HBM
before the timed region.  A pass is captured once into a HIP graph and replayed, so the
timed region holds the kernels and nothing else; every leg replays its graph for at least half a
second before its timed steps, because the shader clock takes that long to settle under a new load.
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
WARM_SECONDS = 0.5
GROUPS = (("q", "k", "v"), ("o",), ("gate", "up"), ("down",))


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--layers", type=int, default=0, help="layers of the stack (0 = all 48)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-fp16-baseline", action="store_true")
    ap.add_argument("--legs", default="1,512", help="comma-separated M values to time")
    ap.add_argument("--no-grouped", action="store_true",
                    help="skip the leg that runs q,k,v and gate,up through fp6_linear_group (4 calls per layer)")
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
    ap.add_argument("--no-plan-check", action="store_true",
                    help="skip the leg that times the automatic plan against a small sweep of forced plans")
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
    B = P.binding
    cfg = inputs.WORKLOADS[WORKLOAD]
    shapes = cfg["shapes"]
    names = [n for (n, _, _) in shapes]
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

    def activations(M):
        return {K: inputs.activation(M, K, seed=inputs.workload_seed(WORKLOAD, 9000 + M + K), device=dev)
                for K in sorted({K for (_, _, K) in shapes})}

    def time_passes(one_pass, steps, warm_s=WARM_SECONDS, warmup=0):
        """ms per pass: eager pass (module load, workspace touch), capture, at least warm_s seconds (and `warmup`
        replays) of the same work, then exactly `steps` timed replays between two events on the launch stream."""
        one_pass()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            one_pass()
        t0, n = time.time(), 0
        while time.time() - t0 < warm_s or n < warmup:
            g.replay()
            torch.cuda.synchronize()
            n += 1
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / steps

    def rates(M, ms, weights=None):
        w = weights_per_pass if weights is None else weights
        return dict(ms_per_step=ms, gbs=0.75 * w / (ms * 1e-3) / 1e9, tflops=2.0 * M * w / (ms * 1e-3) / 1e12)

    def leg_summary(M, r):
        if M <= 118:
            return {"ms_per_step": r["ms_per_step"], "value": r["gbs"], "unit": "GB/s", "frac": r["gbs"] / HBM_PEAK_GBS}
        return {"ms_per_step": r["ms_per_step"], "value": r["tflops"], "unit": "TFLOP/s",
                "frac": r["tflops"] / MFMA_FP16_PEAK_TFLOPS}

    if args.copy_probe:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)      # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    legs = [int(m) for m in args.legs.split(",")]

    # ---- the timed legs: seven fp6_linear calls per layer, one stream, one workspace
    res = {}
    for M in legs:
        xs = activations(M)
        ys = [torch.empty((M, N), dtype=torch.float16, device=dev) for (_, N, _) in shapes]
        ws = P.new_workspace(max(max(P.fp6_linear_workspace_bytes(M, N, K) for (_, N, K) in shapes), 16), dev)

        def one_pass():
            for mats in stack:
                for si, (N, K, hi, lo, sc) in enumerate(mats):
                    P.fp6_linear(xs[K], hi, lo, sc, N, K, out=ys[si], workspace=ws)
        res[M] = rates(M, time_passes(one_pass, args.steps, warmup=args.warmup))

    # ---- the same stack through fp6_linear_group: q,k,v in one call, gate,up in one call (4 calls per layer;
    # one launch each at M <= 16).  Same weights, same planes; results equal up to fp32 summation order.
    grouped = None
    if not args.no_grouped:
        gidx = [[names.index(n) for n in g] for g in GROUPS]
        grouped = {"calls_per_step": layers * len(gidx),
                   "what": "q,k,v and gate,up each through one fp6_linear_group call (separate planes and scales, "
                           "one launch per call at M <= 16; at larger M the call launches its layers one after another)"}
        for M in legs:
            xs = activations(M)
            ys = [torch.empty((M, N), dtype=torch.float16, device=dev) for (_, N, _) in shapes]
            need = max(P.fp6_linear_group_workspace_bytes(M, [(shapes[i][1], shapes[i][2]) for i in g]) for g in gidx)
            ws = P.new_workspace(max(need, 16), dev)

            def group_pass():
                for mats in stack:
                    for g in gidx:
                        P.fp6_linear_group([(xs[mats[i][1]], mats[i][2], mats[i][3], mats[i][4], mats[i][0], mats[i][1])
                                            for i in g], outs=[ys[i] for i in g], workspace=ws)
            grouped["M%d" % M] = leg_summary(M, rates(M, time_passes(group_pass, args.steps, warmup=args.warmup)))

    # ---- measured ceilings: what kernels that do nothing else sustain on this machine, for reading the two
    # roofline fractions against (the nominal peaks stay the denominators of `frac`).
    def read_probe_us(nbytes, copies_bytes=1.2e9):
        """us per launch of the plain read kernel over nbytes, cold: a pool of distinct buffers read in turn."""
        nbytes = max(16, int(nbytes) // 16 * 16)
        copies = max(2, min(64, int(copies_bytes / nbytes) + 1))
        pool = [torch.empty(nbytes, dtype=torch.uint8, device=dev).random_(0, 256) for _ in range(copies)]
        best = None
        for wgs in (1024, 4096):
            sink = torch.zeros(wgs * 4, dtype=torch.int32, device=dev)

            def read_pass():
                for b in pool:
                    P.fp6_probe_read(b, wgs, sink)
            us = time_passes(read_pass, 5, warm_s=0.15) * 1e3 / copies
            best = us if best is None else min(best, us)
        return best

    ceilings = None
    if not args.no_ceilings:
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
            ms = time_passes(read_pass, 10, warm_s=0.3)
            gbs = sum(h.numel() for h in gate) / (ms * 1e-3) / 1e9
            if best is None or gbs > best[0]:
                best = (gbs, wgs, ms * 1e3 / len(gate))
        ceilings["plain_read_per_launch"] = {"GB/s": round(best[0], 1), "workgroups": best[1], "us_per_launch": round(best[2], 2),
                                             "what": "read-only kernel, one launch per 90 MB buffer, cold, graph replay"}
        big = torch.empty(1 << 31, dtype=torch.uint8, device=dev)
        sink = torch.zeros(4096 * 4, dtype=torch.int32, device=dev)
        big.random_(0, 256)
        ms = time_passes(lambda: P.fp6_probe_read(big, 4096, sink), 10, warm_s=0.3)
        ceilings["plain_read_2GiB"] = {"GB/s": round(big.numel() / (ms * 1e-3) / 1e9, 1),
                                       "what": "read-only kernel, one launch over 2 GiB"}
        del big
        tiny = torch.zeros(4096, dtype=torch.uint8, device=dev)
        sink = torch.zeros(256 * 4, dtype=torch.int32, device=dev)

        def empty_pass():
            for _ in range(64):
                P.fp6_probe_read(tiny, 256, sink)
        ceilings["launch_floor_us"] = round(time_passes(empty_pass, 10, warm_s=0.2) * 1e3 / 64, 2)
        # (b) MFMA-only kernel (8 wavefronts per SIMD), with pseudo-random and with zero operands: the
        # clock the chip holds depends on the operand data
        wgs, iters, reps = 2048, 2000, 20
        sink = torch.zeros(wgs * 256, dtype=torch.float32, device=dev)
        for name, rnd in (("random_operands", True), ("zero_operands", False)):
            flop = P.fp6_probe_mfma(wgs, iters, rnd, sink) * reps

            def mfma_pass():
                for _ in range(reps):
                    P.fp6_probe_mfma(wgs, iters, rnd, sink)
            ms = time_passes(mfma_pass, 10, warm_s=0.5)
            ceilings["mfma_only_" + name] = {"TFLOP/s": round(flop / (ms * 1e-3) / 1e12, 1), "us_per_launch": round(ms * 1e3 / reps, 1),
                                             "what": "v_mfma_f32_16x16x32_f16 on register operands, %d workgroups x 4 wavefronts, "
                                                     "sustained" % wgs}
        # (c) the same MFMAs with two integer vector instructions behind each, the mix of the tiled kernel's loop (the
        # unpack issues through the port the MFMAs issue through), at that kernel's two wavefronts per SIMD and at
        # full occupancy
        for name, wgs_mix, iters_mix in (("two_waves_per_simd", 512, 8000), ("full_occupancy", 2048, 2000)):
            sink = torch.zeros(wgs_mix * 256, dtype=torch.float32, device=dev)
            flop = P.fp6_probe_mfma(wgs_mix, iters_mix, True, sink, valu_mix=True) * reps

            def mix_pass():
                for _ in range(reps):
                    P.fp6_probe_mfma(wgs_mix, iters_mix, True, sink, valu_mix=True)
            ms = time_passes(mix_pass, 10, warm_s=0.5)
            ceilings["mfma_with_two_valu_each_" + name] = {
                "TFLOP/s": round(flop / (ms * 1e-3) / 1e12, 1),
                "what": "the MFMA-only kernel, random operands, with a v_perm_b32 and a v_xor_b32 behind every MFMA, "
                        "%d workgroups x 4 wavefronts" % wgs_mix}

    def ceiling_us(M, N, K):
        """Time a launch cannot beat on this machine: the plain read kernel over the same packed bytes (which includes
        its own launch), or the MFMA-only rate over the same flop, whichever is longer."""
        if ceilings is None:
            return None
        rd = read_probe_us(0.75 * N * K)
        mf = 2.0 * M * N * K / (ceilings["mfma_only_random_operands"]["TFLOP/s"] * 1e12) * 1e6 + ceilings["launch_floor_us"]
        return max(rd, mf)

    # ---- per-shape breakdown: the same launches grouped by shape (each shape over its `layers` distinct weights,
    # so every launch is cold), to show which kernel instance sits where against its roofline
    per_shape = {}
    for M in ([] if args.no_per_shape else legs):
        xs = activations(M)
        ws = P.new_workspace(max(max(P.fp6_linear_workspace_bytes(M, N, K) for (_, N, K) in shapes), 16), dev)
        rows = []
        for si, (name, N, K) in enumerate(shapes):
            if si and (N, K) == (shapes[si - 1][1], shapes[si - 1][2]):
                rows.append(dict(rows[-1], shape="%s %dx%d" % (name, N, K)))      # same kernel instance, same plan
                continue
            y = torch.empty((M, N), dtype=torch.float16, device=dev)

            def sweep():
                for mats in stack:
                    _, _, hi, lo, sc = mats[si]
                    P.fp6_linear(xs[K], hi, lo, sc, N, K, out=y, workspace=ws)
            us = time_passes(sweep, max(3, args.steps // 4), warm_s=0.25) * 1e3 / len(stack)
            row = {"shape": "%s %dx%d" % (name, N, K), "us": round(us, 2), "plan": P.plan_text(P.fp6_linear_plan(M, N, K))}
            if M <= 118:
                row["GB/s"] = round(0.75 * N * K / us / 1e3, 1)
                row["frac"] = round(0.75 * N * K / us / 1e3 / HBM_PEAK_GBS, 3)
            else:
                row["TFLOP/s"] = round(2.0 * M * N * K / us / 1e6, 1)
                row["frac"] = round(2.0 * M * N * K / us / 1e6 / MFMA_FP16_PEAK_TFLOPS, 3)
            c = ceiling_us(M, N, K)
            if c is not None:
                row["measured_ceiling_us"] = round(c, 2)
                row["frac_of_measured_ceiling"] = round(c / us, 3)
            rows.append(row)
        per_shape["M%d" % M] = rows

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
        wpp = weights_per_pass + sum(N * K - shapes[1][1] * shapes[1][2] for p_ in kv for (N, K, *_) in p_)
        mha = {"what": "k,v projections 8192x8192 (no grouped-query attention), %.2f G weights per step, 7 calls per layer"
                       % (wpp / 1e9)}
        for M in legs:
            xs = activations(M)
            ys = [torch.empty((M, shapes[0][1] if si in (1, 2) else N), dtype=torch.float16, device=dev)
                  for si, (_, N, _) in enumerate(shapes)]
            need = max(P.fp6_linear_workspace_bytes(M, N, K) for (_, N, K) in shapes)
            ws = P.new_workspace(max(need, 16), dev)

            def mha_pass():
                for mats, pair in zip(stack, kv):
                    for si, (N, K, hi, lo, sc) in enumerate(mats):
                        if si in (1, 2):
                            N, K, hi, lo, sc = pair[si - 1]
                        P.fp6_linear(xs[K], hi, lo, sc, N, K, out=ys[si], workspace=ws)
            mha["M%d" % M] = leg_summary(M, rates(M, time_passes(mha_pass, max(3, args.steps // 2)), wpp))
        del kv

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
            xs = activations(M)
            ys = [torch.empty((M, N), dtype=torch.float16, device=dev) for (_, N, _) in shapes]
            ws = P.new_workspace(max(max(P.fp6_linear_v2_workspace_bytes(M, N, K) for (_, N, K) in shapes), 16), dev)

            def pass2():
                for mats in stack2:
                    for si, (N, K, hi, lo, sc) in enumerate(mats):
                        P.fp6_linear_v2(xs[K], hi, lo, sc, N, K, out=ys[si], workspace=ws)
            layout2["M%d" % M] = leg_summary(M, rates(M, time_passes(pass2, max(3, args.steps // 2))))
            # the same planes against bf16 activations (bf16 form of the conversion, bf16 MFMA, bf16 output)
            xb = {K: inputs.activation_bf16(M, K, seed=inputs.workload_seed(WORKLOAD, 9000 + M + K), device=dev)
                  for K in sorted({K for (_, _, K) in shapes})}
            yb = [torch.empty((M, N), dtype=torch.bfloat16, device=dev) for (_, N, _) in shapes]

            def pass2b():
                for mats in stack2:
                    for si, (N, K, hi, lo, sc) in enumerate(mats):
                        P.fp6_linear_v2_bf16(xb[K], hi, lo, sc, N, K, out=yb[si], workspace=ws)
            layout2["M%d" % M]["bf16_activations_ms_per_step"] = time_passes(pass2b, max(3, args.steps // 2))
        del stack2

    # ---- fp16 dense GEMM on the same GPU, same stack (context, not the target)
    fp16 = None
    if not args.no_fp16_baseline:
        dense = [[P.fp6_dequantize(hi, lo, sc, N, K) for (N, K, hi, lo, sc) in mats] for mats in stack]
        fp16 = {}
        for M in legs:
            xs = activations(M)

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

    def cold_pool(hi, lo, sc, N, K, extra=()):
        copies = max(2, min(64, int(1.0e9 / (0.75 * N * K)) + 1))
        return [(hi.clone(), lo.clone(), sc.clone()) + tuple(extra) for _ in range(copies)]

    # ---- bias-shift ablation (Section 5.3: the same kernel without bias shift) on the six
    # feed-forward shapes of the paper's kernel table (Appendix B), batch 8, cold weights
    ablation = None
    if not args.no_ablation:
        modes = {"bias_shift": 0, "integer_rebias": B.FP6_HINT_DEQUANT(1), "fp16_multiply": B.FP6_HINT_DEQUANT(2)}
        tcfg = inputs.WORKLOADS["paper_table_b1"]
        M = tcfg["Ms"][0]
        ablation = {"M": M, "unit": "us", "shapes": {}}
        for si, (name, N, K) in enumerate(tcfg["shapes"]):
            W = inputs.workload_weight("paper_table_b1", si, device=dev)
            hi, lo, sc = P.fp6_quantize_pack(W)
            del W
            pool = cold_pool(hi, lo, sc, N, K)
            X = inputs.activation(M, K, seed=inputs.workload_seed("paper_table_b1", 500 + si), device=dev)
            Y = torch.empty((M, N), dtype=torch.float16, device=dev)
            row = {}
            for mode, hint in modes.items():
                ws = P.new_workspace(max(P.fp6_linear_variant_workspace_bytes(M, N, K, hint, 0), 16), dev)

                def sweep():
                    for (h, l, s_) in pool:
                        P.fp6_linear_variant(X, h, l, s_, N, K, hint, 0, out=Y, workspace=ws)
                row[mode] = round(time_passes(sweep, 5, warm_s=0.1) * 1e3 / len(pool), 2)
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
            row = {}
            for mode in ("row_wise", "fgq", "fp5"):
                hi, lo, sc = (P.fp6_quantize_pack(W) if mode == "row_wise" else
                              P.fp6_quantize_pack_fgq(W, block) if mode == "fgq" else P.fp5_quantize_pack(W))
                pool = cold_pool(hi, lo, sc, N, K)
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
                row[mode] = round(time_passes(sweep, 5, warm_s=0.1) * 1e3 / len(pool), 2)
                del pool
            fgq["shapes"]["%s %dx%d" % (name, N, K)] = row
            del W
        r = [v["fgq"] / v["row_wise"] for v in fgq["shapes"].values()]
        fgq["mean_slowdown_fgq"] = round(sum(r) / len(r), 3)
        r = [v["fp5"] / v["row_wise"] for v in fgq["shapes"].values()]
        fgq["mean_time_ratio_fp5"] = round(sum(r) / len(r), 3)       # bytes ratio: 0.625 / 0.75 = 0.833

    # ---- the other benchmark configurations (1-4): every shape at every M of the configuration, each timed
    # over a pool of distinct packed copies of at least 1 GB in turn, so every launch reads cold weights; beside
    # each row the plan that ran and what the plain read kernel / the MFMA-only rate allow for the same work
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
                pool = cold_pool(hi, lo, sc, N, K)
                rd = read_probe_us(0.75 * N * K) if ceilings is not None else None
                for M in c["Ms"]:
                    X = inputs.activation(M, K, seed=inputs.workload_seed(wl, 500 + si) + M, device=dev)
                    Y = torch.empty((M, N), dtype=torch.float16, device=dev)
                    ws = P.new_workspace(max(P.fp6_linear_workspace_bytes(M, N, K), 16), dev)

                    def sweep():
                        for (h, l, s_) in pool:
                            P.fp6_linear(X, h, l, s_, N, K, out=Y, workspace=ws)
                    us = time_passes(sweep, 5, warm_s=0.1) * 1e3 / len(pool)
                    t_hbm = 0.75 * N * K / (HBM_PEAK_GBS * 1e9) * 1e6
                    t_mfma = 2.0 * M * N * K / (MFMA_FP16_PEAK_TFLOPS * 1e12) * 1e6
                    row = {"shape": "%s %dx%d" % (name, N, K), "M": M, "us": round(us, 2),
                           "GB/s": round(0.75 * N * K / us / 1e3, 1), "TFLOP/s": round(2.0 * M * N * K / us / 1e6, 1),
                           "bound": "hbm" if t_hbm >= t_mfma else "mfma",
                           "frac": round(max(t_hbm, t_mfma) / us, 3), "plan": P.plan_text(P.fp6_linear_plan(M, N, K))}
                    if rd is not None:
                        mf = (2.0 * M * N * K / (ceilings["mfma_only_random_operands"]["TFLOP/s"] * 1e12) * 1e6 +
                              ceilings["launch_floor_us"])
                        row["measured_ceiling_us"] = round(max(rd, mf), 2)
                        row["frac_of_measured_ceiling"] = round(max(rd, mf) / us, 3)
                    rows.append(row)
                del pool
            configs[wl] = rows

    # ---- planner check: the automatic plan against a small sweep of forced plans on the config-5 shapes
    # (and the config-3 shapes at M = 128), cold weights; `gap` = time of the automatic plan / best forced time
    plan_check = None
    if not args.no_plan_check:
        D_, G_ = B.FP6_VARIANT_DECODE, B.FP6_VARIANT_GEMM
        decode_plans = [("decode full s%d" % s, D_ | B.FP6_HINT_HALF(2), s) for s in (1, 2, 4, 8)] + \
                       [("decode half s%d" % s, D_ | B.FP6_HINT_HALF(1), s) for s in (1, 2, 8)]
        gemm_plans = [("gemm %dx%d s%d" % (bm, 64 * w, s), G_ | B.FP6_HINT_BLOCK_M(bm) | B.FP6_HINT_WIDTH(w), s)
                      for bm in (64, 128) for w in (8, 4) for s in (1, 2, 4)] + \
                     [("gemm 128x256 k2 s%d" % s, G_ | B.FP6_HINT_BLOCK_M(128) | B.FP6_HINT_WIDTH(4) | B.FP6_HINT_KWAYS(2), s)
                      for s in (1, 2)]
        cases = [(WORKLOAD, si, M) for M in legs for si in (0, 1, 4, 6)] + [("cfg3_llama13b", si, 128) for si in range(3)]
        plan_check = {"unit": "us", "rows": []}
        for wl, si, M in cases:
            name, N, K = inputs.WORKLOADS[wl]["shapes"][si]
            W = inputs.workload_weight(wl, si, device=dev)
            hi, lo, sc = P.fp6_quantize_pack(W)
            del W
            pool = cold_pool(hi, lo, sc, N, K)
            X = inputs.activation(M, K, seed=inputs.workload_seed(wl, 700 + si) + M, device=dev)
            Y = torch.empty((M, N), dtype=torch.float16, device=dev)

            def timed(variant, split):
                try:
                    need = P.fp6_linear_plan(M, N, K, variant=variant, split_k=split)["workspace_bytes"]
                except P.Fp6Error:
                    return None
                ws = P.new_workspace(max(need, 16), dev)

                def sweep():
                    for (h, l, s_) in pool:
                        P.fp6_linear_variant(X, h, l, s_, N, K, variant, split, out=Y, workspace=ws)
                return time_passes(sweep, 4, warm_s=0.08) * 1e3 / len(pool)
            auto = timed(B.FP6_VARIANT_AUTO, 0)
            forced = [(t, label) for (label, v, s) in (decode_plans if M <= 16 else gemm_plans)
                      for t in [timed(v, s)] if t is not None]
            best_t, best_label = min(forced)
            plan_check["rows"].append({"shape": "%s %s %dx%d" % (wl.split("_")[0], name, N, K), "M": M,
                                       "auto_plan": P.plan_text(P.fp6_linear_plan(M, N, K)), "auto": round(auto, 2),
                                       "best_forced": round(best_t, 2), "best_forced_plan": best_label,
                                       "gap": round(auto / best_t, 3)})
            del pool
        gaps = [r["gap"] for r in plan_check["rows"]]
        plan_check["mean_gap"] = round(sum(gaps) / len(gaps), 3)
        plan_check["worst_gap"] = max(gaps)

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

    # HBM bytes per step as an EARLIER profiler run of this benchmark counted them (rocprofv3 --pmc FETCH_SIZE /
    # WRITE_SIZE; the summary names its command and library build).  Not measured in this run, so not under `traffic`.
    profiled = {}
    try:
        for line in open(os.path.join(ROOT, "profiles", "bench_cfg5_hbm_traffic.txt")):
            if line.startswith("TRAFFIC_BYTES_PER_STEP_M"):
                k, v = line.strip().split("=")
                profiled[int(k.rsplit("M", 1)[1])] = int(v) * layers // 48
    except OSError:
        pass

    def traffic_note(M):
        if M not in profiled:
            return None
        return {"bytes_per_step": profiled[M], "source": "profiles/bench_cfg5_hbm_traffic.txt (a committed rocprofv3 --pmc "
                                                         "summary of an earlier run of this command, not this run)"}

    kernel_names = {
        1: "decode_half_kernel<4,4> (q, k, v, o, down: 5 of the 7 launches per layer) and decode_kernel<4,4,...> "
           "(gate, up); %d launches per step" % launches,
        512: "gemm_kernel: 128x512 blocks (gate, up), 128x256 blocks with two K-ways per workgroup (q, o, down), "
             "32x256 blocks (k, v); %d launches per step" % launches,
    }

    def roofline_of(M, r):
        rf = ({"bound": "hbm", "achieved": r["gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": r["gbs"] / HBM_PEAK_GBS}
              if M <= 118 else
              {"bound": "mfma", "achieved": r["tflops"], "peak": MFMA_FP16_PEAK_TFLOPS, "unit": "TFLOP/s",
               "frac": r["tflops"] / MFMA_FP16_PEAK_TFLOPS})
        rf["traffic"] = None
        rf["traffic_from_profile"] = traffic_note(M)
        rf["ms_per_step"] = r["ms_per_step"]
        rf["kernel"] = kernel_names.get(M, "all %d launches of a step" % launches)
        if ceilings is not None:
            rf["measured_ceiling"] = (ceilings["plain_read_per_launch"]["GB/s"] if M <= 118 else
                                      ceilings["mfma_only_random_operands"]["TFLOP/s"])
            rf["frac_of_measured_ceiling"] = rf["achieved"] / rf["measured_ceiling"]
            if M > 118:
                rf["mfma_with_unpack_mix_ceiling"] = ceilings["mfma_with_two_valu_each_two_waves_per_simd"]["TFLOP/s"]
                rf["frac_of_mfma_with_unpack_mix_ceiling"] = rf["achieved"] / rf["mfma_with_unpack_mix_ceiling"]
        if grouped is not None and ("M%d" % M) in grouped:
            rf["grouped_calls"] = dict(grouped["M%d" % M], calls_per_step=grouped["calls_per_step"])
        return rf

    lead = res[legs[0]]
    config = {"workload": "%s: %d layers x 7 fp6_linear (q,k,v,o,gate,up,down; hidden 8192, MLP 22016, GQA kv 1024), "
                          "M=%d, %.2f G weights per step" % (WORKLOAD, layers, legs[0], weights_per_pass / 1e9),
              "launches_per_step": launches, "build_seconds": round(build_s, 1), "warm_seconds_per_leg": WARM_SECONDS}
    out = {
        "metric": "fp6_linear achieved HBM GB/s (M=1) and TFLOP/s (M=512) vs roofline, 1 MI355X",
        "value": lead["gbs"] if legs[0] <= 118 else lead["tflops"],
        "unit": "GB/s" if legs[0] <= 118 else "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": lead["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": config,
        "roofline": roofline_of(legs[0], lead),
        "cpu_baseline": cpu,
    }
    for M in legs[1:]:
        # the other half of the metric rides inside the blocks the record keeps
        out["roofline"]["m%d" % M] = roofline_of(M, res[M])
        config["m%d_ms_per_step" % M] = res[M]["ms_per_step"]
        config["m%d_%s" % (M, "GBps" if M <= 118 else "TFLOPs")] = res[M]["gbs"] if M <= 118 else res[M]["tflops"]
    if grouped is not None:
        config["grouped_ms_per_step"] = {k: v["ms_per_step"] for k, v in grouped.items() if k.startswith("M")}
    out["per_shape"] = per_shape
    if ceilings is not None:
        out["measured_ceilings"] = ceilings
    if grouped is not None:
        out["grouped_calls"] = grouped
    if plan_check is not None:
        out["plan_check"] = plan_check
    if mha is not None:
        out["mha_variant"] = mha
    if configs is not None:
        out["other_configs"] = configs
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
