#!/usr/bin/env python3
"""Benchmark: sentences certified per second on the 2-layer configuration (c2), one MI355X.

A step is one pass of the whole hot path over one synthetic batch: tv_certify (10 bisection probes,
each a full bound-propagation sweep) on 32 sentences of 32 tokens, once for each of the l_1, l_2 and
l_inf balls = 96 sentence certifications.  Model weights, tokens and the workspace are resident in HBM
before the timed region.  Prints ONE JSON line with the throughput, the roofline position of the
dominant kernel class (HIP-event timed inside the library during the timed steps) and the float64
CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0       # MI355X HBM3E
MFMA_FP32_PEAK_TF = 157.3   # MI355X dense fp32 matrix
BF16_SPLIT_PEAK_TF = 2500.0 / 6.0   # dense bf16 peak over the six bf16 products that make one fp32 product
# HBM bytes per launch of a kernel class from `rocprofv3 --pmc FETCH_SIZE` / `WRITE_SIZE` on `bench.py --probe`,
# scaled by the counters' readings for the 2^30-byte copy of the same run (2048 and 1024 bytes per unit) and
# averaged over the launches of one certify call; counters cannot be read inside this process, so the figure is
# a constant of the workload and is reported only for the workload it was collected on
PMC_TRAFFIC = {"c2": {"affine_gemm": 407.5e6, "layernorm": 246.8e6, "activation": 492.4e6, "softmax": 247.6e6}}
MFMA_KINDS = ("affine_gemm", "qk_gemm_x", "qk_gemm_y", "pv_gemm_x", "pv_gemm_y", "head_gemm")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="c2")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the copy / fill / MFMA issue-rate probes")
    ap.add_argument("--no-kernel-timing", action="store_true",
                    help="leave the per-launch HIP events out of the timed region")
    ap.add_argument("--op-sweep", action="store_true",
                    help="time single operators over sentence length and hidden size instead of the certify benchmark")
    ap.add_argument("--tile-search", action="store_true",
                    help="rule-pruned tile search of the affine kernel over the layer shapes of c1..c4 (one JSON line each)")
    ap.add_argument("--probe", action="store_true",
                    help="counter probe: a 1 GiB device copy (known traffic) followed by one verify sweep, no timing")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (every box has one); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2209_12708_amd import binding as tv
    from tv_synth import CONFIGS, make_model, make_positions, make_tokens

    if args.tile_search:
        # Layer shapes (K -> N) of every affine map of a configuration: W_q|W_k|W_v stacked, W_o, W_1, W_2.  c4 is
        # searched on 8 of its 64 sentences (the tiles only see the row count through the grid size).
        from paper_2209_12708_amd import tile_search
        for name, sentences in (("c1", None), ("c2", None), ("c3", None), ("c4", 8)):
            c = CONFIGS[name]
            Bn = sentences or c.batch
            D, F = c.enc.hidden, c.enc.ffn
            for K, N in ((D, 3 * D), (D, D), (D, F), (F, D)):
                rec = tile_search.search(Bn, c.n_perturbed, D, c.seq_len, K, N)
                rec["workload"] = name
                rec["sentences"] = Bn
                print(json.dumps({"tile_search": rec}), flush=True)
                torch.cuda.empty_cache()
        return

    w = CONFIGS[args.workload]
    weights = make_model(w)
    tokens, positions = make_tokens(w), make_positions(w)
    dev = torch.device("cuda:0")
    model = tv.Model(weights, dev)
    tok_d, pos_d = torch.as_tensor(tokens, device=dev), torch.as_tensor(positions, device=dev)
    ws = model.workspace(w.batch, w.seq_len, w.n_perturbed)
    full, _ = model.workspace_query(w.batch, w.seq_len, w.n_perturbed)

    if args.op_sweep:
        # Single operators over sentence length (hidden 128) and hidden size (length 16), after the paper's
        # operator-level figures (Sec. 6.2: affine, ReLU, tanh, dot product); synthetic states, 32 sentences, P = 1.
        def timed(fn, reps=20):
            for _ in range(3):
                fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) * 1e3 / reps

        def state(Bn, C, L, n):
            S = torch.randn(Bn, C, L, n, device=dev) * 0.05
            R = torch.rand(Bn, C, L, n, device=dev) * 0.01
            return S, R

        Bn, p = 32, 2
        eps = torch.full((Bn,), 1e-3, device=dev)
        points = [(L, 128) for L in (4, 8, 16, 32, 64, 128)] + [(16, D) for D in (64, 192, 256, 384, 512, 640)]
        for L, D in points:
            C = D + 1
            x = state(Bn, C, L, D)
            W = torch.randn(D, D, device=dev) * 0.05
            b = torch.randn(D, device=dev)
            byts = 2 * 4 * Bn * C * L * D
            rec = {"op_sweep": {"length": L, "hidden": D, "sentences": Bn, "state_MB": round(byts / 1e6, 2)}}
            W3, Wa3 = tv.op_split3(W), tv.op_split3(W, True)
            Sy, Ry = torch.empty_like(x[0]), torch.empty_like(x[1])
            L_ = tv.lib()
            us = timed(lambda: tv._check(L_.tv_op_affine_split(tv._ptr(x[0]), tv._ptr(x[1]), Bn, 1, D, L, D, D, tv._ptr(W3),
                                                                 tv._ptr(Wa3), tv._ptr(b), None, None, tv._ptr(Sy),
                                                                 tv._ptr(Ry), tv._stream())))
            rec["affine_us"] = round(us, 1)
            rec["affine_TFLOPs"] = round(2 * 2.0 * Bn * C * L * D * D / us / 1e6, 1)
            rec["affine_GBps"] = round(2 * byts / us / 1e3, 0)
            for act, nm in ((0, "relu"), (1, "tanh"), (3, "leaky_relu"), (4, "silu")):
                us = timed(lambda: tv.op_activation(act, x[0], x[1], 1, D, 1, p, eps, act_alpha=0.01))
                rec[nm + "_us"] = round(us, 1)
                rec[nm + "_GBps"] = round(2 * byts / us / 1e3, 0)
            if D % 4 == 0 and (D // 4) % 4 == 0:
                q, k, v = x, state(Bn, C, L, D), state(Bn, C, L, D)
                us = timed(lambda: tv.op_attention(q, k, v, 4, 1, p, eps, stop_after=1), reps=10)
                rec["dot_product_us"] = round(us, 1)      # concretization of q, k, v + preparation + the q k^T bound
                del q, k, v
            print(json.dumps(rec), flush=True)
            del x, Sy, Ry
            torch.cuda.empty_cache()
        return

    if args.probe:
        # for `rocprofv3 --pmc FETCH_SIZE` / `WRITE_SIZE`: the copy kernel moves exactly 2^30 bytes each way
        # and calibrates the counter unit; the sweep's dispatches follow it
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        eps = torch.full((w.batch,), 1e-3, dtype=torch.float32, device=dev)
        model.verify(tok_d, pos_d, w.p_norms[-1], eps, workspace=ws)
        torch.cuda.synchronize()
        print(json.dumps({"probe": "copy of 2^30 bytes, then one verify sweep", "workload": args.workload}))
        return

    def ceilings():
        """Achievable ceilings of this part as it runs (the published peaks are the roofline's denominators):
        a device copy and a fill of 1 GiB, two mixed streams with the read : write ratios of the affine layers
        (1 : 3 like the fused QKV product, 2 : 1 like W_o with its residual; torch's elementwise kernels on
        512 MiB units), and the issue rate of the two matrix-core instructions."""
        n = 1 << 28
        a = torch.empty(n, dtype=torch.float32, device=dev).normal_()
        b = torch.empty_like(a)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

        def timed(fn, reps):
            fn()
            torch.cuda.synchronize()
            e0.record()
            for _ in range(reps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) * 1e-3 / reps

        out = {"copy_GBps": round(2 * 4 * n / timed(lambda: b.copy_(a), 5) / 1e9, 1),
               "fill_GBps": round(4 * n / timed(lambda: b.fill_(1.0), 5) / 1e9, 1)}
        h = n // 2
        b3 = torch.empty(3, h, dtype=torch.float32, device=dev)
        out["read1_write3_GBps"] = round(4 * 4 * h / timed(lambda: b3.copy_(a[:h].expand(3, h)), 5) / 1e9, 1)
        out["read2_write1_GBps"] = round(3 * 4 * h / timed(lambda: torch.add(a[:h], a[h:], out=b[:h]), 5) / 1e9, 1)
        del b3
        buf = torch.empty(2048 * 256, dtype=torch.float32, device=dev)
        for name, bf16, iters in (("mfma_f32_TFLOPs", 0, 4000), ("mfma_bf16_TFLOPs", 1, 8000)):
            fl = [0.0]

            def launch():
                fl[0] = tv.probe_mfma(bf16, 2048, iters, buf)
            t = timed(launch, 3)
            out[name] = round(fl[0] / t / 1e12, 1)
        del a, b, buf
        return out

    def step():
        out = None
        for p in w.p_norms:
            out = model.certify(tok_d, pos_d, p, w.eps_lo, w.eps_hi, w.steps, workspace=ws)
        return out

    def breakdown(prof, nsteps):
        total_ms = sum(v["ms"] for v in prof.values())
        out = {}
        for name, v in sorted(prof.items(), key=lambda kv: -kv[1]["ms"]):
            out[name] = {"share": round(v["ms"] / total_ms, 4), "launches_per_step": v["launches"] // nsteps,
                         "avg_us": round(v["ms"] * 1e3 / v["launches"], 2),
                         "GBps": round(v["bytes"] / (v["ms"] * 1e-3) / 1e9, 1) if v["ms"] else 0.0,
                         "TFLOPs": round(v["flops"] / (v["ms"] * 1e-3) / 1e12, 2) if v["ms"] else 0.0}
        return out

    # Two HIP events per launch cost a few microseconds each (about 8 % of a step when every class is timed), so the
    # class breakdown is taken during the last warm-up step and the timed region times only the dominant class: its
    # launch duration is still measured live over exactly the timed steps.
    timing = not args.no_kernel_timing
    kernels, dom = {}, None
    for i in range(args.warmup):
        last_warm = timing and i == args.warmup - 1
        if last_warm:
            torch.cuda.synchronize()
            tv.profile_select(None)
            tv.profile_reset()
            tv.profile_enable(True)
        step()
        if last_warm:
            torch.cuda.synchronize()
            tv.profile_enable(False)
            prof = tv.profile_read()
            kernels = breakdown(prof, 1)
            dom = max(prof, key=lambda k: prof[k]["ms"])
    torch.cuda.synchronize()
    if timing:
        tv.profile_reset()
        tv.profile_select([dom] if dom else None)
        tv.profile_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        last = step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    tv.profile_enable(False)
    tv.profile_select(None)
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    n_cert = w.batch * len(w.p_norms)
    value = n_cert / (ms_per_step * 1e-3)

    roofline = None
    if timing:
        prof = tv.profile_read()
        if not kernels:                      # no warm-up step: every class was timed in the timed region
            kernels = breakdown(prof, args.steps)
        dom = dom or max(prof, key=lambda k: prof[k]["ms"])
        d = prof[dom]
        # the roof that bounds the class: its arithmetic intensity against the ridge of its own compute roof.
        # The affine layers run on the bf16 matrix cores with six products per fp32 product (three bf16 pieces per
        # operand), so their compute roof is the dense bf16 peak / 6 in fp32-equivalent flops; the dot-product
        # contractions use the fp32 MFMA instructions.
        compute_peak = BF16_SPLIT_PEAK_TF if dom == "affine_gemm" else MFMA_FP32_PEAK_TF
        ai = d["flops"] / max(d["bytes"], 1.0)
        tf = d["flops"] / (d["ms"] * 1e-3) / 1e12
        gbs = d["bytes"] / (d["ms"] * 1e-3) / 1e9
        if dom in MFMA_KINDS and ai > compute_peak * 1e12 / (HBM_PEAK_GBS * 1e9):
            roofline = {"kernel": dom, "bound": "mfma", "achieved": round(tf, 2), "peak": round(compute_peak, 1),
                        "unit": "TFLOP/s", "frac": round(tf / compute_peak, 4), "traffic": None}
        else:
            roofline = {"kernel": dom, "bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS,
                        "unit": "GB/s", "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": None}
        if dom in MFMA_KINDS:
            roofline["arithmetic_intensity_flop_per_byte"] = round(ai, 1)
            roofline["algorithmic_TFLOPs"] = round(tf, 2)
            roofline["compute_roof_TFLOPs"] = round(compute_peak, 1)
        roofline["traffic"] = PMC_TRAFFIC.get(args.workload, {}).get(dom)
        roofline["avg_launch_us"] = round(d["ms"] * 1e3 / d["launches"], 2)
        roofline["launches_timed"] = d["launches"]
        roofline["algorithmic_bytes_per_launch"] = d["bytes"] / d["launches"]
        roofline["algorithmic_flops_per_launch"] = d["flops"] / d["launches"]

    # the ceiling probes run after the timed region: seconds of saturated matrix cores just before it would lower
    # the clocks the timed steps see
    ceil = None if args.no_ceilings else ceilings()

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import verifier as V
        try:
            from threadpoolctl import threadpool_info
            cores = max([i.get("num_threads", 1) for i in threadpool_info()] or [os.cpu_count()])
        except Exception:
            cores = os.cpu_count()
        p = w.p_norms[min(1, len(w.p_norms) - 1)]
        c0 = time.perf_counter()
        n_done = 0
        while n_done < 2 and time.perf_counter() - c0 < 20.0:
            e_ref, _ = V.certify(weights, tokens[n_done], positions[n_done], p, w.eps_lo, w.eps_hi, w.steps)
            n_done += 1
        c1 = time.perf_counter()
        gpu_eps = float(last["eps"][n_done - 1]) if p == w.p_norms[-1] else None
        cpu = {"value": round(n_done / (c1 - c0), 4), "unit": "sentences certified/s", "cores": int(cores),
               "kind": "oracle",
               "sample": f"{n_done} sentence(s) of {args.workload}, p={p}, {w.steps} bisection probes each, float64 numpy"}
        del gpu_eps

    line = {
        "metric": "sentences certified/sec (eps binary search)", "value": round(value, 2),
        "unit": "sentences certified/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload}: {w.enc.n_layers}-layer encoder, hidden {w.enc.hidden}, "
                               f"{w.enc.n_heads} heads, FFN {w.enc.ffn}, seq {w.seq_len}, {w.n_perturbed} perturbed "
                               f"position(s), balls p={list(w.p_norms)} (0 = inf), batch {w.batch}, "
                               f"{w.steps} bisection probes on [{w.eps_lo}, {w.eps_hi}]",
                   "certifications_per_step": n_cert, "workspace_bytes": int(ws.numel()),
                   "batch_resident": bool(ws.numel() >= full),
                   "timed_region_times": ("the dominant kernel class" if timing else "nothing"),
                   "class_breakdown_from": ("last warm-up step" if timing and args.warmup > 0 else "timed region")},
        "roofline": roofline, "cpu_baseline": cpu, "measured_ceilings": ceil, "kernels": kernels,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
