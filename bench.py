#!/usr/bin/env python3
"""Benchmark of the AB-training hot path on one MI355X.

A step = one factored-layer forward + backward (lr_linear_fwd + lr_linear_bwd through the C ABI)
on the ViT-B/16 MLP fc1 layer at rank 192, batch 64 x 197 tokens, bf16 with fp32 accumulation
(the configuration the headline metric is quoted on).  The merge half of the metric -- ab_merge
of the full ViT-B/16 linear layer set, 48 layers x G = 4 copies, fp32 -- is timed in the same run
and reported in extra keys.  Inputs are seeded synthetic arrays already resident in HBM when the
timed region starts.

Prints ONE JSON line.  `--gpus N` with N > 1 is refused: this build runs on one GPU.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "factored fwd+bwd TFLOP/s (% bf16 MFMA peak) + ab_merge ms per ViT-B/16 layer set"
PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E
# HBM bytes of one forward chain launch on config 2, from two rocprofv3 --pmc runs of this file
# (profiles/chain2_r192_cfg2_pmc.txt): FETCH_SIZE 15623 KiB x 2.0 (the factor that makes a plain
# 256 MiB copy read 256 MiB) + WRITE_SIZE 80376 KiB x 1.0.  A stored measurement, not a live one.
CHAIN_FWD_TRAFFIC_BYTES = int((15623.2 * 2.0 + 80376.0) * 1024)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--merge-iters", type=int, default=3)
    ap.add_argument("--no-merge", action="store_true", help="skip the ab_merge timing")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline")
    ap.add_argument("--pmc-copy", action="store_true",
                    help="also run one plain 256 MiB device copy: the reference dispatch that scales the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run of this command")
    ap.add_argument("--no-group", action="store_true", help="skip the group-training step timings")
    ap.add_argument("--no-conv", action="store_true", help="skip the native factored-convolution timings")
    ap.add_argument("--all-configs", action="store_true",
                    help="also time every config-3 / config-4 case (extra key `cases`)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures ONE GPU (the multi-group structure is emulated as G factor "
              "copies in one GPU's memory); --gpus N with N > 1 is not supported.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2405_01067_amd import binding as abt
    from paper_2405_01067_amd import inputs as gen

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback.", file=sys.stderr)
        sys.exit(3)
    abt.load()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    bf16 = torch.bfloat16

    def up(x, dtype):
        return torch.from_numpy(np.ascontiguousarray(x)).to(dev).to(dtype)

    class Step:
        """Preallocated buffers of one layer; run() = forward + backward, nothing allocated."""

        def __init__(self, c):
            self.M, self.m, self.n, self.r = c["M"], c["m"], c["n"], c["r"]
            self.X, self.dY, self.A, self.B = (up(c[k], bf16) for k in ("X", "dY", "A", "B"))
            M, m, n, r = self.M, self.m, self.n, self.r
            self.Y = torch.empty((M, m), dtype=bf16, device=dev)
            self.T = torch.empty((M, r), dtype=bf16, device=dev)
            self.dX = torch.empty((M, n), dtype=bf16, device=dev)
            self.dA = torch.empty((m, r), dtype=torch.float32, device=dev)
            self.dB = torch.empty((r, n), dtype=torch.float32, device=dev)
            lib = abt.load()
            nb = lib.lr_linear_bwd_workspace_bytes(M, m, n, r, abt.ABT_BF16)
            self.ws = torch.empty(nb, dtype=torch.uint8, device=dev)
            self.flops = 6.0 * M * r * (m + n)
            # algorithmic bytes: every large tensor touched once per pass (bf16), factors and
            # factor gradients once
            self.bytes_fwd = 2.0 * (M * n + M * m + M * r + m * r + r * n)
            self.bytes_bwd = 2.0 * (M * m + M * n + M * n + 2 * M * r + m * r + r * n) + 4.0 * (m * r + r * n)

        def fwd(self):
            abt.lr_linear_fwd(self.X, self.A, self.B, save_T=True, Y=self.Y, T=self.T, workspace=self.ws)

        def bwd(self):
            abt.lr_linear_bwd(self.dY, self.X, self.T, self.A, self.B, dX=self.dX, dA=self.dA, dB=self.dB,
                              workspace=self.ws)

        def run(self):
            self.fwd()
            self.bwd()

    def time_steps(fn, steps, warmup):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps

    def event_ms(fn, iters, warmup=5, batch=10):
        """Average duration of one fn() from HIP events recorded on the launch stream (the binding
        launches on torch's current stream).  Events bracket `batch` back-to-back calls so that the
        host's launch cost hides behind the kernels and does not count as kernel time."""
        for _ in range(warmup):
            fn()
        n = max(1, iters // batch)
        starts = [torch.cuda.Event(enable_timing=True) for _ in range(n)]
        ends = [torch.cuda.Event(enable_timing=True) for _ in range(n)]
        torch.cuda.synchronize()
        for i in range(n):
            starts[i].record()
            for _ in range(batch):
                fn()
            ends[i].record()
        torch.cuda.synchronize()
        ts = sorted(s.elapsed_time(e) / batch for s, e in zip(starts, ends))
        return sum(ts) / len(ts), ts[len(ts) // 2], ts[0]

    # ------------------------------------------------------------------ headline: config 2
    c2 = gen.config2()
    step = Step(c2)
    sec = time_steps(step.run, args.steps, args.warmup)
    tflops = step.flops / sec / 1e12

    # dominant kernel: the fused chain kernel of the forward (one launch per lr_linear_fwd call),
    # HBM-bound at r = 192 (180 flop per algorithmic byte against a ridge of 312)
    fwd_avg, fwd_med, fwd_min = event_ms(step.fwd, min(args.steps, 100))
    bwd_avg, bwd_med, bwd_min = event_ms(step.bwd, min(args.steps, 100))
    achieved_gbs = step.bytes_fwd / (fwd_avg * 1e-3) / 1e9
    roofline = {
        "kernel": "chain2_bf16_kernel<192, 1, false> (lr_linear_fwd: T = X B^T, Y = T A^T fused, one launch per call)",
        "bound": "hbm", "achieved": round(achieved_gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
        "frac": round(achieved_gbs / PEAK_HBM_GBS, 4), "traffic": CHAIN_FWD_TRAFFIC_BYTES,
        "algorithmic_bytes_per_launch": step.bytes_fwd,
        "avg_launch_ms": round(fwd_avg, 5), "median_launch_ms": round(fwd_med, 5),
        "mfma_frac": round(2.0 * step.M * step.r * (step.m + step.n) / (fwd_avg * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
    }

    out = {
        "metric": METRIC, "value": round(tflops, 2), "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(sec * 1e3, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "configs[1]: ViT-B/16 MLP fc1 factored, W 3072x768, r=192, "
                               "X 12608x768 (batch 64 x 197 tokens), bf16 in / fp32 accumulate, fwd+bwd",
                   "M": step.M, "m": step.m, "n": step.n, "r": step.r,
                   "flops_per_step": step.flops},
        "pct_bf16_mfma_peak": round(100.0 * tflops / PEAK_BF16_TFLOPS, 2),
        "fwd_ms": round(fwd_avg, 5), "bwd_ms": round(bwd_avg, 5),
        "step_hbm_frac": round((step.bytes_fwd + step.bytes_bwd) / sec / 1e9 / PEAK_HBM_GBS, 4),
        "roofline": roofline,
    }

    if args.pmc_copy:
        src = torch.ones(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)          # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    # ------------------------------------------------------------------ optional: configs 3 and 4
    if args.all_configs:
        cases = []
        for name, M, m, n, r, seed in gen.config3_cases() + gen.config4_cases():
            relu = name.startswith("conv")
            st = Step(gen.lr_case(M, m, n, r, seed, relu_x=relu))
            s = time_steps(st.run, 30, 5)
            cases.append({"case": name, "M": M, "m": m, "n": n, "r": r, "ms": round(s * 1e3, 4),
                          "tflops": round(st.flops / s / 1e12, 1),
                          "pct_mfma_peak": round(100 * st.flops / s / 1e12 / PEAK_BF16_TFLOPS, 2),
                          "hbm_frac": round((st.bytes_fwd + st.bytes_bwd) / s / 1e9 / PEAK_HBM_GBS, 4)})
            del st
            torch.cuda.empty_cache()
        out["cases"] = cases

    # ------------------------------------------------------------------ factored 3x3 convolutions, native (extra key)
    # config 4's two 3x3 cases without the patch matrix: same flops as the im2col form, the
    # activation read at its true size (lr_conv_fwd + lr_conv_bwd, all three gradients)
    if not args.no_conv:
        conv = []
        for name, N, H, W, C, m, r in gen.RESNET50_CONVS_NATIVE:
            c = gen.conv_case(N, H, W, C, m, r, 3, 3, seed=11)
            act, dYc, Ac, Bc = (up(c[k], bf16) for k in ("act", "dY", "A", "B"))
            Mc, nc = N * H * W, 9 * C
            Yc = torch.empty((Mc, m), dtype=bf16, device=dev)
            Tc = torch.empty((Mc, r), dtype=bf16, device=dev)
            dAct = torch.empty_like(act)
            dAc = torch.empty((m, r), dtype=torch.float32, device=dev)
            dBc = torch.empty((r, nc), dtype=torch.float32, device=dev)
            geom = abt.ConvGeom(N, H, W, C, 3, 3)
            import ctypes
            wsb = abt.load().lr_conv_bwd_workspace_bytes(ctypes.byref(geom), m, r, abt.ABT_BF16)
            wsc = torch.empty(wsb, dtype=torch.uint8, device=dev)

            def conv_step():
                abt.lr_conv_fwd(act, Ac, Bc, 3, 3, save_T=True, Y=Yc, T=Tc)
                abt.lr_conv_bwd(dYc, act, Tc, Ac, Bc, 3, 3, dAct=dAct, dA=dAc, dB=dBc, workspace=wsc)

            sc = time_steps(conv_step, 50, 10)
            flops = 6.0 * Mc * r * (m + nc)
            # algorithmic bytes: activation, its gradient, Y, dY, T (written, read), dT (written, read twice)
            byt = 2.0 * (2 * Mc * C + 2 * Mc * m + 5 * Mc * r + 2 * (m * r + r * nc)) + 4.0 * (m * r + r * nc)
            conv.append({"case": name, "N": N, "H": H, "W": W, "C": C, "m": m, "r": r, "ms": round(sc * 1e3, 4),
                         "tflops": round(flops / sc / 1e12, 1),
                         "pct_mfma_peak": round(100 * flops / sc / 1e12 / PEAK_BF16_TFLOPS, 2),
                         "hbm_frac": round(byt / sc / 1e9 / PEAK_HBM_GBS, 4)})
            del act, dYc, Ac, Bc, Yc, Tc, dAct, dAc, dBc, wsc
            torch.cuda.empty_cache()
        out["conv_native"] = conv

    # ------------------------------------------------------------------ merge: config 5 (gap-centred threshold)
    if not args.no_merge:
        table = gen.config5_layers()
        layers = []
        alg_bytes = 0.0
        for idx, name, m, n, seed in table:
            lay = gen.merge_layer(m, n, seed)
            k_cap = gen.CFG5_K_IN
            layers.append(dict(
                A_copies=[up(a, torch.float32) for a in lay["A_copies"]],
                B_copies=[up(b, torch.float32) for b in lay["B_copies"]],
                tau=gen.CFG5_TAU_GAP, k_cap=k_cap,
                A_out=torch.empty((m, k_cap), dtype=torch.float32, device=dev),
                B_out=torch.empty((k_cap, n), dtype=torch.float32, device=dev),
                S_out=torch.empty((k_cap,), dtype=torch.float32, device=dev),
                k_out=torch.zeros((), dtype=torch.int32, device=dev)))
            alg_bytes += 4.0 * (gen.CFG5_G * (m + n) * gen.CFG5_K_IN + (m + n) * gen.CFG5_GAP_AT)
        ws_holder = {}

        def merge_once():
            outs = abt.ab_merge_batched(layers, workspace=ws_holder.get("ws"), check_converged=False)
            ws_holder["ws"] = outs[0]["workspace"]
            return outs

        outs = merge_once()
        torch.cuda.synchronize()
        sweeps = [abt.merge_info(ws_holder["ws"], i)[0] for i in range(len(layers))]
        ranks = [int(o["k"].item()) for o in outs]
        t0 = time.perf_counter()
        for _ in range(args.merge_iters):
            merge_once()
        torch.cuda.synchronize()
        merge_ms = (time.perf_counter() - t0) / args.merge_iters * 1e3
        out["ab_merge_ms_per_layer_set"] = round(merge_ms, 3)
        out["ab_merge"] = {"layers": len(layers), "G": gen.CFG5_G, "k_in": gen.CFG5_K_IN, "tau": gen.CFG5_TAU_GAP,
                           "ranks_min_max": [min(ranks), max(ranks)], "jacobi_sweeps_max": max(sweeps),
                           "algorithmic_bytes": alg_bytes,
                           "hbm_frac_whole_merge": round(alg_bytes / (merge_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 5)}
        del layers, outs
        ws_holder.clear()
        torch.cuda.empty_cache()

    # ------------------------------------------------------------------ ab_factorize: dense ViT-B/16 weights (extra key)
    if not args.no_merge:
        rng = np.random.default_rng(7)
        shapes = (("qkv", 2304, 768), ("proj", 768, 768), ("fc1", 3072, 768), ("fc2", 768, 3072))
        dense = []
        for name, m, n in shapes:           # one planted matrix per shape, used for all 12 blocks
            sigma = gen.power_law_spectrum(min(m, n), gap_at=gen.CFG5_GAP_AT)
            Lf, Rf, _, _ = gen.planted_factor_pair(rng, m, n, sigma)
            dense.append(up((Lf @ Rf).astype(np.float32), torch.float32))
        fl = [dict(W=dense[i % 4], tau=gen.CFG5_TAU_GAP, k_cap=gen.CFG5_K_IN) for i in range(48)]
        o = abt.ab_factorize_batched(fl)                      # warm-up, also checks convergence
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        o = abt.ab_factorize_batched(fl, workspace=o[0]["workspace"], check_converged=False)
        torch.cuda.synchronize()
        fz_ms = (time.perf_counter() - t0) * 1e3
        out["ab_factorize"] = {"ms_per_layer_set": round(fz_ms, 1), "layers": 48, "K": 768,
                               "ranks_min_max": [min(int(x["k"].item()) for x in o), max(int(x["k"].item()) for x in o)],
                               "note": "48 dense ViT-B/16 weights with the config-5 spectrum in one batched call"}
        del dense, fl, o
        torch.cuda.empty_cache()

    # ------------------------------------------------------------------ group-training step (extra key)
    # A-groups skip dB, B-groups skip dA (5/6 of the full step's flops); then one AdamW launch over
    # the trained factors of all 48 ViT-B/16 layers at rank 192 (fp32 state, bf16 copy written).
    if not args.no_group:
        def step_A():
            step.fwd()
            abt.lr_linear_bwd(step.dY, step.X, step.T, step.A, step.B, dX=step.dX, dA=step.dA, need_dB=False,
                              workspace=step.ws)

        def step_B():
            step.fwd()
            abt.lr_linear_bwd(step.dY, step.X, step.T, step.A, step.B, dX=step.dX, dB=step.dB, need_dA=False,
                              workspace=step.ws)

        ga_ms = event_ms(step_A, min(args.steps, 100))[0]
        gb_ms = event_ms(step_B, min(args.steps, 100))[0]
        tensors, elems = [], 0
        for blk in range(gen.VIT_B16_BLOCKS):
            for li, (name, m, n) in enumerate(gen.VIT_B16_LINEARS):
                cnt = m * 192 if (blk + li) % 2 == 0 else 192 * n
                elems += cnt
                tensors.append(dict(param=torch.zeros(cnt, device=dev), grad=torch.full((cnt,), 1e-3, device=dev),
                                    exp_avg=torch.zeros(cnt, device=dev), exp_avg_sq=torch.zeros(cnt, device=dev),
                                    param_bf16=torch.empty(cnt, dtype=bf16, device=dev)))
        counter = {"t": 0}
        plan = abt.AdamwPlan(tensors)            # the table is marshalled once, as a training loop would

        def adamw_once():
            counter["t"] += 1
            abt.ab_adamw_step(plan, step=counter["t"], lr=1e-3, lr_scale=1.0)

        ad_ms = event_ms(adamw_once, min(args.steps, 100))[0]
        ad_bytes = 30.0 * elems
        # the same volume through a plain device copy (half read, half written): what this box
        # sustains for a mixed read/write stream
        src = torch.empty(int(ad_bytes) // 2, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        cp_ms = event_ms(lambda: dst.copy_(src), min(args.steps, 100))[0]
        del src, dst
        flops56 = step.flops * 5.0 / 6.0
        out["group_step"] = {"workload": "config 2 layer, one factor frozen; AdamW over the trained factors of 48 layers",
                             "A_group_ms": round(ga_ms, 4), "B_group_ms": round(gb_ms, 4),
                             "A_group_tflops": round(flops56 / (ga_ms * 1e-3) / 1e12, 1),
                             "B_group_tflops": round(flops56 / (gb_ms * 1e-3) / 1e12, 1),
                             "adamw_ms": round(ad_ms, 4), "adamw_elements": elems,
                             "adamw_GBps": round(ad_bytes / (ad_ms * 1e-3) / 1e9, 1),
                             "adamw_hbm_frac": round(ad_bytes / (ad_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                             "device_copy_same_bytes_GBps": round(ad_bytes / (cp_ms * 1e-3) / 1e9, 1)}
        del tensors, plan
        torch.cuda.empty_cache()

    # ------------------------------------------------------------------ CPU oracle beside it (reported, not a target)
    if not args.no_cpu:
        from oracle import ab_oracle as orc
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count() or 1
        reps = 0
        t0 = time.perf_counter()
        while reps < 3 or (time.perf_counter() - t0 < 10.0 and reps < 200):
            orc.lr_linear_fwd(c2["X"], c2["A"], c2["B"])
            orc.lr_linear_bwd(c2["dY"], c2["X"], c2["A"], c2["B"])
            reps += 1
        cpu_s = (time.perf_counter() - t0) / reps
        out["cpu_baseline"] = {"value": round(step.flops / cpu_s / 1e12, 4), "unit": "TFLOP/s", "cores": cores,
                               "kind": "oracle",
                               "sample": f"the full config-2 step (fwd + bwd, fp64 NumPy/OpenBLAS) {reps} times, "
                                         f"{cpu_s:.3f} s each"}
        if not args.no_merge:
            block = [gen.merge_layer(m, n, seed) for idx, name, m, n, seed in gen.config5_layers()[:4]]
            t0 = time.perf_counter()
            for lay in block:
                orc.ab_merge(lay["A_copies"], lay["B_copies"], tau=gen.CFG5_TAU_GAP)
            blk_s = time.perf_counter() - t0
            out["cpu_baseline"]["ab_merge_ms_per_layer_set_extrapolated"] = round(blk_s * 12 * 1e3, 1)
            out["cpu_baseline"]["ab_merge_sample"] = "one ViT-B/16 block (4 of the 48 layers) timed, x 12"

    print(json.dumps(out))


if __name__ == "__main__":
    main()
