#!/usr/bin/env python3
"""Benchmark of the AB-training hot path on one MI355X.

A step = one pass over the twelve ViT-B/16 cases at batch 256 x 197 tokens (four linear shapes
x ranks 96, 192, 384): factored-layer forward + backward through the C ABI (lr_linear_fwd +
lr_linear_bwd), bf16 with fp32 accumulation, 2.50 TFLOP of algorithmic work (6 M r (m + n) per
case).  `value` = that work / the time of a step.  Every case keeps two sets of activation
buffers and alternates between them, so no launch finds its inputs in the 256 MB last-level cache.

Extra keys, all on by default: every case against both roofs (HIP-event medians, with the number
on one unrotated buffer set beside it, labelled), the batch-64 fc1 layer, the three ResNet-50
im2col cases, the native 3x3 convolutions, the fp32 toy case, the merge of the full ViT-B/16
layer set (48 layers x G = 4 copies, per-stage ms, both thresholds, with W, by concatenation),
the decomposition of 48 dense weights, the group-training step, and the CPU oracle timed on the
same cases.  Inputs are seeded synthetic arrays already resident in HBM when a timed region starts.

Prints ONE JSON line.  `--gpus N` with N > 1 is refused: this build runs on one GPU.
"""
import argparse
import ctypes
import gc
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
CACHE_BYTES = 256 << 20     # last-level cache: a rotated working set must exceed it
# HBM bytes of one launch of the dominant kernel (forward chain of fc1 at r = 384, M = 50432) from two
# rocprofv3 --pmc runs of `bench.py --only-launch fc1_r384 --pmc-copy` (profiles/chain_fwd_pmc_counters.txt,
# second table): FETCH_SIZE 58308.8 KiB x 2.00 (the factor that makes a plain 256 MiB copy read 256 MiB)
# + WRITE_SIZE 340459.5 KiB x 1.00.  A stored measurement: re-collect it when the kernel changes.
DOMINANT_TRAFFIC_BYTES = int((58308.8 * 2.0 + 340459.5) * 1024)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--merge-iters", type=int, default=10)
    ap.add_argument("--event-iters", type=int, default=60, help="timed launches per HIP-event median")
    ap.add_argument("--no-merge", action="store_true", help="skip the merge and factorisation timings")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline")
    ap.add_argument("--no-extra", action="store_true",
                    help="skip configs 1, 2, 4, the native convolutions and the group-training step")
    ap.add_argument("--only-launch", metavar="CASE", default=None,
                    help="profiling aid: run nothing but --steps forward launches of this config-3 case "
                         "(e.g. fc1_r384; config2 for the batch-64 layer) after --warmup, so that a kernel trace of the command holds "
                         "exactly that launch; prints its HIP-event timing")
    ap.add_argument("--only-step", metavar="CASE", default=None,
                    help="profiling aid: like --only-launch, but whole steps (forward + backward) of the case")
    ap.add_argument("--only-merge", action="store_true",
                    help="profiling aid: run nothing but the merge of the ViT-B/16 layer set (warm-up merges, "
                         "then --merge-iters timed ones)")
    ap.add_argument("--pmc-copy", action="store_true",
                    help="also run one plain 256 MiB device copy: the reference dispatch that scales the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run of this command")
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
    lib = abt.load()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    bf16 = torch.bfloat16
    t_start = time.perf_counter()

    def note(msg):
        print(f"[bench {time.perf_counter() - t_start:6.1f}s] {msg}", file=sys.stderr, flush=True)

    def up(x, dtype):
        return torch.from_numpy(np.ascontiguousarray(x)).to(dev).to(dtype)

    class Step:
        """One layer's training step on preallocated buffers.  `sets` copies of the activations
        (inputs cloned, outputs separate); call i uses set i mod sets.  Nothing is allocated in a call."""

        def __init__(self, c, sets):
            self.M, self.m, self.n, self.r = c["M"], c["m"], c["n"], c["r"]
            M, m, n, r = self.M, self.m, self.n, self.r
            self.A, self.B = up(c["A"], bf16), up(c["B"], bf16)
            X, dY = up(c["X"], bf16), up(c["dY"], bf16)
            self.sets = []
            for i in range(sets):
                self.sets.append(dict(
                    X=X if i == 0 else X.clone(), dY=dY if i == 0 else dY.clone(),
                    Y=torch.empty((M, m), dtype=bf16, device=dev), T=torch.empty((M, r), dtype=bf16, device=dev),
                    dX=torch.empty((M, n), dtype=bf16, device=dev)))
            self.dA = torch.empty((m, r), dtype=torch.float32, device=dev)
            self.dB = torch.empty((r, n), dtype=torch.float32, device=dev)
            self.ws = torch.empty(lib.lr_linear_bwd_workspace_bytes(M, m, n, r, abt.ABT_BF16), dtype=torch.uint8, device=dev)
            self.flops = 6.0 * M * r * (m + n)
            # algorithmic bytes: every large tensor touched once per pass (bf16), factors and
            # factor gradients once
            self.bytes_fwd = 2.0 * (M * n + M * m + M * r + m * r + r * n)
            self.bytes_bwd = 2.0 * (M * m + M * n + M * n + 2 * M * r + m * r + r * n) + 4.0 * (m * r + r * n)
            self.set_bytes = 2.0 * (2 * M * n + 2 * M * m + M * r)
            self.i = 0

        def fwd(self, i):
            b = self.sets[i % len(self.sets)]
            abt.lr_linear_fwd(b["X"], self.A, self.B, save_T=True, Y=b["Y"], T=b["T"], workspace=self.ws)

        def bwd(self, i, **kw):
            b = self.sets[i % len(self.sets)]
            if not kw:
                kw = dict(dX=b["dX"], dA=self.dA, dB=self.dB)
            abt.lr_linear_bwd(b["dY"], b["X"], b["T"], self.A, self.B, workspace=self.ws, **kw)

        def run(self, i):
            self.fwd(i)
            self.bwd(i)

    def sets_for(set_bytes):
        """At least two sets, and enough that the rotated working set is over twice the cache."""
        return max(2, int(-(-2 * CACHE_BYTES // set_bytes)))

    def event_ms(fn, iters=None, warmup=10, batch=10):
        """Durations of fn(i) from HIP events on the launch stream (the binding launches on torch's
        current stream).  Events bracket `batch` back-to-back calls so that the host's launch cost
        hides behind the kernels.  Returns (mean, median, min) in ms over the batches."""
        iters = iters or args.event_iters
        for i in range(warmup):
            fn(i)
        nb = max(3, iters // batch)
        starts = [torch.cuda.Event(enable_timing=True) for _ in range(nb)]
        ends = [torch.cuda.Event(enable_timing=True) for _ in range(nb)]
        torch.cuda.synchronize()
        k = warmup
        for b in range(nb):
            starts[b].record()
            for _ in range(batch):
                fn(k)
                k += 1
            ends[b].record()
        torch.cuda.synchronize()
        ts = sorted(s.elapsed_time(e) / batch for s, e in zip(starts, ends))
        return sum(ts) / len(ts), ts[len(ts) // 2], ts[0]

    def roofs(st, ms, flops=None, nbytes=None):
        """A measured time against both roofs (algorithmic flops and bytes)."""
        flops = st.flops if flops is None else flops
        nbytes = st.bytes_fwd + st.bytes_bwd if nbytes is None else nbytes
        mfma_us = flops / PEAK_BF16_TFLOPS / 1e6
        hbm_us = nbytes / PEAK_HBM_GBS / 1e3
        return {"tflops": round(flops / ms / 1e9, 1),
                "pct_mfma_peak": round(100 * flops / ms / 1e9 / PEAK_BF16_TFLOPS, 2),
                "hbm_frac": round(nbytes / ms / 1e6 / PEAK_HBM_GBS, 4),
                "mfma_limit_us": round(mfma_us, 1), "hbm_limit_us": round(hbm_us, 1),
                "bound": "mfma" if mfma_us > hbm_us else "hbm",
                "frac_of_bound": round(max(mfma_us, hbm_us) / (ms * 1e3), 4)}

    def case_report(name, st):
        fwd = event_ms(st.fwd)
        bwd = event_ms(st.bwd)
        both = event_ms(st.run)
        warm = event_ms(lambda i: st.run(0))
        rep = {"case": name, "M": st.M, "m": st.m, "n": st.n, "r": st.r, "buffer_sets": len(st.sets),
               "rotated_MB": round(st.set_bytes * len(st.sets) / 1e6),
               "ms": round(both[1], 4), "ms_min": round(both[2], 4), "fwd_ms": round(fwd[1], 4), "bwd_ms": round(bwd[1], 4),
               "ms_one_buffer_set_cache_warm": round(warm[1], 4)}
        rep.update(roofs(st, both[1]))
        rep["fwd_launch"] = roofs(st, fwd[0], flops=st.flops / 3.0, nbytes=st.bytes_fwd)
        rep["fwd_launch"]["avg_ms"] = round(fwd[0], 5)
        return rep

    def cpu_cores():
        try:
            from threadpoolctl import threadpool_info
            return max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            return os.cpu_count() or 1

    cpu = {"flops": 0.0, "sec": 0.0, "cases": []}

    def cpu_oracle_step(name, c, flops):
        """The oracle's forward + backward of one case, once, in fp64 on the host."""
        from oracle import ab_oracle as orc
        t0 = time.perf_counter()
        orc.lr_linear_fwd(c["X"], c["A"], c["B"])
        orc.lr_linear_bwd(c["dY"], c["X"], c["A"], c["B"])
        dt = time.perf_counter() - t0
        cpu["flops"] += flops
        cpu["sec"] += dt
        cpu["cases"].append(name)

    # ------------------------------------------------------------------ profiling aid: one launch only
    def pmc_copy():
        src = torch.ones(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)          # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    if args.only_launch or args.only_step:
        which = args.only_launch or args.only_step
        case = [cs for cs in gen.config3_cases() if cs[0] == which]
        if which == "config2":
            c = gen.config2()
            name, M, m, n, r = "config2", c["M"], c["m"], c["n"], c["r"]
        elif case:
            name, M, m, n, r, seed = case[0]
            c = gen.lr_case(M, m, n, r, seed)
        else:
            print(f"bench.py: no config-3 case named {which} (or config2)", file=sys.stderr)
            sys.exit(2)
        st = Step(c, sets_for(2.0 * (2 * M * n + 2 * M * m + M * r)))
        avg, med, mn = event_ms(st.fwd if args.only_launch else st.run, iters=args.steps, warmup=args.warmup)
        if args.pmc_copy:
            pmc_copy()
        print(json.dumps({"only_launch" if args.only_launch else "only_step": name, "avg_ms": avg, "median_ms": med,
                          "min_ms": mn, "calls": args.warmup + max(3, args.steps // 10) * 10}))
        return

    if args.only_merge:
        out = {"only_merge": True}
        args.no_extra, args.no_cpu, args.no_merge = True, True, False
        cases = []
    if not args.only_merge:
        # ------------------------------------------------------------------ headline: config 3
        steps3 = []
        for name, M, m, n, r, seed in gen.config3_cases():
            c = gen.lr_case(M, m, n, r, seed)
            st = Step(c, sets_for(2.0 * (2 * M * n + 2 * M * m + M * r)))
            steps3.append((name, st))
            if not args.no_cpu:
                cpu_oracle_step(name, c, st.flops)
            del c
            gc.collect()
        note(f"config 3: {len(steps3)} cases resident, {torch.cuda.memory_allocated() / 2**30:.1f} GiB")
        total_flops = sum(st.flops for _, st in steps3)

        def whole_step(i):
            for _, st in steps3:
                st.run(i)

        for i in range(args.warmup):
            whole_step(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            whole_step(args.warmup + i)
        torch.cuda.synchronize()
        sec = (time.perf_counter() - t0) / args.steps
        tflops = total_flops / sec / 1e12
        note(f"config 3: {sec * 1e3:.3f} ms per step, {tflops:.1f} TFLOP/s")

        cases = [case_report(name, st) for name, st in steps3]
        summed_ms = sum(cs["ms"] for cs in cases)

        # dominant kernel of a step: the fused chain kernel at R = 384 on the widest layer (fc1: the
        # forward launch T = X B^T, Y = T A^T; the backward runs the same kernel for dT, dX).  The case
        # is MFMA-bound (474 flop per algorithmic byte against a ridge of 312).
        dom_name = "fc1_r384"
        dom = dict(steps3)[dom_name]
        dom_avg = event_ms(dom.fwd)[0]
        dom_flops = 2.0 * dom.M * dom.r * (dom.m + dom.n)
        achieved = dom_flops / (dom_avg * 1e-3) / 1e12
        roofline = {
            "kernel": "chain3_bf16_kernel<384> (lr_linear_fwd of fc1 at r = 384, M = 50432: "
                      "T = X B^T and Y = T A^T fused, one launch per call)",
            "bound": "mfma", "achieved": round(achieved, 1), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
            "frac": round(achieved / PEAK_BF16_TFLOPS, 4), "traffic": DOMINANT_TRAFFIC_BYTES,
        "traffic_source": "stored measurement, not live: profiles/chain_fwd_pmc_counters.txt",
            "algorithmic_flops_per_launch": dom_flops, "algorithmic_bytes_per_launch": dom.bytes_fwd,
            "avg_launch_ms": round(dom_avg, 5),
            "hbm_frac": round(dom.bytes_fwd / (dom_avg * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
            "profile": "profiles/chain3_r384_cfg3_fc1_kernel_trace.txt",
        }

        out = {
            "metric": METRIC, "value": round(tflops, 2), "unit": "TFLOP/s",
            "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "ms_per_step": round(sec * 1e3, 5), "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": "configs[2]: all four ViT-B/16 linear shapes (qkv 2304x768, proj 768x768, "
                                   "fc1 3072x768, fc2 768x3072) factored at r in {96, 192, 384}, X 50432 rows "
                                   "(batch 256 x 197 tokens), bf16 in / fp32 accumulate, fwd+bwd of all twelve "
                                   "cases = one step",
                       "cases": len(steps3), "flops_per_step": total_flops,
                       "buffer_sets_per_case": "2 or more, alternated (rotated working set > 2 x 256 MB)"},
            "pct_bf16_mfma_peak": round(100.0 * tflops / PEAK_BF16_TFLOPS, 2),
            "config3_sum_of_case_medians_ms": round(summed_ms, 4),
            "config3_tflops_from_case_medians": round(total_flops / summed_ms / 1e9, 1),
            "roofline": roofline,
            "cases": cases,
        }
        for _, st in steps3:
            del st
        del steps3, dom
        gc.collect()
        torch.cuda.empty_cache()

    if args.pmc_copy:
        pmc_copy()

    # ------------------------------------------------------------------ config 2 (batch 64 fc1, r = 192)
    step2 = None
    if not args.no_extra:
        c2 = gen.config2()
        step2 = Step(c2, sets_for(2.0 * (2 * c2["M"] * c2["n"] + 2 * c2["M"] * c2["m"] + c2["M"] * c2["r"])))
        if not args.no_cpu:
            cpu_oracle_step("config2", c2, step2.flops)
        del c2
        rep = case_report("fc1_r192_batch64", step2)
        for i in range(20):
            step2.run(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(200):
            step2.run(i)
        torch.cuda.synchronize()
        w = (time.perf_counter() - t0) / 200
        rep["wall_clock_ms_200_steps"] = round(w * 1e3, 4)
        rep["wall_clock_tflops"] = round(step2.flops / w / 1e12, 1)
        out["config2"] = rep
        note(f"config 2: {rep['ms']} ms rotated, {rep['ms_one_buffer_set_cache_warm']} ms cache-warm")

        # -------------------------------------------------------------- config 4 (ResNet-50 im2col cases)
        c4 = []
        for name, M, m, n, r, seed in gen.config4_cases():
            c = gen.lr_case(M, m, n, r, seed, relu_x=True)
            st = Step(c, sets_for(2.0 * (2 * M * n + 2 * M * m + M * r)))
            if not args.no_cpu:
                cpu_oracle_step(name, c, st.flops)
            del c
            c4.append(case_report(name, st))
            del st
            gc.collect()
            torch.cuda.empty_cache()
        out["config4"] = c4
        note("config 4 done")

        # -------------------------------------------------------------- config 1 (fp32 toy case: latency)
        c1 = gen.config1_dense(0)
        # factors of the toy weight: any well-scaled pair serves a timing; inputs of the parity
        # test come from the oracle's own decomposition, here the planted Gaussian pair suffices
        rng = np.random.default_rng(0)
        A1 = up(gen.gaussian(rng, (256, 32), std=32 ** -0.5), torch.float32)
        B1 = up(gen.gaussian(rng, (32, 256), std=256 ** -0.5), torch.float32)
        X1, dY1 = up(c1["X"], torch.float32), up(c1["dY"], torch.float32)
        Y1 = torch.empty((64, 256), device=dev)
        T1 = torch.empty((64, 32), device=dev)
        dX1 = torch.empty((64, 256), device=dev)
        dA1 = torch.empty((256, 32), device=dev)
        dB1 = torch.empty((32, 256), device=dev)
        ws1 = torch.empty(max(lib.lr_linear_bwd_workspace_bytes(64, 256, 256, 32, abt.ABT_F32),
                              lib.lr_linear_fwd_workspace_bytes(64, 256, 256, 32, abt.ABT_F32)), dtype=torch.uint8, device=dev)

        def step1(i):
            abt.lr_linear_fwd(X1, A1, B1, save_T=True, Y=Y1, T=T1, workspace=ws1)
            abt.lr_linear_bwd(dY1, X1, T1, A1, B1, dX=dX1, dA=dA1, dB=dB1, workspace=ws1)

        s1 = event_ms(step1)
        copies = [A1, A1 + 1e-3 * torch.randn_like(A1)], [B1, B1 + 1e-3 * torch.randn_like(B1)]
        o1 = abt.ab_merge(copies[0], copies[1], tau=0.1)
        for _ in range(3):
            abt.ab_merge(copies[0], copies[1], tau=0.1, workspace=o1["workspace"], check_converged=False)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(10):
            abt.ab_merge(copies[0], copies[1], tau=0.1, workspace=o1["workspace"], check_converged=False)
        torch.cuda.synchronize()
        out["config1"] = {"workload": "fp32, W 256x256 at r = 32, X 64x256: launch-latency bound",
                          "step_ms": round(s1[1], 4), "merge_ms_G2": round((time.perf_counter() - t0) / 10 * 1e3, 3),
                          "merge_rank": int(o1["k"].item())}

        # -------------------------------------------------------------- factored 3x3 convolutions, native
        # config 4's two 3x3 cases without the patch matrix: same flops as the im2col form, the
        # activation read at its true size (lr_conv_fwd + lr_conv_bwd, all three gradients)
        conv = []
        native = [(nm, N, H, W, C, m, r, 3, 3, 1) for nm, N, H, W, C, m, r in gen.RESNET50_CONVS_NATIVE] + \
                 [row + (2,) for row in gen.RESNET50_CONVS_STRIDED]
        for name, N, H, W, C, m, r, kh, kw, stride in native:
            c = gen.conv_case(N, H, W, C, m, r, kh, kw, seed=11, stride=stride)
            Mc, nc = N * (-(-H // stride)) * (-(-W // stride)), kh * kw * C
            sets = sets_for(2.0 * (2 * N * H * W * C + 2 * Mc * m + Mc * r))
            act0, dY0 = up(c["act"], bf16), up(c["dY"], bf16)
            Ac, Bc = up(c["A"], bf16), up(c["B"], bf16)
            bufs = [dict(act=act0 if i == 0 else act0.clone(), dY=dY0 if i == 0 else dY0.clone(),
                         Y=torch.empty((Mc, m), dtype=bf16, device=dev), T=torch.empty((Mc, r), dtype=bf16, device=dev),
                         dAct=torch.empty_like(act0)) for i in range(sets)]
            dAc = torch.empty((m, r), dtype=torch.float32, device=dev)
            dBc = torch.empty((r, nc), dtype=torch.float32, device=dev)
            geom = abt.ConvGeom(N, H, W, C, kh, kw, stride)
            wsc = torch.empty(lib.lr_conv_bwd_workspace_bytes(ctypes.byref(geom), m, r, abt.ABT_BF16), dtype=torch.uint8, device=dev)

            def conv_step(i):
                b = bufs[i % len(bufs)]
                abt.lr_conv_fwd(b["act"], Ac, Bc, kh, kw, save_T=True, Y=b["Y"], T=b["T"], stride=stride)
                abt.lr_conv_bwd(b["dY"], b["act"], b["T"], Ac, Bc, kh, kw, dAct=b["dAct"], dA=dAc, dB=dBc, workspace=wsc,
                                stride=stride)

            sc = event_ms(conv_step)[1]
            flops = 6.0 * Mc * r * (m + nc)
            # algorithmic bytes: activation, its gradient, Y, dY, T (written, read), dT (written, read twice)
            byt = 2.0 * (2 * N * H * W * C + 2 * Mc * m + 5 * Mc * r + 2 * (m * r + r * nc)) + 4.0 * (m * r + r * nc)
            conv.append({"case": name, "N": N, "H": H, "W": W, "C": C, "m": m, "r": r, "kh": kh, "kw": kw,
                         "stride": stride, "buffer_sets": sets,
                         "ms": round(sc, 4), "tflops": round(flops / sc / 1e9, 1),
                         "pct_mfma_peak": round(100 * flops / sc / 1e9 / PEAK_BF16_TFLOPS, 2),
                         "hbm_frac": round(byt / sc / 1e6 / PEAK_HBM_GBS, 4)})
            del act0, dY0, Ac, Bc, bufs, dAc, dBc, wsc
            torch.cuda.empty_cache()
        out["conv_native"] = conv
        note("config 1, native convolutions done")

    # ------------------------------------------------------------------ merge: config 5
    if not args.no_merge:
        table = gen.config5_layers()
        host_layers = [gen.merge_layer(m, n, seed) for _, _, m, n, seed in table]
        k_cap = gen.CFG5_K_IN
        base = []
        alg_bytes = 0.0
        for (idx, name, m, n, seed), lay in zip(table, host_layers):
            base.append(dict(
                A_copies=[up(a, torch.float32) for a in lay["A_copies"]],
                B_copies=[up(b, torch.float32) for b in lay["B_copies"]],
                k_cap=k_cap,
                A_out=torch.empty((m, k_cap), dtype=torch.float32, device=dev),
                B_out=torch.empty((k_cap, n), dtype=torch.float32, device=dev),
                S_out=torch.empty((k_cap,), dtype=torch.float32, device=dev),
                k_out=torch.zeros((), dtype=torch.int32, device=dev)))
            alg_bytes += 4.0 * (gen.CFG5_G * (m + n) * gen.CFG5_K_IN + (m + n) * gen.CFG5_GAP_AT)
        note("config 5: inputs resident")

        def timed_merges(layers, iters, warm):
            """Median, min of `iters` batched merges (each bracketed by a device synchronisation on
            both sides) after `warm` untimed ones; the workspace is allocated once."""
            o = abt.ab_merge_batched(layers, check_converged=False)
            ws = o[0]["workspace"]
            for _ in range(max(0, warm - 1)):
                abt.ab_merge_batched(layers, workspace=ws, check_converged=False)
            ts = []
            for _ in range(iters):
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                o = abt.ab_merge_batched(layers, workspace=ws, check_converged=False)
                torch.cuda.synchronize()
                ts.append((time.perf_counter() - t0) * 1e3)
            ts.sort()
            sweeps = [abt.merge_info(ws, i)[0] for i in range(len(layers))]
            ranks = [int(x["k"].item()) for x in o]
            return ts[len(ts) // 2], ts[0], sweeps, ranks, ws

        gap = [dict(b, tau=gen.CFG5_TAU_GAP) for b in base]
        med, mn, sweeps, ranks, ws = timed_merges(gap, args.merge_iters, 4)
        prev = abt.set_merge_stage_timing(True)
        abt.ab_merge_batched(gap, workspace=ws, check_converged=False)
        stages = abt.merge_stage_ms()
        abt.set_merge_stage_timing(prev)
        streaming_ms = stages["mean_gram"] + stages["back_projection"]
        out["ab_merge_ms_per_layer_set"] = round(med, 3)
        out["ab_merge"] = {
            "workload": "configs[4]: 48 ViT-B/16 layers x G = 4 copies, k_in = 384, gap-centred threshold (k' = 192)",
            "layers": len(gap), "G": gen.CFG5_G, "k_in": gen.CFG5_K_IN, "tau": gen.CFG5_TAU_GAP,
            "ms_median": round(med, 3), "ms_min": round(mn, 3), "timed_merges": args.merge_iters, "warmup_merges": 4,
            "ranks_min_max": [min(ranks), max(ranks)], "jacobi_sweeps_min_max": [min(sweeps), max(sweeps)],
            "stage_ms": {k: round(v, 3) for k, v in stages.items()},
            "stage_ms_sum": round(sum(stages.values()), 3),
            "algorithmic_bytes": alg_bytes,
            "streaming_stages_hbm_frac": round(alg_bytes / (streaming_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
            "hbm_frac_whole_merge": round(alg_bytes / (med * 1e-3) / 1e9 / PEAK_HBM_GBS, 5)}
        note(f"merge: {med:.2f} ms median, stages {out['ab_merge']['stage_ms']}")
        del ws
        # literal threshold (k' = 17 or 18)
        lit = [dict(b, tau=gen.CFG5_TAU_LITERAL) for b in base]
        med, mn, sweeps, ranks, ws = timed_merges(lit, 3, 2)
        out["ab_merge"]["tau_0.1"] = {"ms_median": round(med, 3), "ranks_min_max": [min(ranks), max(ranks)],
                                      "jacobi_sweeps_min_max": [min(sweeps), max(sweeps)]}
        del ws, lit
        # with the dense average W written as well (340 MB more)
        withw = [dict(b, tau=gen.CFG5_TAU_GAP, want_W=True) for b in base]
        for (idx, name, m, n, seed), lay in zip(table, withw):
            lay["W_out"] = torch.empty((m, n), dtype=torch.float32, device=dev)
        med, mn, sweeps, ranks, ws = timed_merges(withw, 3, 2)
        out["ab_merge"]["with_W_out"] = {"ms_median": round(med, 3)}
        del ws, withw
        torch.cuda.empty_cache()
        # by concatenation (mode 1): copies of rank 192 each, core of min(G k, m, n) = 768 columns
        cat = []
        for b in base:
            cat.append(dict(A_copies=[a[:, :gen.CFG5_GAP_AT].contiguous() for a in b["A_copies"]],
                            B_copies=[x[:gen.CFG5_GAP_AT, :].contiguous() for x in b["B_copies"]],
                            tau=gen.CFG5_TAU_GAP, mode=1, k_cap=k_cap))
        med, mn, sweeps, ranks, ws = timed_merges(cat, 3, 2)
        out["ab_merge"]["mode1_k192_core768"] = {"ms_median": round(med, 1), "ranks_min_max": [min(ranks), max(ranks)],
                                                 "jacobi_sweeps_min_max": [min(sweeps), max(sweeps)]}
        note(f"merge variants done (mode 1: {med:.1f} ms)")
        del ws, cat, gap, base
        gc.collect()
        torch.cuda.empty_cache()

    if not args.no_merge and not args.only_merge:
        # -------------------------------------------------------------- ab_factorize: dense ViT-B/16 weights
        rng = np.random.default_rng(7)
        dense = []
        for name, m, n in gen.VIT_B16_LINEARS:     # one planted matrix per shape, used for all 12 blocks
            sigma = gen.power_law_spectrum(min(m, n), gap_at=gen.CFG5_GAP_AT)
            Lf, Rf, _, _ = gen.planted_factor_pair(rng, m, n, sigma)
            dense.append(up((Lf @ Rf).astype(np.float32), torch.float32))
        fl = [dict(W=dense[i % 4], tau=gen.CFG5_TAU_GAP, k_cap=gen.CFG5_K_IN) for i in range(48)]
        o = abt.ab_factorize_batched(fl)                      # warm-up, also checks convergence
        ts = []
        for _ in range(3):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            o = abt.ab_factorize_batched(fl, workspace=o[0]["workspace"], check_converged=False)
            torch.cuda.synchronize()
            ts.append((time.perf_counter() - t0) * 1e3)
        out["ab_factorize"] = {"ms_per_layer_set": round(sorted(ts)[1], 1), "layers": 48, "K": 768,
                               "ranks_min_max": [min(int(x["k"].item()) for x in o), max(int(x["k"].item()) for x in o)],
                               "note": "48 dense ViT-B/16 weights with the config-5 spectrum in one batched call"}
        del dense, fl, o
        torch.cuda.empty_cache()
        note("factorize done")

    # ------------------------------------------------------------------ group-training step (extra key)
    # A-groups skip dB, B-groups skip dA (5/6 of the full step's flops); then one AdamW launch over
    # the trained factors of all 48 ViT-B/16 layers at rank 192 (fp32 state, bf16 copy written).
    if step2 is not None:
        def step_A(i):
            b = step2.sets[i % len(step2.sets)]
            step2.fwd(i)
            step2.bwd(i, dX=b["dX"], dA=step2.dA, need_dB=False)

        def step_B(i):
            b = step2.sets[i % len(step2.sets)]
            step2.fwd(i)
            step2.bwd(i, dX=b["dX"], dB=step2.dB, need_dA=False)

        ga_ms = event_ms(step_A)[1]
        gb_ms = event_ms(step_B)[1]
        # four groups (two train A, two train B), each with its own buffers: group by group, and in the
        # grouped calls (one forward launch, four backward launches for all groups)
        G4 = 4
        base = step2.sets[0]
        gsets = [dict(X=base["X"].clone(), dY=base["dY"].clone(), A=step2.A.clone(), B=step2.B.clone(),
                      Y=torch.empty_like(base["Y"]), T=torch.empty_like(base["T"]), dX=torch.empty_like(base["dX"]),
                      dA=torch.empty_like(step2.dA), dB=torch.empty_like(step2.dB)) for _ in range(G4)]
        gws = torch.empty(lib.lr_linear_bwd_grouped_workspace_bytes(G4, step2.M, step2.m, step2.n, step2.r, abt.ABT_BF16),
                          dtype=torch.uint8, device=dev)

        def groups_one_by_one(i):
            for g, b in enumerate(gsets):
                abt.lr_linear_fwd(b["X"], b["A"], b["B"], save_T=True, Y=b["Y"], T=b["T"], workspace=step2.ws)
                if g < G4 // 2:
                    abt.lr_linear_bwd(b["dY"], b["X"], b["T"], b["A"], b["B"], dX=b["dX"], dA=b["dA"], need_dB=False, workspace=step2.ws)
                else:
                    abt.lr_linear_bwd(b["dY"], b["X"], b["T"], b["A"], b["B"], dX=b["dX"], dB=b["dB"], need_dA=False, workspace=step2.ws)

        fwd_groups = [dict(X=b["X"], A=b["A"], B=b["B"], Y=b["Y"], T=b["T"]) for b in gsets]
        bwd_groups = [dict(dY=b["dY"], X=b["X"], T=b["T"], A=b["A"], B=b["B"], dX=b["dX"],
                           dA=b["dA"] if g < G4 // 2 else None, dB=None if g < G4 // 2 else b["dB"]) for g, b in enumerate(gsets)]

        def groups_grouped(i):
            abt.lr_linear_fwd_grouped(fwd_groups)
            abt.lr_linear_bwd_grouped(bwd_groups, workspace=gws)

        g1_ms = event_ms(groups_one_by_one, batch=4)[1]
        gg_ms = event_ms(groups_grouped, batch=4)[1]
        del gsets, gws, fwd_groups, bwd_groups
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

        def adamw_once(i):
            counter["t"] += 1
            abt.ab_adamw_step(plan, step=counter["t"], lr=1e-3, lr_scale=1.0)

        ad_ms = event_ms(adamw_once)[1]
        ad_bytes = 30.0 * elems
        # the same volume through a plain device copy (half read, half written): what this box
        # sustains for a mixed read/write stream
        src = torch.empty(int(ad_bytes) // 2, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        cp_ms = event_ms(lambda i: dst.copy_(src))[1]
        del src, dst
        flops56 = step2.flops * 5.0 / 6.0
        out["group_step"] = {"workload": "config 2 layer, one factor frozen; AdamW over the trained factors of 48 layers",
                             "A_group_ms": round(ga_ms, 4), "B_group_ms": round(gb_ms, 4),
                             "A_group_tflops": round(flops56 / (ga_ms * 1e-3) / 1e12, 1),
                             "B_group_tflops": round(flops56 / (gb_ms * 1e-3) / 1e12, 1),
                             "four_groups_one_by_one_ms": round(g1_ms, 4), "four_groups_grouped_calls_ms": round(gg_ms, 4),
                             "four_groups_grouped_tflops": round(4 * flops56 / (gg_ms * 1e-3) / 1e12, 1),
                             "adamw_ms": round(ad_ms, 4), "adamw_elements": elems,
                             "adamw_GBps": round(ad_bytes / (ad_ms * 1e-3) / 1e9, 1),
                             "adamw_hbm_frac": round(ad_bytes / (ad_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                             "device_copy_same_bytes_GBps": round(ad_bytes / (cp_ms * 1e-3) / 1e9, 1)}
        del tensors, plan
        torch.cuda.empty_cache()

    # ------------------------------------------------------------------ CPU oracle beside it (reported, not a target)
    if not args.no_cpu:
        out["cpu_baseline"] = {"value": round(cpu["flops"] / cpu["sec"] / 1e12, 4), "unit": "TFLOP/s",
                               "cores": cpu_cores(), "kind": "oracle",
                               "sample": f"the oracle's forward + backward (fp64 NumPy products) once on each of "
                                         f"{len(cpu['cases'])} cases (all of config 3"
                                         + (", config 2, config 4" if not args.no_extra else "")
                                         + f"): {cpu['flops'] / 1e12:.2f} TFLOP in {cpu['sec']:.1f} s"}
        if not args.no_merge:
            from oracle import ab_oracle as orc
            t0 = time.perf_counter()
            for lay in host_layers[:4]:
                orc.ab_merge(lay["A_copies"], lay["B_copies"], tau=gen.CFG5_TAU_GAP)
            blk_s = time.perf_counter() - t0
            out["cpu_baseline"]["ab_merge_ms_per_layer_set_extrapolated"] = round(blk_s * 12 * 1e3, 1)
            out["cpu_baseline"]["ab_merge_sample"] = "one ViT-B/16 block (4 of the 48 layers) timed, x 12"

    out["bench_seconds"] = round(time.perf_counter() - t_start, 1)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
