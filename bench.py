#!/usr/bin/env python3
"""Benchmark of the AdaPM optimizer step on one MI355X.

A "step" is one pass of the whole hot path (blockwise v statistics, full-momentum update,
low-rank momentum with bias correction, fused parameter update) over every block of the
GPT-2-1.5B-shaped table, on synthetic low-rank-plus-tail gradients already resident in HBM.

Default: refresh period T = 100 (the paper's experimental setting).  Whatever --steps K and
--warmup W are, the K timed steps open with a step that runs Alg. 2 (its step number is put on
the refresh grid) and continue with steps that hold R; every step is bracketed by HIP events,
and `value` is the T-amortised throughput params / ((t_refresh + (T-1) t_held) / T).  The
literal Alg. 1 (T = 1, Alg. 2 every step: the only reading the paper pins) is timed separately,
with its own roofline block, and reported in `literal_T1`.

Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16
FP64_VECTOR_PEAK_TFLOPS = 78.6  # fp64 vector arithmetic (the exact path's products run as fp64 fused multiply-adds)


def block_bytes(b, refresh):
    """compulsory bytes of one block in one step: inputs once, outputs once, storage types."""
    ge = {"f32": 4, "bf16": 2}
    mn = b.rows * b.cols
    tot = mn * (ge[b.grad_dtype] + 2 * ge[b.param_dtype])
    nv = mn if b.v_mode == "element" else (b.rows // b.v_group_rows if b.v_mode == "rowgroup" else 1)
    tot += 8 * nv
    if b.mom == "full":
        tot += 8 * mn
    if b.mom == "lowrank":
        tot += 8 * (b.rows + b.cols) * b.rank if refresh else (8 * b.rows + 4 * b.cols) * b.rank
    return tot


def cpu_baseline(wl, T, lr, nlayers=6, held_steps=3):
    """The oracle, as it stands, on the first transformer layers of the workload (blocks are independent):
    one step that runs Alg. 2 and a few steps with R held, combined with the same T weighting.  Sized to
    10 - 30 s of CPU work at the GPT-2-1.5B shape."""
    import numpy as np
    import torch
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from oracle import adapm_oracle as O
    from parity_util import oracle_block, to_np
    from paper_2510_09103_amd import workloads as WL
    layers = sorted({b.name.split(".")[0] for b in wl.blocks if "." in b.name},
                    key=lambda s: (len(s), s))[:nlayers]
    sub = WL.subset(wl, [b.name for b in wl.blocks if b.name.split(".")[0] in layers and "." in b.name])
    blocks = [oracle_block(b) for b in sub.blocks]
    hp = O.HParams(beta1=wl.beta1, beta2=wl.beta2, eps=wl.eps, clip=wl.clip, K=wl.K, T=T)
    state = O.init_state(blocks, hp)
    Ws = [to_np(p) for p in WL.initial_params(sub, device="cpu")]
    stream = WL.GradientStream(sub, device="cpu")
    times = []
    for t in range(1, 2 + (held_steps if T > 1 else 0)):
        G = [to_np(g) for g in stream.next()]
        t0 = time.perf_counter()
        Ws, state = O.step(blocks, hp, Ws, G, state, t, lr)
        times.append(time.perf_counter() - t0)
    held = sum(times[1:]) / max(len(times) - 1, 1)
    per_step = times[0] if T <= 1 else (times[0] + (T - 1) * held) / T
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    return {
        "value": sub.numel / per_step, "unit": "params/s", "cores": int(threads), "kind": "oracle",
        "sample": (f"numpy fp64 oracle on the {len(sub.blocks)} blocks of layers {', '.join(layers)} ({sub.numel} params), "
                   f"{sum(times):.1f} s of CPU work: step with Alg. 2 {times[0]:.2f} s"
                   + (f", mean of {len(times) - 1} held-R steps {held:.2f} s, weighted 1:{T - 1}" if T > 1 else "")),
        "host_cpus": os.cpu_count(),
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--T", type=int, default=100, help="refresh period (1 = Alg. 2 every step)")
    ap.add_argument("--workload", default="gpt2_1p5b")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-literal", action="store_true")
    ap.add_argument("--grad-sets", type=int, default=2)
    ap.add_argument("--grad-clip", type=float, default=0.0, help="global gradient-norm clipping threshold (0 = off)")
    ap.add_argument("--rank", type=int, default=0, help="override the rank of every low-rank block (rank / T sweeps)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU (blocks are independent, the library has no collectives); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    if args.T > 1 and args.steps < 2:
        print("bench.py: with a refresh period T > 1 the timed region needs --steps >= 2: its first step runs Alg. 2, "
              "the others hold R, and the value weighs the two kinds 1 : T - 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2510_09103_amd import binding as B
    from paper_2510_09103_amd import workloads as WL
    from paper_2510_09103_amd.optimizer import AdaPM, make_hparams

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    wl = WL.CONFIGS[args.workload]()
    if args.rank > 0:
        from dataclasses import replace
        wl = replace(wl, blocks=tuple(replace(b, rank=min(args.rank, b.rows, b.cols)) if b.mom == "lowrank" else b
                                      for b in wl.blocks))
    lr = wl.lr
    params = WL.initial_params(wl, device=dev)
    stream = WL.GradientStream(wl, device=dev)
    grad_sets = [stream.next() for _ in range(args.grad_sets)]
    del stream
    torch.cuda.synchronize()

    def make(T):
        return AdaPM(wl.blocks, make_hparams(beta1=wl.beta1, beta2=wl.beta2, eps=wl.eps, clip=wl.clip, K=wl.K, T=T),
                     device=dev, grad_clip=args.grad_clip)

    def schedule(T, n, after):
        """Step numbers of a region of n steps: with T > 1 the region opens with a step that runs Alg. 2 (the first
        one on the refresh grid after `after`) and continues with steps that hold R, so that both kinds are timed
        whatever n is; with T = 1 every step runs Alg. 2.  The library takes the step number as an argument."""
        if T <= 1:
            return list(range(after + 1, after + n + 1))
        first = ((after + T - 1) // T) * T + 1
        return [first + i for i in range(n)]

    def timed(opt, steps):
        """Run the steps back to back; returns (wall ms of the whole region, per-step device ms from HIP events
        recorded between the steps on the stream the library launches on: torch's current stream)."""
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(len(steps) + 1)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i, t in enumerate(steps):
            ev[i].record()
            opt.step(params, grad_sets[t % len(grad_sets)], t, lr)
        ev[-1].record()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) * 1e3
        return wall, [ev[i].elapsed_time(ev[i + 1]) for i in range(len(steps))]

    def kernel_profile(opt, steps, T):
        """Per-kernel durations from HIP events that the library records around every launch, over the same kind of
        region.  Returns {label: {avg_ms, launches, total_ms, per_step_ms}}: per_step_ms is the kernel's share of a
        T-amortised step (kernels of steps that run Alg. 2 weigh 1/T)."""
        B.adapm_profile_enable(opt.ctx, True)
        out = {}
        n_ref = sum(1 for t in steps if T <= 1 or (t - 1) % T == 0)
        n_held = len(steps) - n_ref
        for kind, sel in (("refresh", [t for t in steps if T <= 1 or (t - 1) % T == 0]),
                          ("held", [t for t in steps if not (T <= 1 or (t - 1) % T == 0)])):
            if not sel:
                continue
            for t in sel:
                opt.step(params, grad_sets[t % len(grad_sets)], t, lr)
            torch.cuda.synchronize()
            w = (1.0 / T if T > 1 else 1.0) if kind == "refresh" else (T - 1.0) / T
            for k, (ms, cnt) in B.adapm_profile_read(opt.ctx).items():
                d = out.setdefault(k, {"total_ms": 0.0, "launches": 0, "per_step_ms": 0.0, "step_ms": 0.0})
                d["total_ms"] += ms
                d["launches"] += cnt
                d["per_step_ms"] += w * ms / len(sel)
                d["step_ms"] = ms / len(sel)          # per step of the kind the kernel runs in
                d["launches_per_step"] = cnt / len(sel)
        B.adapm_profile_enable(opt.ctx, False)
        for d in out.values():
            d["avg_ms"] = d["total_ms"] / d["launches"]
        return out, n_ref, n_held

    lr_blocks = [b for b in wl.blocks if b.mom == "lowrank"]
    full_blocks = [b for b in wl.blocks if b.mom != "lowrank"]

    def rank_class(b):
        return min(c for c in (32, 64, 128) if b.rank <= c) if b.rank <= 128 else 0

    n_gd = sum(1 for k_ in range(1, wl.K + 1) if k_ != wl.K)      # iterations of Alg. 2 with a non-zero step (eta_K = 0)

    def roofline_of(label, k, refresh_step):
        """Roofline block of one kernel class: algorithmic bytes (HBM-bound kernels) or flops (the contractions of
        Alg. 2) of one pass of the class over all of its blocks, over the live duration of that pass.  A pass is one
        launch, or one launch per group of blocks where Alg. 2 runs group by group; the stripe kernels make one pass
        per GD iteration."""
        roof = None
        passes = n_gd if label.startswith("alg2_") else 1
        k = dict(k, avg_ms=k["step_ms"] / passes, launches_per_pass=k["launches_per_step"] / passes)
        if label.startswith("fused_project") or label.startswith("fused_refresh_update"):
            rank = int(label.split("_r")[-1])
            alg = sum(block_bytes(b, refresh_step) for b in lr_blocks if rank_class(b) == rank)
            if label.startswith("fused_refresh_update"):
                # the update after Alg. 2 reads G, W, v and both factor pairs and writes W: the factors' own write is
                # the stripes' business
                alg = sum(b.rows * b.cols * 6 + 8 * (b.rows + b.cols) * b.rank for b in lr_blocks if rank_class(b) == rank)
            roof = {"bound": "hbm", "peak": HBM_PEAK_GBS, "unit": "GB/s", "achieved": alg / (k["avg_ms"] * 1e-3) / 1e9}
        elif label in ("update_full", "update_full_grouped"):
            alg = sum(block_bytes(b, False) for b in full_blocks)
            roof = {"bound": "hbm", "peak": HBM_PEAK_GBS, "unit": "GB/s", "achieved": alg / (k["avg_ms"] * 1e-3) / 1e9}
        elif label.startswith("alg2_stripe_step"):
            # one launch = one of the two streaming products of a GD iteration over every block of a rank class
            # (G R^T or G^T L: 2 m n r flop) and the thin products of the GD step behind it (2 x 2 d r^2, d = m or n)
            rank = int(label.split("_r")[-1])
            side_L = "_L_" in label
            blocks = [b for b in lr_blocks if rank_class(b) == rank]
            alg = sum(2.0 * b.rows * b.cols * b.rank + 4.0 * (b.rows if side_L else b.cols) * b.rank ** 2 for b in blocks)
            issued = sum(2 * 2.0 * b.rows * b.cols * rank + 3 * 4.0 * (b.rows if side_L else b.cols) * rank ** 2 for b in blocks)
            alg_bytes = sum(b.rows * b.cols * 2 + 12 * (b.rows if side_L else b.cols) * b.rank for b in blocks)
            sec = k["avg_ms"] * 1e-3
            # arithmetic intensity (about 110 flop per byte at r = 128, 220 as issued) is below the machine balance
            # (2.5 PFLOP/s / 8 TB/s = 312 flop per byte): HBM is the nearer roof; the matrix-core figures ride along
            roof = {"bound": "hbm", "peak": HBM_PEAK_GBS, "unit": "GB/s", "achieved": alg_bytes / sec / 1e9,
                    "flop_per_byte": alg / alg_bytes,
                    "mfma": {"peak_TFLOPs": MFMA_BF16_PEAK_TFLOPS, "achieved_TFLOPs": alg / sec / 1e12,
                             "frac": alg / sec / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                             "issued_TFLOPs": issued / sec / 1e12,
                             "issued_frac": issued / sec / 1e12 / MFMA_BF16_PEAK_TFLOPS},
                    "note": "bytes: G once plus the factor it updates (current and previous read, new written: fp32); mfma.achieved = "
                            "flops of the mathematical products; mfma.issued = matrix-core work with every fp32 "
                            "operand as a (hi, lo) bf16 pair (2 instructions per product of G, 3 per thin product) "
                            "at the padded rank class"}
        elif label in ("project_f64", "reconstruct_f64", "alg2_products_f64"):
            # exact path: batched fp64 products on the vector units.  project: G Q^T; reconstruct: the m x n term of
            # the update from the thin factors; Alg. 2: G R^T and L^T G per GD iteration (plus the r x r ones)
            per_block = {"project_f64": lambda b: 2.0 * b.rows * b.cols * b.rank,
                         "reconstruct_f64": lambda b: 2.0 * b.rows * b.cols * b.rank,
                         "alg2_products_f64": lambda b: 4.0 * b.rows * b.cols * b.rank + 8.0 * (b.rows + b.cols) * b.rank ** 2}[label]
            alg = sum(per_block(b) for b in lr_blocks)
            roof = {"bound": "alu", "peak": FP64_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "achieved": alg / (k["avg_ms"] * 1e-3) / 1e12,
                    "note": "fp64 multiply-adds of the products, against the chip's fp64 vector rate (256 compute units x "
                            "4 SIMDs x 16 lanes x 2 flop x 2.4 GHz = 78.6 TFLOP/s)"}
        if roof is None:
            return None
        roof.update(kernel=label, frac=roof["achieved"] / roof["peak"], avg_ms=k["avg_ms"],
                    launches_per_pass=k["launches_per_pass"], traffic=None)
        return roof

    opt = make(args.T)
    K, W = args.steps, args.warmup
    for t in range(1, W + 1):
        opt.step(params, grad_sets[t % len(grad_sets)], t, lr)
    steps = schedule(args.T, K, W)
    wall_ms, per_step = timed(opt, steps)
    is_ref = [args.T <= 1 or (t - 1) % args.T == 0 for t in steps]
    n_refresh = sum(is_ref)
    t_ref = sum(d for d, r in zip(per_step, is_ref) if r) / max(n_refresh, 1)
    t_held = sum(d for d, r in zip(per_step, is_ref) if not r) / max(K - n_refresh, 1) if K > n_refresh else t_ref
    # T-amortised step: one step in T runs Alg. 2 (with the re-expression of the factors), T - 1 hold R
    ms_per_step = t_ref if args.T <= 1 else (t_ref + (args.T - 1) * t_held) / args.T

    kernels, n_refresh_prof, _ = kernel_profile(opt, schedule(args.T, K, steps[-1]), args.T)
    dominant = max(kernels, key=lambda k: kernels[k]["per_step_ms"])
    roof = roofline_of(dominant, kernels[dominant], args.T <= 1)
    if roof is None:
        roof = {"bound": "alu", "kernel": dominant, "avg_ms": kernels[dominant]["avg_ms"], "achieved": None, "peak": None,
                "unit": None, "frac": None, "traffic": None}
    def counter_traffic(roof_block, T):
        """HBM bytes per pass of the block's kernel from the committed counter summary (not a measurement of this run)."""
        tfile = os.path.join(ROOT, "profiles", "hbm_traffic_per_launch.txt")
        roof_block["traffic_source"] = None
        if args.rank != 0 or not os.path.exists(tfile):
            return
        for line in open(tfile):
            parts = line.split()
            if len(parts) == 4 and parts[0] == args.workload and parts[1] == f"T{T}" and parts[2] == roof_block["kernel"]:
                roof_block["traffic"] = float(parts[3])
                roof_block["traffic_source"] = ("profiles/hbm_traffic_per_launch.txt: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE "
                                                "of this command on an earlier run, not of this run")

    counter_traffic(roof, args.T)

    bytes_refresh = B.adapm_algorithmic_bytes(opt.ctx, True)
    bytes_held = B.adapm_algorithmic_bytes(opt.ctx, False)
    step_bytes = bytes_refresh if args.T <= 1 else (bytes_refresh + (args.T - 1) * bytes_held) / args.T
    launches_held = B.adapm_last_launch_count(opt.ctx)
    state_bytes, ws_bytes = opt.state_bytes, opt.workspace_bytes
    opt.close()
    del opt
    torch.cuda.empty_cache()

    literal = None
    if not args.no_literal and args.T != 1:
        o1 = make(1)
        for t in range(1, 4):                      # three warm-up steps
            o1.step(params, grad_sets[t % len(grad_sets)], t, lr)
        n1 = 5
        wall1, per1 = timed(o1, schedule(1, n1, 3))
        ms1 = sum(per1) / n1
        k1, _, _ = kernel_profile(o1, schedule(1, 3, 3 + n1), 1)
        dom1 = max(k1, key=lambda k: k1[k]["per_step_ms"])
        fl = B.adapm_algorithmic_flops(o1.ctx, True)
        stripe_ms = sum(v["per_step_ms"] for k, v in k1.items() if k.startswith("alg2_stripe_step"))
        literal = {"ms_per_step": ms1, "wall_ms_per_step": wall1 / n1, "params_per_s": wl.numel / (ms1 * 1e-3), "steps": n1,
                   "warmup": 3, "contraction_TFLOPs": fl / (ms1 * 1e-3) / 1e12,
                   "launches_per_step": B.adapm_last_launch_count(o1.ctx),
                   "algorithmic_GBs": B.adapm_algorithmic_bytes(o1.ctx, True) / (ms1 * 1e-3) / 1e9,
                   "hbm_frac_whole_step": B.adapm_algorithmic_bytes(o1.ctx, True) / (ms1 * 1e-3) / 1e9 / HBM_PEAK_GBS,
                   "mfma_frac_whole_step": fl / (ms1 * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                   "roofline": roofline_of(dom1, k1[dom1], True),   # counter traffic added below
                   "kernels_ms_per_step": {k: v["per_step_ms"] for k, v in k1.items()},
                   "stripe_products_ms_per_step": stripe_ms,
                   "workspace_bytes": o1.workspace_bytes}
        if literal["roofline"] is not None:
            counter_traffic(literal["roofline"], 1)
        o1.close()
        del o1
        torch.cuda.empty_cache()

    adam_bytes = 8 * wl.numel
    out = {
        "metric": "AdaPM optimizer-step throughput at GPT-2-1.5B shape" if args.workload == "gpt2_1p5b"
                  else f"AdaPM optimizer-step throughput ({args.workload})",
        "value": wl.numel / (ms_per_step * 1e-3), "unit": "params/s",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32",
        "precision_note": "fp32 arithmetic and state; bf16 parameters and gradients; contractions on bf16 MFMA with every "
                          "fp32 operand as a (hi, lo) bf16 pair, fp32 accumulation",
        "data": "synthetic",
        "config": {"workload": args.workload, "blocks": len(wl.blocks), "params": wl.numel, "refresh_period_T": args.T,
                   "refresh_steps_in_timed_region": n_refresh, "timed_step_numbers": [steps[0], steps[-1]],
                   "rank": max([b.rank for b in wl.blocks] + [0]),
                   "second_moment": "blockwise" if any(b.v_mode != "element" for b in wl.blocks) else "element",
                   "grad_sets_rotated": len(grad_sets), "global_grad_clip": args.grad_clip},
        "value_definition": ("T-amortised step: (t_refresh + (T-1) t_held) / T, both legs timed by HIP events inside the "
                             "timed region (its first step runs Alg. 2, the others hold R)" if args.T > 1 else
                             "Alg. 1 as printed: Alg. 2 in every step"),
        "reading_note": ("the step that holds R between two runs of Alg. 2 is this build's reading of the paper's "
                         "undefined 'update frequency T'; the paper pins only T = 1 (literal_T1)" if args.T > 1 else None),
        "refresh_step_ms": t_ref, "held_step_ms": t_held if args.T > 1 else None,
        "timed_region_wall_ms_per_step": wall_ms / K,
        "achieved_algorithmic_GBs": step_bytes / (ms_per_step * 1e-3) / 1e9,
        "algorithmic_bytes_per_step": step_bytes,
        "hbm_frac_whole_step": step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "launches_per_held_step": launches_held,
        "memory": {"state_bytes": state_bytes, "workspace_bytes": ws_bytes, "state_plus_workspace_bytes": state_bytes + ws_bytes,
                   "adam_two_moments_bytes": adam_bytes, "state_over_adam": state_bytes / adam_bytes,
                   "state_plus_workspace_over_adam": (state_bytes + ws_bytes) / adam_bytes,
                   "paper_table2_note": "Table 2 (GPT-2-1.5B, the paper's own partition): Adam 12.48 G, AdaPM 6.98 G, "
                                        "AdaPM-mini 0.74 G; this workload is BASELINE's config (r = 128 on every matrix)"},
        "roofline": roof,
        "kernels": kernels,
        "literal_T1": literal,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, args.T, lr)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
