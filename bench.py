#!/usr/bin/env python3
"""Benchmark of the AdaPM optimizer step on one MI355X.

A "step" is one pass of the whole hot path (blockwise v statistics, full-momentum update,
low-rank momentum with bias correction, fused parameter update) over every block of the
GPT-2-1.5B-shaped table, on synthetic low-rank-plus-tail gradients already resident in HBM.

Default: refresh period T = 100 (the paper's experimental setting), K = 100 timed steps after
W = 3 warm-up steps, so the timed region holds exactly one step that runs Alg. 2 and 99 steps
with R held: `value` is the T-amortised throughput.  The literal Alg. 1 (T = 1, Alg. 2 every
step) is timed separately and reported in `literal_T1`.

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

    def run(opt, t0, nsteps):
        for i in range(nsteps):
            t = t0 + i
            opt.step(params, grad_sets[t % len(grad_sets)], t, lr)

    opt = make(args.T)
    K, W = args.steps, args.warmup
    run(opt, 1, W)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t_host0 = time.perf_counter()
    e0.record()
    run(opt, W + 1, K)
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t_host0) * 1e3
    dev_ms = e0.elapsed_time(e1)
    ms_per_step = wall_ms / K
    n_refresh = sum(1 for t in range(W + 1, W + K + 1) if args.T <= 1 or (t - 1) % args.T == 0)

    # per-kernel durations over an identical region, from HIP events around every launch
    B.adapm_profile_enable(opt.ctx, True)
    run(opt, W + K + 1, K)
    torch.cuda.synchronize()
    prof = B.adapm_profile_read(opt.ctx)
    B.adapm_profile_enable(opt.ctx, False)
    n_refresh_prof = sum(1 for t in range(W + K + 1, W + 2 * K + 1) if args.T <= 1 or (t - 1) % args.T == 0)
    kernels = {k: {"avg_ms": v[0] / v[1], "launches": v[1], "total_ms": v[0]} for k, v in prof.items()}
    dominant = max(kernels, key=lambda k: kernels[k]["total_ms"])

    lr_blocks = [b for b in wl.blocks if b.mom == "lowrank"]
    full_blocks = [b for b in wl.blocks if b.mom != "lowrank"]
    if dominant.startswith("fused_project"):
        rank = int(dominant.split("_r")[-1])
        # the kernel of a rank class serves every rank up to it (32, 64, 128)
        alg = sum(block_bytes(b, False) for b in lr_blocks if min(c for c in (32, 64, 128) if b.rank <= c) == rank)
        roof = {"bound": "hbm", "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "achieved": alg / (kernels[dominant]["avg_ms"] * 1e-3) / 1e9}
    elif dominant == "update_full":
        alg = sum(block_bytes(b, False) for b in full_blocks)
        roof = {"bound": "hbm", "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "achieved": alg / (kernels[dominant]["avg_ms"] * 1e-3) / 1e9}
    else:
        # a contraction kernel of Alg. 2: flops of one launch (products counted once, not per bf16 split)
        per_launch = B.adapm_algorithmic_flops(opt.ctx, True) / max(1, kernels[dominant]["launches"] // max(1, n_refresh_prof))
        roof = {"bound": "mfma", "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "achieved": per_launch / (kernels[dominant]["avg_ms"] * 1e-3) / 1e12}
    traffic = None
    tfile = os.path.join(ROOT, "profiles", "hbm_traffic_per_launch.txt")
    if args.workload == "gpt2_1p5b" and args.T == 100 and args.rank == 0 and os.path.exists(tfile):
        for line in open(tfile):
            parts = line.split()
            if len(parts) == 2 and parts[0] == dominant:
                traffic = float(parts[1])
    roof.update(kernel=dominant, frac=roof["achieved"] / roof["peak"], traffic=traffic,
                avg_ms=kernels[dominant]["avg_ms"])

    bytes_refresh = B.adapm_algorithmic_bytes(opt.ctx, True)
    bytes_held = B.adapm_algorithmic_bytes(opt.ctx, False)
    step_bytes = (n_refresh * bytes_refresh + (K - n_refresh) * bytes_held) / K
    launches_held = B.adapm_last_launch_count(opt.ctx)
    state_bytes, ws_bytes = opt.state_bytes, opt.workspace_bytes
    opt.close()
    del opt
    torch.cuda.empty_cache()

    literal = None
    if not args.no_literal and args.T != 1:
        o1 = make(1)
        run(o1, 1, 1)
        torch.cuda.synchronize()
        n1 = 5
        t0 = time.perf_counter()
        run(o1, 2, n1)
        torch.cuda.synchronize()
        ms1 = (time.perf_counter() - t0) * 1e3 / n1
        fl = B.adapm_algorithmic_flops(o1.ctx, True)
        literal = {"ms_per_step": ms1, "params_per_s": wl.numel / (ms1 * 1e-3), "steps": n1,
                   "contraction_TFLOPs": fl / (ms1 * 1e-3) / 1e12, "launches_per_step": B.adapm_last_launch_count(o1.ctx),
                   "algorithmic_GBs": B.adapm_algorithmic_bytes(o1.ctx, True) / (ms1 * 1e-3) / 1e9}
        o1.close()
        del o1
        torch.cuda.empty_cache()

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
                   "refresh_steps_in_timed_region": n_refresh, "rank": max([b.rank for b in wl.blocks] + [0]),
                   "second_moment": "blockwise" if any(b.v_mode != "element" for b in wl.blocks) else "element",
                   "grad_sets_rotated": len(grad_sets), "global_grad_clip": args.grad_clip},
        "device_ms_per_step": dev_ms / K,
        "achieved_algorithmic_GBs": step_bytes / (ms_per_step * 1e-3) / 1e9,
        "algorithmic_bytes_per_step": step_bytes,
        "hbm_frac_whole_step": step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "launches_per_held_step": launches_held,
        "state_bytes": state_bytes, "workspace_bytes": ws_bytes,
        "roofline": roof,
        "kernels": kernels,
        "literal_T1": literal,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, args.T, lr)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
