"""Kernel-level benchmark of ONE wide sum layer on one MI355X (App. C.1 / the block-sparse speed-up figure of
Sec. 6.1, and the block-size analysis of Sec. 4.2).

    python -m paper_2406_00766_amd.layer_bench --sweep keep          # 200 sets of 1024 x 1024, K = 32, blocks dropped
    python -m paper_2406_00766_amd.layer_bench --sweep K             # 28 sets of 1024 x 1024 (29 K nodes, 29 M edges), K = 1..128
    python paper_2406_00766_amd/layer_bench.py --sets 28 --K 8 --keep 1 --steps 3      # one point (e.g. under rocprofv3 --pmc)

Every point compiles the layer (wrapped into a small circuit by workloads.sum_layer), runs pc_forward +
pc_backward and prints ONE JSON line with the per-launch durations of the sum-layer kernels (HIP events on the
launch stream, read through pc_profile_read).  The kernel classes also hold the root layer's launches: one block
row with M / K child blocks, a few microseconds.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:                     # also runnable as a script from any directory (e.g. under rocprofv3)
    sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3


def run_point(n_sets, M, K, keep, B, steps, warmup, seed):
    import torch
    from paper_2406_00766_amd import binding as pcb
    from paper_2406_00766_amd import workloads as W

    w = W.sum_layer(n_sets, M, K, B, seed, keep=keep)
    t0 = time.time()
    c = pcb.Circuit(w, "cuda:0")
    torch.cuda.synchronize()
    compile_s = time.time() - t0
    c.set_batch(w.x)
    for _ in range(warmup):
        c.forward()
        c.backward()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        c.forward()
        c.backward()
    torch.cuda.synchronize()
    step_ms = 1e3 * (time.perf_counter() - t0) / steps
    pcb.pc_profile_enable(c.handle, True)
    for _ in range(steps):
        c.forward()
        c.backward()
    prof = pcb.pc_profile_read(c.handle)
    pcb.pc_profile_enable(c.handle, False)
    edges = w.meta["n_layer_edges"]
    flop = 2.0 * edges * B
    out = {"workload": w.name, "K": K, "keep": keep, "batch": B, "layer_edges": edges,
           "kept_fraction": edges / float(n_sets * M * M), "step_ms": step_ms, "compile_s": compile_s}
    for name in ("sum_fwd", "sum_bwd_child", "sum_bwd_param"):
        launches, ms = prof[name]
        per_step = ms / steps
        out[name] = {"ms_per_step": per_step, "launches_per_step": launches / steps,
                     "tflops": flop / (per_step * 1e-3) / 1e12,
                     "frac_fp32_mfma_peak": flop / (per_step * 1e-3) / 1e12 / PEAK_FP32_MFMA_TFLOPS}
    c.close()
    del c
    torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--sweep", choices=["keep", "K"], default=None)
    ap.add_argument("--sets", type=int, default=None)
    ap.add_argument("--M", type=int, default=1024)
    ap.add_argument("--K", type=int, default=32)
    ap.add_argument("--keep", type=float, default=1.0)
    ap.add_argument("--B", type=int, default=512)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--seed", type=int, default=240600766 + 7)
    args = ap.parse_args()

    if args.sweep == "keep":
        points = [(args.sets or 200, args.M, 32, k) for k in (1.0, 0.8, 0.6, 0.4, 0.2, 0.1, 0.05, 0.02)]
    elif args.sweep == "K":
        points = [(args.sets or 28, args.M, k, 1.0) for k in (1, 2, 4, 8, 16, 32, 64, 128)]
    else:
        points = [(args.sets or 200, args.M, args.K, args.keep)]
    for n_sets, M, K, keep in points:
        print(f"# point sets={n_sets} M={M} K={K} keep={keep}", file=sys.stderr, flush=True)
        print(json.dumps(run_point(n_sets, M, K, keep, args.B, args.steps, args.warmup, args.seed)), flush=True)


if __name__ == "__main__":
    main()
