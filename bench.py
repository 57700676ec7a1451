"""Benchmark: forward + backward (parameter flows accumulated) of one compiled circuit on one MI355X.

One "step" = pc_forward + pc_backward over one resident batch of the chosen configuration
(default: config 4, the HMM with T=32, H=4096, V=50257, B=256 the MFMA target is quoted on).
Prints ONE JSON line: samples/s, the roofline of the dominant kernel class (per-launch durations
measured with HIP events on the launch stream inside the library) and the CPU oracle's rate on the
host cores as a baseline.  `--gpus N` with N > 1 is refused: this build runs on one GPU.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3      # MI355X dense fp32 matrix peak: 256 CU x 256 flop/clk x 2.4 GHz
PEAK_HBM_GBS = 8000.0              # MI355X HBM3E

# HBM bytes per launch (FETCH_SIZE + WRITE_SIZE, scale factor 1.00) from the rocprofv3 --pmc runs summarised in
# profiles/cfg4_hmm_T32_H4096_B256_hbm_traffic.txt; counters cannot be read from inside this process.
MEASURED_TRAFFIC = {
    ("cfg4_hmm_T32_H4096_V50257_B256", "sum_bwd_child"): (51565.5 + 4096.0) * 1024,
    ("cfg4_hmm_T32_H4096_V50257_B256", "sum_fwd"): (49346.5 + 4128.0) * 1024,
    ("cfg4_hmm_T32_H4096_V50257_B256", "sum_bwd_param"): (957554.9 + 67584.0) * 1024,
}


def algorithmic_work(w):
    """Per-step algorithmic flops / bytes per kernel class (ideal-IO model of Sec. 3: every child value
    read once per consumer block, every output written once; padded and pruned blocks not counted)."""
    import numpy as np
    from paper_2406_00766_amd import workloads as W
    K, B = w.K, w.B
    deg = np.diff(w.child_ptr)
    is_in, is_prod, is_sum = (w.type == W.INPUT), (w.type == W.PRODUCT), (w.type == W.SUM)
    n_par = np.bincount(w.child, minlength=w.n_blocks)
    prod_children = np.zeros(w.n_blocks, dtype=bool)
    for u in np.nonzero(is_prod)[0]:
        prod_children[w.child[w.child_ptr[u]:w.child_ptr[u + 1]]] = True
    Es = w.n_sum_edges()
    row = K * B * 4                                   # bytes of one block row-slab
    work = {
        "sum_fwd": ("TFLOP/s", 2.0 * Es * B),
        "sum_bwd_child": ("TFLOP/s", 2.0 * Es * B),
        "sum_bwd_param": ("TFLOP/s", 2.0 * Es * B),
        "input_fwd": ("GB/s", float(is_in.sum()) * row * 2),
        "input_bwd": ("GB/s", float(is_in.sum()) * row * 3),
        "prod_fwd": ("GB/s", float((deg[is_prod] + 1).sum()) * row),
        "prod_bwd": ("GB/s", float((n_par[prod_children] + 2).sum()) * row),
        "lognf": ("GB/s", float(is_sum.sum()) * row * 3),
    }
    return work, Es


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="4", help="1..5, the configurations of BASELINE.json; 'rat' = the RAT-SPN stand-in")
    ap.add_argument("--batch", type=int, default=None, help="batch size (default per configuration)")
    ap.add_argument("--K", type=int, default=None, help="node block size (default per config)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-em", action="store_true", help="skip the secondary timing that adds pc_em_step")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 256 MiB device-to-device copy kernel (scale reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2406_00766_amd import binding as pcb
    from paper_2406_00766_amd import workloads as W

    t0 = time.time()
    w = W.rat_config(K=args.K, B=args.batch) if args.config == "rat" else W.config(int(args.config), K=args.K, B=args.batch)
    gen_s = time.time() - t0
    work, Es = algorithmic_work(w)

    if args.calibrate_copy:                            # reads 256 MiB, writes 256 MiB: what FETCH_SIZE / WRITE_SIZE are scaled by
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    t0 = time.time()
    c = pcb.Circuit(w, "cuda:0")
    torch.cuda.synchronize()
    compile_s = time.time() - t0
    c.set_batch(w.x)
    B = w.B

    def step():
        c.forward()
        c.backward()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / args.steps
    value = B * args.steps / elapsed

    # same K steps again with per-launch HIP events (on the launch stream, inside the library)
    pcb.pc_profile_enable(c.handle, True)
    for _ in range(args.steps):
        step()
        prof = pcb.pc_profile_read(c.handle)
    pcb.pc_profile_enable(c.handle, False)
    kernels = {}
    for name, (launches, ms) in prof.items():
        if launches == 0:
            continue
        ent = {"launches_per_step": launches / args.steps, "ms_per_step": ms / args.steps,
               "avg_launch_us": 1e3 * ms / launches}
        if name in work:
            unit, amount = work[name]
            rate = amount * args.steps / (ms * 1e-3)
            if unit == "TFLOP/s":
                ent.update(bound="mfma", achieved=rate / 1e12, peak=PEAK_FP32_MFMA_TFLOPS, unit=unit,
                           frac=rate / 1e12 / PEAK_FP32_MFMA_TFLOPS, work_per_launch=amount * args.steps / launches)
            else:
                ent.update(bound="hbm", achieved=rate / 1e9, peak=PEAK_HBM_GBS, unit=unit,
                           frac=rate / 1e9 / PEAK_HBM_GBS, work_per_launch=amount * args.steps / launches)
        kernels[name] = ent
    dom = max((k for k in kernels if "bound" in kernels[k]), key=lambda k: kernels[k]["ms_per_step"])
    d = kernels[dom]
    roofline = {"kernel": dom, "bound": d["bound"], "achieved": d["achieved"], "peak": d["peak"], "unit": d["unit"],
                "frac": d["frac"], "traffic": MEASURED_TRAFFIC.get((w.name, dom)), "avg_launch_us": d["avg_launch_us"],
                "work_per_launch": d["work_per_launch"]}

    em = None
    if not args.no_em:
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
            c.em_step(0.01, 0.0)
        torch.cuda.synchronize()
        em_elapsed = time.perf_counter() - t0
        em = {"samples_per_s": B * args.steps / em_elapsed, "ms_per_step": 1e3 * em_elapsed / args.steps}

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import pc_oracle as orc
        cores = orc.num_threads()
        per_sample_s = 3 * 17e-9 * max(Es, 1)         # three passes over the edges at ~17 ns per edge visit
        n = int(min(B, max(min(B, cores), round(25.0 * cores / per_sample_s))))   # about 25 s of CPU work
        wb = w.with_batch(w.x[:n])
        t0 = time.perf_counter()
        orc.backward(wb, w.theta, w.tables, wb.x)
        dt = time.perf_counter() - t0
        cpu = {"value": n / dt, "unit": "samples/s", "cores": cores, "kind": "oracle",
               "sample": f"first {n} samples of the batch, forward + node flows + parameter flows, {dt:.1f} s"}

    out = {
        "metric": "PC forward+backward samples/sec at 1 MI355X; % of MFMA / HBM roofline",
        "value": value, "unit": "samples/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "structure": w.meta["kind"], "K": w.K, "batch": B, "sum_edges": Es,
                   "n_blocks": w.n_blocks, "n_layers": c.sizes.n_layers},
        "roofline": roofline, "cpu_baseline": cpu, "kernels": kernels, "with_em_step": em,
        "compile_s": compile_s, "generate_s": gen_s,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
