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
PEAK_BF16_MFMA_TFLOPS = 2500.0     # MI355X dense bf16 matrix peak
PEAK_HBM_GBS = 8000.0              # MI355X HBM3E

def longest_path_depth(w):
    """Depth of every block (inputs 0, else 1 + the deepest child): the layering of Sec. 3, recomputed here only to
    count bytes per launch (one launch per product layer)."""
    import numpy as np
    n = w.n_blocks
    depth = np.zeros(n, dtype=np.int64)
    n_par = np.bincount(w.child, minlength=n)
    parents_ptr = np.concatenate([[0], np.cumsum(n_par)])
    fill = parents_ptr[:-1].copy()
    parents = np.empty(len(w.child), dtype=np.int64)
    src = np.repeat(np.arange(n), np.diff(w.child_ptr))
    for e, c in enumerate(w.child):
        parents[fill[c]] = src[e]
        fill[c] += 1
    pending = np.diff(w.child_ptr).astype(np.int64)
    ready = [u for u in range(n) if pending[u] == 0]
    while ready:
        u = ready.pop()
        for p in parents[parents_ptr[u]:parents_ptr[u + 1]]:
            depth[p] = max(depth[p], depth[u] + 1)
            pending[p] -= 1
            if pending[p] == 0:
                ready.append(p)
    return depth, parents_ptr, parents


def algorithmic_work(w):
    """Per-step algorithmic work per kernel class.

    Sum kernels: 2 E_s B flops each.  HBM-bound kernels: the COMPULSORY HBM bytes of the ideal-IO model of Sec. 3
    applied per launch -- every distinct row a launch needs is read from HBM once (a row read by several workgroups of
    one launch is served by L2 after the first), every output row is written once.  The second figure, `per_consumer`,
    charges a row once per block that reads it (what the L2 <-> CU side moves)."""
    import numpy as np
    from paper_2406_00766_amd import workloads as W
    K, B = w.K, w.B
    deg = np.diff(w.child_ptr)
    is_in, is_prod, is_sum = (w.type == W.INPUT), (w.type == W.PRODUCT), (w.type == W.SUM)
    n_par = np.bincount(w.child, minlength=w.n_blocks)
    depth, pptr, parents = longest_path_depth(w)
    Es = w.n_sum_edges()
    row = K * B * 4                                   # bytes of one block's rows
    # product layers: one launch per depth
    prod_fwd = prod_bwd = 0.0
    prod_children = np.zeros(w.n_blocks, dtype=bool)
    for d in np.unique(depth[is_prod]):
        prods = np.nonzero(is_prod & (depth == d))[0]
        ch = np.unique(np.concatenate([w.child[w.child_ptr[u]:w.child_ptr[u + 1]] for u in prods]))
        prod_children[ch] = True
        prod_fwd += (len(ch) + len(prods)) * row      # distinct child rows in, product rows out
        # backward: parent flows in, child flows out; a child fed before by a deeper layer is read first; where the
        # flow of a sum child becomes final its log-probabilities are read and log F - l is written as well
        pd = [depth[parents[pptr[c]:pptr[c + 1]]] for c in ch]
        not_first = sum(1 for x in pd if x.max() > d)
        final_sum = sum(1 for c, x in zip(ch, pd) if is_sum[c] and x.min() == d)
        prod_bwd += (len(prods) + len(ch) + not_first + 2 * final_sum) * row
    # input layer: distinct (table, category) rows of K floats
    in_blocks = np.nonzero(is_in)[0]
    vars_of_table, cats_of_var = {}, {}
    for t, v in zip(w.in_table[in_blocks].tolist(), w.in_var[in_blocks].tolist()):
        vars_of_table.setdefault(t, set()).add(v)
    n_tab_rows = 0
    for t, vs in vars_of_table.items():
        cats = set()
        for v in vs:
            if v not in cats_of_var:
                cats_of_var[v] = set(np.unique(w.x[:, v]).tolist())
            cats |= cats_of_var[v]
        n_tab_rows += len(cats)
    tab_bytes = n_tab_rows * K * 4                    # a table is [n_cats][K]: K floats per category that occurs
    n_in = float(is_in.sum())
    work = {
        "sum_fwd": ("TFLOP/s", 2.0 * Es * B, None),
        "sum_bwd_child": ("TFLOP/s", 2.0 * Es * B, None),
        "sum_bwd_param": ("TFLOP/s", 2.0 * Es * B, None),
        "input_fwd": ("GB/s", n_in * row + tab_bytes, n_in * row * 2),
        "input_bwd": ("GB/s", n_in * row + 2 * tab_bytes, n_in * row * 3),
        "prod_fwd": ("GB/s", prod_fwd, float((deg[is_prod] + 1).sum()) * row),
        "prod_bwd": ("GB/s", prod_bwd, float((n_par[prod_children] + 2).sum()) * row),
    }
    return work, Es


def measured_traffic(w, kernel_class):
    """HBM bytes per launch of a kernel class from the committed rocprofv3 counter summary of this workload
    (FETCH_SIZE + WRITE_SIZE), or None when there is none for this workload and block size."""
    from paper_2406_00766_amd import profile_summary as ps
    path = os.path.join(ROOT, "profiles", f"{w.name}_K{w.K}_hbm_traffic.txt")
    if not os.path.exists(path):
        return None, None
    head, per = ps.read_counters(path)
    if head.get("workload") != w.name or head.get("K") != str(w.K) or kernel_class not in per:
        return None, None
    return per[kernel_class].get("hbm_bytes_per_launch"), os.path.relpath(path, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="4", help="1..5, the configurations of BASELINE.json; 'rat' = the RAT-SPN stand-in")
    ap.add_argument("--batch", type=int, default=None, help="batch size (default per configuration)")
    ap.add_argument("--K", type=int, default=None, help="node block size (default per config)")
    ap.add_argument("--product-scratch", action="store_true",
                    help="compile in the memory-saving mode of Sec. 5 (product values in one scratch window, recomputed in the backward pass)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-em", action="store_true", help="skip the secondary timing that adds pc_em_step")
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
    if args.product_scratch:
        w = pcb.pc_order_for_scratch(w)
    gen_s = time.time() - t0
    work, Es = algorithmic_work(w)

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
        prof = pcb.pc_profile_read(c.handle, with_bf16=True)
    pcb.pc_profile_enable(c.handle, False)
    kernels = {}
    any_bf16 = False
    for name, (launches, ms, bf16_launches) in prof.items():
        if launches == 0:
            continue
        ent = {"launches_per_step": launches / args.steps, "ms_per_step": ms / args.steps,
               "avg_launch_us": 1e3 * ms / launches}
        if name in work:
            unit, amount, per_consumer = work[name]
            rate = amount * args.steps / (ms * 1e-3)
            if unit == "TFLOP/s" and 2 * bf16_launches >= launches:
                # most launches of the class run as bf16-split products (three bf16 MFMAs per fp32 product): the
                # roofline is the bf16 one with 3x the flops; the fp32-equivalent rate is kept beside it
                any_bf16 = True
                ent.update(bound="mfma", mfma_dtype="bf16x3", achieved=3 * rate / 1e12, peak=PEAK_BF16_MFMA_TFLOPS, unit=unit,
                           frac=3 * rate / 1e12 / PEAK_BF16_MFMA_TFLOPS, work_per_launch=3 * amount * args.steps / launches,
                           fp32_equivalent_tflops=rate / 1e12, fp32_equivalent_frac_of_fp32_peak=rate / 1e12 / PEAK_FP32_MFMA_TFLOPS,
                           bf16_launches_per_step=bf16_launches / args.steps)
            elif unit == "TFLOP/s":
                ent.update(bound="mfma", mfma_dtype="f32", achieved=rate / 1e12, peak=PEAK_FP32_MFMA_TFLOPS, unit=unit,
                           frac=rate / 1e12 / PEAK_FP32_MFMA_TFLOPS, work_per_launch=amount * args.steps / launches)
            else:
                ent.update(bound="hbm", achieved=rate / 1e9, peak=PEAK_HBM_GBS, unit=unit,
                           frac=rate / 1e9 / PEAK_HBM_GBS, work_per_launch=amount * args.steps / launches,
                           per_consumer_gbs=per_consumer * args.steps / (ms * 1e-3) / 1e9)
        kernels[name] = ent
    dom = max((k for k in kernels if "bound" in kernels[k]), key=lambda k: kernels[k]["ms_per_step"])
    d = kernels[dom]
    traffic, traffic_file = measured_traffic(w, dom)
    roofline = {"kernel": dom, "bound": d["bound"], "achieved": d["achieved"], "peak": d["peak"], "unit": d["unit"],
                "frac": d["frac"], "traffic": traffic, "traffic_source": traffic_file, "avg_launch_us": d["avg_launch_us"],
                "work_per_launch": d["work_per_launch"]}
    for k in ("mfma_dtype", "fp32_equivalent_tflops", "fp32_equivalent_frac_of_fp32_peak"):
        if k in d:
            roofline[k] = d[k]

    # achievable peaks of this device beside the published ones: a plain streaming copy and a register-only MFMA loop
    buf = torch.empty(2 * 256 * 1024 * 1024, dtype=torch.uint8, device="cuda:0")
    half = buf.numel() // 2
    measured_peak = {"hbm_copy_gbs": pcb.pc_measure_copy(buf[:half], buf[half:], half, 10),
                     "mfma_f32_tflops": pcb.pc_measure_mfma_f32(buf, buf.numel(), 5),
                     "how": "256 MiB device-to-device copy kernel (bytes read + written); v_mfma_f32_32x32x2_f32 loop, 2 waves per SIMD"}
    del buf

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
        "dtype": "bf16x3->f32 (fp32 operands split into two bf16 values, three bf16 MFMAs per product, fp32 accumulation)" if any_bf16 else "f32",
        "data": "synthetic",
        "config": {"workload": w.name, "structure": w.meta["kind"], "K": w.K, "batch": B, "sum_edges": Es,
                   "n_blocks": w.n_blocks, "n_layers": c.sizes.n_layers, "product_scratch": bool(args.product_scratch),
                   "workspace_bytes": pcb.pc_workspace_bytes(c.handle, B)},
        "roofline": roofline, "measured_peak": measured_peak, "cpu_baseline": cpu, "kernels": kernels, "with_em_step": em,
        "compile_s": compile_s, "generate_s": gen_s,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
