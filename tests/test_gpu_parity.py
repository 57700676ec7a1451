"""GPU parity: the HIP path (through the C ABI) against the float64 oracle, element by element.

Tolerances (from the build's target): log-likelihoods and node log-probabilities within 1e-4 relative;
node, parameter and table flows within 1e-3 relative plus the absolute floor that tests/tolerances.py derives from
what fp32 cannot hold (FLT_MIN per ancestor for a node flow, FLT_MIN e^24 theta per term for a parameter flow: some
1e-32 and 1e-28 theta in these circuits -- thirty decades below the largest flow); compiled tables bit-exact.
"""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import compile_oracle as co
from oracle import pc_oracle as orc
from paper_2406_00766_amd import binding as pcb
from paper_2406_00766_amd import workloads as W
from tests import tolerances as tol

pytestmark = pytest.mark.gpu

LL_RTOL = tol.LL_RTOL
FLOW_RTOL = tol.FLOW_RTOL


def to_user_rows(buf, K, B):
    """[n_rows, stride] device buffer (compiled node offsets) -> float64 [B, n_blocks*K] (user numbering)."""
    return buf[K:, :B].double().cpu().numpy().T.copy()


def gpu_run(w, mask=None, backward=True):
    c = pcb.Circuit(w)
    c.set_batch(w.x, mask)
    c._ws.fill_(255)                       # NaN bit patterns: nothing may rely on a cleared workspace
    ll = c.forward().double().cpu().numpy()
    out = {"ll": ll}
    if backward:
        c.backward()
    torch.cuda.synchronize()
    l, F, R = c.node_buffers()
    K, B = w.K, w.B
    lp = l[:, :B].double() + R[:, :B].double().repeat_interleave(K, dim=0)
    out["lp"] = lp[K:].cpu().numpy().T.copy()
    if backward:
        out["flow"] = to_user_rows(F, K, B)
        out["theta_flow"] = c.theta_flow.double().cpu().numpy().reshape(w.theta.shape)
        out["table_flow"] = c.table_flow.double().cpu().numpy().reshape(w.tables.shape)
    out["circuit"] = c
    return out


def assert_logprob_close(got, ref, what):
    inf = np.isneginf(ref)
    assert np.array_equal(np.isneginf(got), inf), f"{what}: -inf pattern differs"
    assert not np.isnan(got).any(), f"{what}: NaN"
    g, r = got[~inf], ref[~inf]
    err = np.abs(g - r)
    bound = LL_RTOL * np.abs(r) + 1e-5
    assert np.all(err <= bound), f"{what}: max err {err.max():.3e} (worst excess {np.max(err - bound):.3e})"


def assert_flow_close(got, ref, what, floor):
    """|got - ref| <= 1e-3 |ref| + floor, element by element; prints the worst relative error per decade of |ref|."""
    assert not np.isnan(got).any() and np.all(np.isfinite(got)), f"{what}: non-finite"
    print(f"    {what}: largest {np.abs(ref).max():.3e}, floor up to {np.max(floor):.2e}")
    for d, n, worst, below in tol.error_by_decade(got, ref, floor):
        print(f"      1e{d:+03d}: {n:9d} entries, worst relative error {worst:.1e}" + (f" ({below} under the floor)" if below else ""))
    excess, at = tol.flow_excess(got, ref, floor)
    assert excess <= 0.0, (f"{what}: entry {at} is {got[at]:.6e}, reference {ref[at]:.6e} "
                           f"(relative error {abs(got[at] - ref[at]) / max(abs(ref[at]), 1e-300):.2e}, "
                           f"floor {float(np.broadcast_to(floor, ref.shape)[at]):.2e})")


def flow_floors(w, theta, ref, B, reps=1):
    """Absolute floors for node / theta / table flows of a run whose oracle results are `ref`; reps: every sample of
    the oracle's batch occurs that many times in the GPU batch (batch-summed flows and their floors scale with it)."""
    return {"flow": tol.node_flow_floor(w),
            "theta_flow": reps * tol.theta_flow_floor(w, theta, ref["lp"], ref["flow"]),
            "table_flow": reps * tol.table_flow_floor(w, B)}


def oracle_run(w, mask=None):
    ll, lp, flow, tf, gf = orc.backward(w, w.theta, w.tables, w.x, mask)
    return {"ll": ll, "lp": lp, "flow": flow, "theta_flow": tf, "table_flow": gf}


def check_all(w, mask=None):
    ref = oracle_run(w, mask)
    got = gpu_run(w, mask)
    assert_logprob_close(got["ll"], ref["ll"], "ll")
    assert_logprob_close(got["lp"], ref["lp"], "node log-probs")
    fl = flow_floors(w, w.theta, ref, w.B)
    assert_flow_close(got["flow"], ref["flow"], "node flows", fl["flow"])
    assert_flow_close(got["theta_flow"], ref["theta_flow"], "theta flows", fl["theta_flow"])
    assert_flow_close(got["table_flow"], ref["table_flow"], "table flows", fl["table_flow"])
    return got, ref


def assert_device_tables_match_oracle(handle, w):
    ref = co.compile_tables(w)
    got = pcb.compiled_tables(handle)
    assert len(got) == len(ref["layers"])
    for a, b in zip(got, ref["layers"]):
        assert (a["kind"], a["depth"]) == (b["kind"], b["depth"])
        for key in ("fwd", "bwd"):
            assert len(a[key]) == len(b[key])
            for ga, gb in zip(a[key], b[key]):
                for xa, xb in zip(ga, gb):
                    assert np.array_equal(xa, np.asarray(xb).reshape(xa.shape))


# ------------------------------------------------------------------------------------------------
REDUCED = [(i, None) for i in range(1, 7)] + [(1, 16), (2, 64), (3, 32), (3, 128), (4, 32), (4, 128), (6, 64), (6, 16)]


@pytest.mark.parametrize("idx,K", REDUCED)
def test_reduced_configs_match_oracle(idx, K):
    w = W.reduced(idx, K=K)
    print(f"case reduced({idx}, K={K}) {w.name}", flush=True)
    got, _ = check_all(w)
    assert_device_tables_match_oracle(got["circuit"].handle, w)


@pytest.mark.parametrize("make", [
    lambda: W.hmm(4, 6, 5, 3, 7, 7),                       # K = 3: generic kernels
    lambda: W.hmm(5, 8, 9, 1, 33, 8),                      # K = 1
    lambda: W.hclt(7, 10, 5, 40, 9, n_cats=6),             # K = 5
    lambda: W.pd(3, 1, 8, 4, 19, 10, n_cats=3, keep=0.5),  # K = 4, block-sparse
    lambda: W.pd(2, 2, 24, 8, 65, 11, n_cats=4),           # K = 8
    lambda: W.hmm(6, 32, 20, 16, 70, 12),                  # K = 16, tied parameter blocks
    lambda: W.hmm(5, 8, 9, 2, 300, 13),                    # K = 2, tied, several column tiles
    lambda: W.hclt(9, 16, 4, 90, 14, n_cats=7),            # K = 4
])
def test_small_block_sizes(make):
    w = make()
    print(f"case generic {w.name}", flush=True)
    check_all(w)


@pytest.mark.parametrize("n_sets,M,K,keep,B", [
    (5, 128, 32, 0.3, 50),      # MFMA kernels, several groups of different widths
    (3, 256, 32, 1.0, 70),      # dense sets
    (3, 256, 64, 0.5, 33),
    (4, 64, 8, 0.4, 40),        # small blocks: vector-ALU block kernels
    (3, 64, 16, 0.6, 130),
    (3, 32, 4, 0.5, 65),
    (3, 32, 2, 0.5, 64),
    (3, 32, 1, 0.5, 37),        # block size 1: one block per node
    (2, 24, 3, 0.7, 20),        # other block sizes: generic kernels
])
def test_block_sparse_sum_layer(n_sets, M, K, keep, B):
    w = W.sum_layer(n_sets, M, K, B, 2406 + K, keep=keep, n_cats=16)
    print(f"case layer {w.name}", flush=True)
    got, _ = check_all(w)
    assert_device_tables_match_oracle(got["circuit"].handle, w)


@pytest.mark.parametrize("make", [
    # tied parameter blocks at K = 128, 64 and 32 (39-40 pairs x 3 chunks per parameter block, dealt to several
    # workgroups / waves that add their partial flows atomically); short reductions: the single-tile kernels
    lambda: W.hmm(40, 256, 60, 128, 70, 41),
    lambda: W.hmm(40, 128, 60, 64, 70, 45),
    lambda: W.hmm(41, 64, 30, 32, 70, 42),
    # 256 categories, K = 64, B = 300: the input-layer flows go through two slabs of samples (256 + 64), some masked
    lambda: W.hclt(12, 128, 64, 300, 43, n_cats=256),
    # 64 chunks per row, few waves: the backward instantiation that waits for a chunk's loads at once
    lambda: W.hmm(3, 2048, 40, 128, 40, 46),
    # more than 1024 categories: per-sample atomics
    lambda: W.hmm(5, 64, 1500, 32, 130, 44, tokens="zipf"),
    # K = 128 / 64 layers just under the size from which the bf16-split kernels take over (ragged third column tile)
    lambda: W.hmm(3, 2048, 40, 128, 90, 52, alpha_trans=0.1, alpha_emis=0.1),
    lambda: W.hmm(3, 2048, 40, 64, 70, 53, alpha_trans=0.1, alpha_emis=0.1),
])
def test_kernel_variants_selected_by_shape(make):
    w = make()
    print(f"case variant {w.name}", flush=True)
    rng = np.random.default_rng(5)
    mask = (rng.random(w.x.shape) < 0.15).astype(np.uint8)
    check_all(w, mask)


def bf16_sum_launches(w):
    """(forward, backward) sum-layer launches of one pass that ran as bf16-split products."""
    c = pcb.Circuit(w)
    c.set_batch(w.x)
    pcb.pc_profile_enable(c.handle, True)
    c.forward(); c.backward()
    torch.cuda.synchronize()
    prof = pcb.pc_profile_read(c.handle, with_bf16=True)
    pcb.pc_profile_enable(c.handle, False)
    c.close()
    return prof["sum_fwd"][2], prof["sum_bwd_child"][2]


@pytest.mark.parametrize("make,reps,tiles", [
    # rows of 2048 children (Dirichlet(0.1) rows as in the large HMM configuration) in the three shapes of the bf16-split
    # sum kernels: 64 x 32 tiles per wave (K = 128; K = 64 with a ragged third 32-column tile) and 64 x 64 tiles (from
    # 200 such tiles on)
    (lambda: W.hmm(3, 2048, 40, 128, 64, 52, alpha_trans=0.1, alpha_emis=0.1), 4, "64x32"),
    (lambda: W.hmm(3, 4096, 40, 64, 45, 56, alpha_trans=0.1, alpha_emis=0.1), 2, "64x32"),
    (lambda: W.hmm(3, 2048, 40, 64, 64, 53, alpha_trans=0.1, alpha_emis=0.1), 7, "64x64"),
    (lambda: W.hmm(3, 2048, 40, 128, 64, 59, alpha_trans=0.1, alpha_emis=0.1), 7, "64x64"),
])
def test_bf16_split_sum_kernels(make, reps, tiles):
    w = make()
    print(f"case bf16 {w.name} x {reps} ({tiles} tiles)", flush=True)
    wt = w.with_batch(np.tile(w.x, (reps, 1)))
    Bs = (wt.B + 31) // 32 * 32
    n_tiles64 = (2048 if "H2048" in w.name else 4096) // 64 * (Bs // 64)
    assert (Bs % 64 == 0 and n_tiles64 >= 200) == (tiles == "64x64")       # the shape the launcher will pick
    fwd, bwd = bf16_sum_launches(wt)
    assert fwd == 2 and bwd == 2, "the transition layers did not take the bf16-split kernels"
    check_repeated(w, reps)


def check_repeated(w, reps, mask=None):
    """The oracle on w's samples, the GPU on those samples repeated `reps` times: per-sample quantities must repeat,
    batch-summed flows (and their floors) are `reps` times the oracle's.  Long batches at the oracle cost of a short one."""
    ref = oracle_run(w, mask)
    wt = w.with_batch(np.tile(w.x, (reps, 1)))
    got = gpu_run(wt, None if mask is None else np.tile(mask, (reps, 1)))
    assert_logprob_close(got["ll"], np.tile(ref["ll"], reps), "ll")
    assert_logprob_close(got["lp"], np.tile(ref["lp"], (reps, 1)), "node log-probs")
    fl = flow_floors(w, w.theta, ref, w.B, reps)
    assert_flow_close(got["flow"], np.tile(ref["flow"], (reps, 1)), "node flows", fl["flow"])
    assert_flow_close(got["theta_flow"], reps * ref["theta_flow"], "theta flows", fl["theta_flow"])
    assert_flow_close(got["table_flow"], reps * ref["table_flow"], "table flows", fl["table_flow"])


@pytest.mark.parametrize("make,reps", [
    # The parameter-flow kernels have a two-tile form for long reductions -- at K = 32 from 12 chunks of 32 samples per
    # wave, at K = 64 and 128 from 64 chunks per workgroup (the forms the full-size configurations run).
    (lambda: W.reduced(2, B=400), 1),                              # K = 32, untied: 13 chunks per block
    (lambda: W.hmm(41, 64, 30, 32, 100, 47), 10),                   # K = 32, tied, pairs dealt to 27 waves: 32 chunks each
    (lambda: W.hclt(12, 128, 64, 256, 48, n_cats=16), 8),           # K = 64, untied: 64 chunks per block
    (lambda: W.hclt(6, 256, 128, 128, 49, n_cats=16), 16),          # K = 128, untied: 64 chunks per block
    (lambda: W.hmm(40, 256, 60, 128, 128, 50), 16),                 # K = 128, tied, pairs dealt to 26 workgroups: 64 chunks each
    (lambda: W.hmm(12, 1024, 200, 128, 100, 51, alpha_trans=0.1, alpha_emis=0.1, tokens="zipf"), 8),   # K = 128, 72 blocks, 3 workgroups each
    # from 128 chunks per workgroup the products are bf16-split (the form the large HMM configuration runs)
    (lambda: W.hmm(12, 1024, 200, 128, 100, 54, alpha_trans=0.1, alpha_emis=0.1, tokens="zipf"), 13),  # K = 128: 135 chunks
    (lambda: W.hmm(40, 128, 60, 64, 32, 55), 127),                                                    # K = 64: 128 chunks
])
def test_two_tile_parameter_flow_kernels(make, reps):
    w = make()
    print(f"case two-tile {w.name} x {reps}", flush=True)
    check_repeated(w, reps)


def test_layer_with_more_groups_than_one_launch_covers():
    """Alg. 2 with G = 16 and tol = 0 gives one group per distinct child count; a launch covers eight groups."""
    import dataclasses
    w = dataclasses.replace(W.sum_layer(3, 512, 32, 70, W.SEED_BASE + 11, keep=0.5), max_groups=16, tol_permille=0)
    print(f"case many groups {w.name}", flush=True)
    got, _ = check_all(w)
    h = got["circuit"].handle
    assert_device_tables_match_oracle(h, w)
    n_layers = pcb.pc_get_sizes(h).n_layers
    assert max(pcb.pc_get_layer(h, li).n_fwd_groups for li in range(n_layers)) > 8


@pytest.mark.parametrize("seed,K,B", [(s, K, B) for s in range(4) for K, B in ((32, 70), (4, 33))] +
                         [(7, 64, 40), (8, 128, 33), (9, 3, 20), (10, 16, 65), (11, 1, 64)])
def test_random_dags_with_skip_connections_tying_and_unused_blocks(seed, K, B):
    w = W.random_circuit(5, 5, 5, K, B, 200 + seed)
    print(f"case random {w.name}", flush=True)
    rng = np.random.default_rng(seed)
    mask = (rng.random(w.x.shape) < 0.2).astype(np.uint8) if seed % 2 else None
    got, _ = check_all(w, mask)
    assert_device_tables_match_oracle(got["circuit"].handle, w)


@pytest.mark.parametrize("make", [
    # sharply peaked parameters (a quarter of the weights at FLT_MIN), 64 tied layers: node log_nf values spread over
    # 100+ nats inside a block, so a wrong block maximum or an unbalanced factor split shows up as inf / lost flows
    lambda: W.hmm(64, 64, 200, 32, 50, 31, alpha_trans=0.01, alpha_emis=0.01, tokens="zipf"),
    lambda: W.hmm(12, 64, 300, 16, 70, 38, alpha_trans=0.02, alpha_emis=0.02, tokens="zipf"),
    lambda: W.hmm(6, 256, 5000, 128, 40, 32, alpha_trans=0.02, alpha_emis=0.02, tokens="zipf"),
    lambda: W.hmm(10, 128, 500, 64, 45, 39, alpha_trans=0.01, alpha_emis=0.01, tokens="zipf"),
])
def test_sharply_peaked_parameters(make):
    w = make()
    print(f"case peaked {w.name}", flush=True)
    check_all(w)


@pytest.mark.parametrize("seed,K", [(3001, 1), (3002, 4), (3014, 4), (3038, 8), (3017, 4), (3018, 1), (3005, 32), (3006, 64),
                                    (3010, 128), (3012, 16)])
def test_random_dags_with_weights_at_the_fp32_floor(seed, K):
    """A quarter of the weights sit at FLT_MIN: a child with such a weight and a large value sets the running maximum
    while a child 87 nats below it with weight 1 contributes as much -- the sum must keep both."""
    s = seed - 3000
    w = W.random_circuit(4 + s % 4, 4 + s % 6, 3 + s % 4, K, 40 if K > 1 else 64, seed, tie_prob=0.5, alpha=0.02)
    print(f"case floor {w.name}", flush=True)
    check_all(w)


def test_block_references_and_block_maxima_are_what_they_claim():
    """R of a product block = sum of its children's R + the ROUNDED column maximum of the block's residuals, so after
    the forward pass every product block's residuals peak within [-0.5, 0.5]; nfmax = column maximum of log_nf."""
    w = W.hmm(8, 64, 100, 32, 40, 40, alpha_trans=0.05, alpha_emis=0.05, tokens="zipf")
    c = pcb.Circuit(w); c.set_batch(w.x); c._ws.fill_(255)
    c.forward(); c.backward(); torch.cuda.synchronize()
    K, B = w.K, w.B
    l, F, R = c.node_buffers()
    for u in np.nonzero(w.type == W.PRODUCT)[0]:
        top = l[(u + 1) * K:(u + 2) * K, :B].max(dim=0).values.cpu().numpy()
        assert np.all(np.abs(top) <= 0.5 + 1e-4), f"product block {u}: residual maximum {np.abs(top).max()}"
    Rh = R[:, :B].cpu().numpy()
    assert np.array_equal(Rh, np.rint(Rh))                 # references are integers: their differences are exact
    for u in np.nonzero(w.type == W.SUM)[0]:                # a sum block's reference = the largest of its children's
        ch = w.child[w.child_ptr[u]:w.child_ptr[u + 1]]
        assert np.array_equal(Rh[u + 1], Rh[ch + 1].max(axis=0)), f"sum block {u}"
    lay = pcb.pc_workspace_layout(c.handle, B)
    n = c.sizes.n_rows * lay.stride
    N = c._ws[lay.n_offset:lay.n_offset + 4 * n].view(torch.float32).view(c.sizes.n_rows, lay.stride)
    ref = orc.backward(w, w.theta, w.tables, w.x, None)
    lp, flow = ref[1], ref[2]
    with np.errstate(divide="ignore"):
        for u in np.nonzero(w.type == W.SUM)[0]:
            if u == w.root_block:
                continue
            got = N[(u + 1) * K:(u + 2) * K, :B].max(dim=0).values.cpu().numpy() - R[u + 1, :B].cpu().numpy()
            want = (np.log(flow[:, u * K:(u + 1) * K]) - lp[:, u * K:(u + 1) * K]).max(axis=1)
            assert np.allclose(got, want, rtol=1e-4, atol=1e-3), f"sum block {u}"
    c.close()


@pytest.mark.parametrize("make", [
    lambda: W.non_alternating(5, 5, 5, 32, 40, 913),
    lambda: W.non_alternating(4, 4, 4, 4, 33, 900),
    lambda: W.non_alternating_from(W.reduced(2), 6),          # HCLT, K = 32: every edge of the tree may be doubled
    lambda: W.non_alternating_from(W.reduced(5), 7),          # pruned PD
    lambda: W.non_alternating_from(W.reduced(3, B=40), 8),    # K = 64
])
def test_collapsed_non_alternating_dag(make):
    """Footnote to Def. 2: pc_compile refuses consecutive sum / sum and product / product blocks; pc_collapse rewrites
    them.  The GPU runs the library's collapsed DAG; the oracle runs (a) the same collapsed DAG, flows and all, and
    (b) the ORIGINAL DAG node by node, whose log-likelihoods the collapsed circuit must reproduce."""
    w = make()
    print(f"case collapse {w.name}", flush=True)
    with pytest.raises(pcb.PcError) as e:
        pcb.pc_compile(w)
    assert e.value.status_name == "PC_ERR_NOT_ALTERNATING"
    wc = pcb.pc_collapse(w)
    ref = co.collapse(w, w.theta)
    for k in ("type", "child_ptr", "child", "param_blk"):
        assert np.array_equal(getattr(wc, k), getattr(ref, k)), k
    got, _ = check_all(wc)
    assert_device_tables_match_oracle(got["circuit"].handle, wc)
    assert_logprob_close(got["ll"], orc.forward(w, w.theta, w.tables, w.x)[1], "ll against the original DAG")


@pytest.mark.parametrize("make", [
    lambda: W.reduced(5),                                  # pruned PD: product blocks of several depths feed one sum layer
    lambda: W.reduced(2, B=70),                            # HCLT
    lambda: W.reduced(4, K=32),                            # tied HMM: parameter flows accumulate layer by layer
    lambda: W.reduced(6),                                  # RAT-SPN
    lambda: W.hclt(9, 16, 4, 90, 14, n_cats=7),            # K = 4: vector-ALU kernels
    lambda: W.hmm(4, 6, 5, 3, 7, 7),                       # K = 3: generic kernels
    lambda: W.random_circuit(5, 5, 5, 32, 40, 203),        # product blocks read by sum blocks of several depths: copied
    lambda: W.random_circuit(5, 5, 5, 4, 33, 204),
])
def test_product_scratch_mode(make):
    """Sec. 5: product log-probabilities live in one scratch window and are recomputed in the backward pass.  Same
    results as the oracle on the reordered circuit; the workspace is smaller; compiled tables bit-exact."""
    w0 = make()
    w = pcb.pc_order_for_scratch(w0)
    assert w.product_scratch == 1
    print(f"case product scratch {w.name}", flush=True)
    ref = oracle_run(w)
    c = pcb.Circuit(w)
    assert_device_tables_match_oracle(c.handle, w)
    c0 = pcb.Circuit(w0)
    assert pcb.pc_workspace_bytes(c.handle, w.B) < pcb.pc_workspace_bytes(c0.handle, w.B)
    c0.close()
    c.set_batch(w.x)
    c._ws.fill_(255)
    ll = c.forward().double().cpu().numpy()
    c.backward()
    torch.cuda.synchronize()
    assert_logprob_close(ll, ref["ll"], "ll")
    K, B = w.K, w.B
    l, F, R = c.node_buffers()
    keep = np.repeat(w.type != W.PRODUCT, K)               # product rows of l are not kept in this mode
    n_keep = int((w.type != W.PRODUCT).sum())
    lp = (l[K:(n_keep + 1) * K, :B].double() + R[1:n_keep + 1, :B].double().repeat_interleave(K, dim=0)).cpu().numpy().T
    assert_logprob_close(lp, ref["lp"][:, keep], "log-probabilities of input and sum nodes")
    fl = flow_floors(w, w.theta, ref, B)
    assert_flow_close(F[K:(n_keep + 1) * K, :B].double().cpu().numpy().T.copy(), ref["flow"][:, keep], "flows of input and sum nodes",
                      fl["flow"])
    assert_flow_close(c.theta_flow.double().cpu().numpy().reshape(w.theta.shape), ref["theta_flow"], "theta flows", fl["theta_flow"])
    assert_flow_close(c.table_flow.double().cpu().numpy().reshape(w.tables.shape), ref["table_flow"], "table flows", fl["table_flow"])
    # the same results as the circuit in its original form: product blocks carry no parameters, so reordering and
    # copying them leaves log-likelihoods and parameter flows what they were
    ref0 = oracle_run(w0)
    assert np.allclose(ref["ll"], ref0["ll"], rtol=1e-12, atol=1e-12)
    assert np.allclose(ref["theta_flow"], ref0["theta_flow"], rtol=1e-9, atol=0)
    assert np.allclose(ref["table_flow"], ref0["table_flow"], rtol=1e-9, atol=0)
    c.close()


def test_config1_full_size():
    w = W.config(1)
    print("case cfg1 full", flush=True)
    got, _ = check_all(w)
    assert_device_tables_match_oracle(got["circuit"].handle, w)


@pytest.mark.parametrize("B", [1, 31, 32, 33, 129, 300])
def test_ragged_batches(B):
    w = W.reduced(2, B=B)
    print(f"case ragged B={B}", flush=True)
    check_all(w)


def test_marginalised_variables_and_zero_probability_samples():
    w = W.reduced(2, B=50)
    rng = np.random.default_rng(1)
    mask = (rng.random(w.x.shape) < 0.3).astype(np.uint8)
    mask[0, :] = 1                                          # fully marginalised sample: ll = 0
    print("case mask", flush=True)
    got, ref = check_all(w, mask)
    assert abs(got["ll"][0]) < 1e-4
    # zero-probability samples: category 0 made impossible in every table
    w2 = W.reduced(1, B=40)
    w2.tables = w2.tables.copy(); w2.tables[:, 0, :] = 0.0
    x = np.where(w2.x == 0, 1, w2.x); x[3, 2] = 0; x[17, 0] = 0
    w2 = w2.with_batch(x)
    print("case zero-prob", flush=True)
    got, ref = check_all(w2)
    assert np.isneginf(got["ll"][3]) and np.isneginf(got["ll"][17]) and np.isfinite(got["ll"][4])
    assert np.all(got["flow"][3] == 0.0)


def test_flows_accumulate_over_calls_and_em_step_matches_oracle():
    w = W.reduced(3, B=64)
    c = pcb.Circuit(w)
    ref_tf = ref_gf = None
    floor_tf, floor_gf = 0.0, 0.0
    for part in (slice(0, 40), slice(40, 64)):
        wb = w.with_batch(w.x[part])
        c.set_batch(wb.x)
        c.forward(); c.backward()
        _, lp, flow, ref_tf, ref_gf = orc.backward(wb, w.theta, w.tables, wb.x, None, ref_tf, ref_gf)
        fl = flow_floors(wb, w.theta, {"lp": lp, "flow": flow}, wb.B)
        floor_tf, floor_gf = floor_tf + fl["theta_flow"], floor_gf + fl["table_flow"]
    torch.cuda.synchronize()
    assert_flow_close(c.theta_flow.double().cpu().numpy().reshape(w.theta.shape), ref_tf, "accumulated theta flows", floor_tf)
    assert_flow_close(c.table_flow.double().cpu().numpy().reshape(w.tables.shape), ref_gf, "accumulated table flows", floor_gf)
    for step, pc in ((1.0, 0.0), (0.3, 0.1)):
        th0 = c.theta.cpu().numpy().reshape(w.theta.shape).copy()
        tb0 = c.tables.cpu().numpy().reshape(w.tables.shape).copy()
        tf = c.theta_flow.double().cpu().numpy().reshape(w.theta.shape)
        gf = c.table_flow.double().cpu().numpy().reshape(w.tables.shape)
        ref_th, ref_tb = orc.em_step(w, th0, tb0, tf, gf, step=step, pseudocount=pc)
        c.em_step(step, pc)
        torch.cuda.synchronize()
        th = c.theta.cpu().numpy().reshape(w.theta.shape)
        tb = c.tables.cpu().numpy().reshape(w.tables.shape)
        assert np.allclose(th, ref_th, rtol=1e-4, atol=1e-9) and np.allclose(tb, ref_tb, rtol=1e-4, atol=1e-9)
        assert float(c.theta_flow.abs().max()) == 0.0 and float(c.table_flow.abs().max()) == 0.0
        assert np.all(th[0] == 0.0)
        # next round of flows for the second EM variant
        c.set_batch(w.x); c.forward(); c.backward()


@pytest.mark.parametrize("K", [1, 3, 4, 8, 12, 16, 64, 128])
def test_em_step_at_every_block_size(K):
    """The EM kernels have 16-byte forms (K a multiple of 4 for the tables, a power of two for the parameters) and plain
    ones; random DAGs have sum blocks with fewer than K real nodes, tied parameter blocks and unused blocks."""
    w = W.random_circuit(5, 4, 4, K, 40, 700 + K, tie_prob=0.4)
    print(f"case em {w.name}", flush=True)
    c = pcb.Circuit(w)
    c.set_batch(w.x)
    for step, pc in ((1.0, 0.0), (0.4, 0.05)):
        c.forward(); c.backward()
        torch.cuda.synchronize()
        th0 = c.theta.cpu().numpy().reshape(w.theta.shape).copy()
        tb0 = c.tables.cpu().numpy().reshape(w.tables.shape).copy()
        tf = c.theta_flow.double().cpu().numpy().reshape(w.theta.shape)
        gf = c.table_flow.double().cpu().numpy().reshape(w.tables.shape)
        ref_th, ref_tb = orc.em_step(w, th0, tb0, tf, gf, step=step, pseudocount=pc)
        c.em_step(step, pc)
        torch.cuda.synchronize()
        th = c.theta.cpu().numpy().reshape(w.theta.shape)
        tb = c.tables.cpu().numpy().reshape(w.tables.shape)
        assert np.allclose(th, ref_th, rtol=1e-4, atol=1e-9), f"theta, step {step}"
        assert np.allclose(tb, ref_tb, rtol=1e-4, atol=1e-9), f"tables, step {step}"
        assert float(c.theta_flow.abs().max()) == 0.0 and float(c.table_flow.abs().max()) == 0.0
    c.close()


def test_em_on_tied_hmm_matches_oracle_and_improves_likelihood():
    w = W.reduced(4, B=96)
    c = pcb.Circuit(w)
    c.set_batch(w.x)
    ll0 = c.forward().double().sum().item()
    c.backward()
    tf = c.theta_flow.double().cpu().numpy().reshape(w.theta.shape)
    gf = c.table_flow.double().cpu().numpy().reshape(w.tables.shape)
    ref_th, ref_tb = orc.em_step(w, w.theta, w.tables, tf, gf, step=1.0, pseudocount=0.0)
    c.em_step(1.0, 0.0)
    torch.cuda.synchronize()
    assert np.allclose(c.theta.cpu().numpy().reshape(w.theta.shape), ref_th, rtol=1e-4, atol=1e-9)
    assert np.allclose(c.tables.cpu().numpy().reshape(w.tables.shape), ref_tb, rtol=1e-4, atol=1e-9)
    ll1 = c.forward().double().sum().item()
    assert ll1 >= ll0


@pytest.mark.parametrize("make", [
    lambda: W.reduced(2),
    # the bf16-split path: plane splits, product kernels that write planes, bf16 sum kernels (256 samples: 64 x 32 tiles)
    lambda: W.hmm(3, 2048, 40, 128, 256, 65, alpha_trans=0.1, alpha_emis=0.1),
])
def test_forward_and_backward_replayed_from_a_captured_graph(make):
    """pc_forward / pc_backward only enqueue kernels, so a caller may capture them into a HIP graph.  The graph is
    replayed several times with eager work and synchronisations in between; every replay must reproduce the eager
    result (log-likelihoods and parameter flows bit for bit: no atomics on those paths)."""
    w = make()
    print(f"case graph {w.name}", flush=True)
    c = pcb.Circuit(w)
    c.set_batch(w.x)
    c.forward(); c.backward()
    torch.cuda.synchronize()
    ref_ll, ref_tf, ref_gf = c.ll.clone(), c.theta_flow.clone(), c.table_flow.clone()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        c.forward(); c.backward()                              # warm-up on the capture stream
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            c.forward(); c.backward()
    torch.cuda.synchronize()
    for replay in range(4):
        c.theta_flow.zero_(); c.table_flow.zero_(); c.ll.fill_(float("nan"))     # eager work between the replays
        c._ws.fill_(255)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(c.ll, ref_ll), f"replay {replay}"
        assert torch.equal(c.theta_flow, ref_tf), f"replay {replay}"
        assert torch.allclose(c.table_flow, ref_gf, rtol=1e-5, atol=1e-7), f"replay {replay}"
    del graph
    c.close()


def test_forward_is_deterministic_and_state_errors():
    w = W.reduced(5)
    c = pcb.Circuit(w)
    c.set_batch(w.x)
    a = c.forward().clone()
    b = c.forward().clone()
    torch.cuda.synchronize()
    assert torch.equal(a, b)                               # no atomics on the forward path
    # backward with a different batch size than the forward
    with pytest.raises(pcb.PcError) as e:
        pcb.pc_backward(c.handle, c.theta, c.tables, c.x, None, c.B - 1, c._ws, c._ws.numel(), c.theta_flow, c.table_flow)
    assert e.value.status_name == "PC_ERR_STATE"
    with pytest.raises(pcb.PcError) as e:
        pcb.pc_forward(c.handle, c.theta, c.tables, c.x, None, c.B, c._ws, 1024, c.ll)
    assert e.value.status_name == "PC_ERR_WORKSPACE"
    with pytest.raises(pcb.PcError) as e:
        pcb.pc_forward(c.handle, c.theta, c.tables, c.x, None, 0, c._ws, c._ws.numel(), c.ll)
    assert e.value.status_name == "PC_ERR_ARG"
    with pytest.raises(pcb.PcError) as e:                  # the kernels use 16-byte accesses
        pcb.pc_forward(c.handle, c.theta[1:], c.tables, c.x, None, c.B, c._ws, c._ws.numel(), c.ll)
    assert e.value.status_name == "PC_ERR_ARG"
    with pytest.raises(pcb.PcError) as e:
        pcb.pc_forward(c.handle, c.theta, c.tables, c.x, None, 2097153, c._ws, c._ws.numel(), c.ll)
    assert e.value.status_name == "PC_ERR_TOO_LARGE"
    # EM invalidates the forward state
    c.forward(); c.backward(); c.em_step()
    with pytest.raises(pcb.PcError):
        c.backward()


def test_sum_block_without_parents_gets_zero_flow():
    # an extra sum block over the product blocks of the HCLT root variable that nothing refers to: it is
    # evaluated in the forward pass, carries flow 0, and must not disturb the flows of its children
    w = W.reduced(2, B=40)
    K, nb = w.K, w.meta["M"] // w.K
    prods = [b for b in range(w.n_blocks) if w.type[b] == W.PRODUCT][:nb]          # P_0[0..nb-1]
    rng = np.random.default_rng(4)
    extra_theta = rng.dirichlet(np.ones(nb * K), size=K).astype(np.float32).reshape(K, nb, K).transpose(1, 0, 2)
    w2 = w.with_batch(w.x)
    w2.n_blocks = w.n_blocks + 1
    w2.type = np.append(w.type, np.uint8(W.SUM))
    w2.n_real = np.append(w.n_real, np.int32(K))
    w2.in_var = np.append(w.in_var, np.int32(-1)); w2.in_table = np.append(w.in_table, np.int32(-1))
    w2.child_ptr = np.append(w.child_ptr, w.child_ptr[-1] + nb)
    w2.child = np.append(w.child, np.array(prods, dtype=np.int32))
    w2.param_blk = np.append(w.param_blk, np.arange(w.n_param_blocks, w.n_param_blocks + nb, dtype=np.int32))
    w2.n_param_blocks = w.n_param_blocks + nb
    w2.theta = np.concatenate([w.theta, extra_theta])
    print("case orphan sum block", flush=True)
    got, ref = check_all(w2)
    orphan = w.n_blocks
    assert np.all(got["flow"][:, orphan * K:(orphan + 1) * K] == 0.0)
    assert np.all(got["theta_flow"][-nb:] == 0.0)
    assert np.all(np.isfinite(got["lp"][:, orphan * K:(orphan + 1) * K]))


def test_out_of_range_category_has_probability_zero():
    for w in (W.reduced(1, B=8), W.reduced(4, B=40), W.reduced(5, B=33)):       # direct, sorted and histogram table flows
        x = w.x.copy(); x[2, 1] = w.n_cats + 5; x[5, 0] = -3
        print(f"case out-of-range {w.name}", flush=True)
        got, ref = check_all(w.with_batch(x))
        ll = got["ll"]
        assert np.isneginf(ll[2]) and np.isneginf(ll[5]) and np.isfinite(ll[0])
        assert np.all(got["flow"][2] == 0.0) and np.all(got["flow"][5] == 0.0)


@pytest.mark.parametrize("make", [
    lambda: W.hmm(7, 64, 3000, 32, 300, 61, tokens="zipf"),             # two slabs (256 + 64 columns), K = 32: two node slices
    lambda: W.hmm(5, 32, 2000, 16, 70, 62, tokens="zipf"),              # K = 16, one slice, small-block kernels elsewhere
    lambda: W.hmm(4, 256, 5000, 128, 33, 63, tokens="zipf"),            # K = 128, a few samples
    lambda: W.hclt(9, 64, 64, 90, 64, n_cats=1200),                     # untied tables: one input block per table
])
def test_large_vocabulary_table_flows(make):
    """More than 1024 categories (per-sample adds into the table rows), with masked and out-of-range samples, a ragged
    second slab of columns, tied and untied tables."""
    w = make()
    print(f"case large vocabulary {w.name}", flush=True)
    rng = np.random.default_rng(6)
    mask = (rng.random(w.x.shape) < 0.2).astype(np.uint8)
    x = w.x.copy(); x[1, 0] = w.n_cats + 3; x[w.B - 1, w.n_vars - 1] = -7
    wx = w.with_batch(x)
    check_all(wx, mask)


def test_parameter_flows_repeat_bit_for_bit_where_no_pairs_are_split():
    """Parameter flows are written by exactly one workgroup per parameter block, in a fixed order, unless the launcher
    deals the tied pairs of a block over several waves or workgroups (fewer than 128 parameter blocks with at least two
    tied pairs each: small tied models).  Untied circuits and large tied models are therefore reproducible to the bit;
    so are log-probabilities and node flows everywhere."""
    cases = [W.reduced(2, B=100),                                        # untied, K = 32
             W.reduced(5, B=64),                                         # untied, block-sparse, K = 32
             W.hmm(4, 1024, 50, 64, 64, 57, tokens="zipf"),               # tied, 257 parameter blocks of 64 x 64
             W.hmm(3, 2048, 50, 128, 256, 58, tokens="zipf")]             # tied, 257 parameter blocks of 128 x 128
    for w in cases:
        print(f"case bit-repeat {w.name}", flush=True)
        a, b = gpu_run(w), gpu_run(w)
        for key in ("ll", "lp", "flow", "theta_flow"):
            assert np.array_equal(a[key], b[key], equal_nan=True), f"{w.name}: {key} differs between two runs"
        a["circuit"].close(); b["circuit"].close()
