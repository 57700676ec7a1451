"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration bench.py times.

The oracle is too slow for whole batches here, so (a) the first few samples of the full-batch GPU run are
compared with the oracle node by node (log-probabilities and node flows are per-sample quantities), (b) the
batch-summed parameter flows of that run are checked through a property that holds at any size (per sum node, the
edge flows add up to the node's flow, Def. 2), (c) a second full-batch GPU run -- the same launch configuration, the
one bench.py times -- on the oracle's n samples repeated B / n times is compared with B / n times the oracle's
parameter and table flows, element by element, and (d) a GPU run on exactly the oracle's sub-batch likewise.
"""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import pc_oracle as orc
from paper_2406_00766_amd import binding as pcb
from paper_2406_00766_amd import workloads as W
from tests.test_gpu_parity import (assert_device_tables_match_oracle, assert_flow_close, assert_logprob_close,
                                   flow_floors)

pytestmark = pytest.mark.gpu

# (label, workload factory, samples the oracle checks one by one)
CASES = [
    ("config 2", lambda: W.config(2), 16),
    ("config 3", lambda: W.config(3), 4),
    ("config 4", lambda: W.config(4), 4),
    ("config 5", lambda: W.config(5), 4),
    ("rat-spn", lambda: W.rat_config(), 8),
    ("block-sparse layer, 200 sets, 30 % kept", lambda: W.sum_layer(200, 1024, 32, 512, W.SEED_BASE + 7, keep=0.3), 4),
    ("layer of 28 sets at block size 8", lambda: W.sum_layer(28, 1024, 8, 512, W.SEED_BASE + 7), 4),
]


@pytest.mark.parametrize("label,make,n", CASES, ids=[c[0] for c in CASES])
def test_full_size_config(label, make, n):
    print(f"case full-size {label}: generating", flush=True)
    w = make()
    K, B = w.K, w.B
    c = pcb.Circuit(w)
    print("  compiled tables (built by the device compiler) against the compile oracle, bit for bit", flush=True)
    assert_device_tables_match_oracle(c.handle, w)
    c.set_batch(w.x)
    c._ws.fill_(255)                       # NaN bit patterns: nothing may rely on a cleared workspace
    print("  gpu forward/backward at full batch", flush=True)
    ll = c.forward().double().cpu().numpy()
    c.backward()
    torch.cuda.synchronize()
    l, F, R = c.node_buffers()
    lp_gpu = (l[K:, :n].double() + R[1:, :n].double().repeat_interleave(K, dim=0)).cpu().numpy().T
    flow_gpu = F[K:, :n].double().cpu().numpy().T
    tf = c.theta_flow.double().cpu().numpy().reshape(w.theta.shape)
    gf = c.table_flow.double().cpu().numpy().reshape(w.tables.shape)

    print(f"  oracle on the first {n} samples", flush=True)
    wb = w.with_batch(w.x[:n])
    ref_ll, ref_lp, ref_flow, ref_tf, ref_gf = orc.backward(wb, w.theta, w.tables, wb.x)
    floors = flow_floors(wb, w.theta, {"lp": ref_lp, "flow": ref_flow}, n)
    assert_logprob_close(ll[:n], ref_ll, "ll")
    assert_logprob_close(lp_gpu, ref_lp, "node log-probs")
    assert_flow_close(flow_gpu, ref_flow, "node flows", floors["flow"])
    assert np.all(np.isfinite(ll))

    # properties of the batch-summed flows at the full batch size
    assert np.all(np.isfinite(tf)) and np.all(np.isfinite(gf)) and tf.min() >= 0 and gf.min() >= 0
    assert np.isclose(gf.sum(), B * w.n_vars, rtol=1e-4)
    Fsum = F[K:, :B].double().sum(dim=1).cpu().numpy().reshape(w.n_blocks, K)     # per node, summed over the batch
    # sum blocks that share their parameter blocks (tied: the layers of an HMM) share the rows of the flow blocks:
    # per row, the flows over all children add up to the summed node flows of the blocks that use the row
    by_list = {}
    for u in np.nonzero(w.type == W.SUM)[0]:
        by_list.setdefault(tuple(w.param_blk[w.child_ptr[u]:w.child_ptr[u + 1]]), []).append(u)
    keys = list(by_list)
    rng = np.random.default_rng(0)
    for i in rng.choice(len(keys), size=min(200, len(keys)), replace=False):
        row = tf[np.asarray(keys[i]) + 1].sum(axis=(0, 2))
        want = Fsum[by_list[keys[i]]].sum(axis=0)
        assert np.allclose(row, want, rtol=5e-4, atol=1e-30), f"edge flows of sum blocks {by_list[keys[i]][:3]}.. do not add up"

    reps = B // n
    print(f"  gpu at full batch on the oracle's samples repeated {reps} times", flush=True)
    c.theta_flow.zero_(); c.table_flow.zero_()
    c.set_batch(np.tile(wb.x, (reps, 1)))
    ll_t = c.forward().double().cpu().numpy()
    c.backward()
    torch.cuda.synchronize()
    assert_logprob_close(ll_t, np.tile(ref_ll, reps), "ll of the repeated samples")
    assert_flow_close(c.theta_flow.double().cpu().numpy().reshape(w.theta.shape), reps * ref_tf, "theta flows, full batch",
                      reps * floors["theta_flow"])
    assert_flow_close(c.table_flow.double().cpu().numpy().reshape(w.tables.shape), reps * ref_gf, "table flows, full batch",
                      reps * floors["table_flow"])

    print("  gpu on the oracle's sub-batch", flush=True)
    c.theta_flow.zero_(); c.table_flow.zero_()
    c.set_batch(wb.x)
    c.forward(); c.backward()
    torch.cuda.synchronize()
    assert_flow_close(c.theta_flow.double().cpu().numpy().reshape(w.theta.shape), ref_tf, "theta flows", floors["theta_flow"])
    assert_flow_close(c.table_flow.double().cpu().numpy().reshape(w.tables.shape), ref_gf, "table flows", floors["table_flow"])
    c.close()


def test_config5_in_product_scratch_mode():
    """Sec. 5 at full size: config 5 compiled with product_scratch = 1 (block order of pc_order_for_scratch).  The
    workspace shrinks; log-likelihoods, the flows of input and sum nodes and -- on the oracle's samples repeated over
    the whole batch -- every parameter and table flow match the oracle."""
    print("case full-size config 5, product scratch: generating", flush=True)
    w0 = W.config(5)
    w = pcb.pc_order_for_scratch(w0)
    K, B, n = w.K, w.B, 4
    c = pcb.Circuit(w)
    assert_device_tables_match_oracle(c.handle, w)
    h0 = pcb.pc_compile(w0, host_only=True)
    full, small = pcb.pc_workspace_bytes(h0, B), pcb.pc_workspace_bytes(c.handle, B)
    pcb.pc_destroy(h0)
    print(f"  workspace {small / 2**30:.2f} GiB against {full / 2**30:.2f} GiB", flush=True)
    assert small < 0.6 * full
    wb = w.with_batch(w.x[:n])
    ref_ll, ref_lp, ref_flow, ref_tf, ref_gf = orc.backward(wb, w.theta, w.tables, wb.x)
    floors = flow_floors(wb, w.theta, {"lp": ref_lp, "flow": ref_flow}, n)
    c.set_batch(w.x)
    c._ws.fill_(255)
    ll = c.forward().double().cpu().numpy()
    c.backward()
    torch.cuda.synchronize()
    assert np.all(np.isfinite(ll))
    assert_logprob_close(ll[:n], ref_ll, "ll")
    l, F, R = c.node_buffers()
    keep = np.repeat(w.type != W.PRODUCT, K)
    n_keep = int((w.type != W.PRODUCT).sum())
    lp = (l[K:(n_keep + 1) * K, :n].double() + R[1:n_keep + 1, :n].double().repeat_interleave(K, dim=0)).cpu().numpy().T
    assert_logprob_close(lp, ref_lp[:, keep], "log-probabilities of input and sum nodes")
    assert_flow_close(F[K:(n_keep + 1) * K, :n].double().cpu().numpy().T.copy(), ref_flow[:, keep], "flows of input and sum nodes",
                      floors["flow"])
    reps = B // n
    c.theta_flow.zero_(); c.table_flow.zero_()
    c.set_batch(np.tile(wb.x, (reps, 1)))
    c.forward(); c.backward()
    torch.cuda.synchronize()
    assert_flow_close(c.theta_flow.double().cpu().numpy().reshape(w.theta.shape), reps * ref_tf, "theta flows, full batch",
                      reps * floors["theta_flow"])
    assert_flow_close(c.table_flow.double().cpu().numpy().reshape(w.tables.shape), reps * ref_gf, "table flows, full batch",
                      reps * floors["table_flow"])
    c.close()
