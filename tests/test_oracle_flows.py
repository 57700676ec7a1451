"""Pins of the oracle's backward pass (PC flows, Def. 2) and EM step.

* root flow is 1 and every node's flow is the sum of its parents' contributions (Def. 2), re-derived
  here by a *gather over parents* in numpy, the opposite traversal of the oracle's scatter;
* flows are gradients (Sec. 5, App. B.2): F_{n,c} = d log p / d log theta_{n,c}, checked with torch
  autograd (float64) through the textbook HMM forward algorithm and latent-tree message passing, and
  with central finite differences of the oracle's own forward pass on a pruned grid structure;
* for an HMM the accumulated flows are the Baum-Welch expected counts (alpha-beta recursions);
* per sum node the edge flows add up to the node flow; per variable the input flows add up to 1.
"""
import numpy as np
import pytest
import torch

from oracle import pc_oracle as orc
from paper_2406_00766_amd import workloads as W
from tests import refs


def parents_gather_flows(w, theta, lp):
    """Node flows recomputed parent-side: F_n = sum over parents (Def. 2), float64 numpy."""
    K, n = w.K, w.n_blocks
    B = lp.shape[0]
    par = [[] for _ in range(n)]
    for u in range(n):
        for e in range(w.child_ptr[u], w.child_ptr[u + 1]):
            par[w.child[e]].append((u, e))
    order = []                                   # parents before children (Kahn on parent counts)
    indeg = np.array([len(p) for p in par])
    ready = [u for u in range(n) if indeg[u] == 0]
    while ready:
        u = ready.pop()
        order.append(u)
        for e in range(w.child_ptr[u], w.child_ptr[u + 1]):
            c = w.child[e]
            indeg[c] -= 1
            if indeg[c] == 0:
                ready.append(c)
    F = np.zeros((B, n, K))
    th = theta.astype(np.float64)
    L = lp.reshape(B, n, K)
    for u in order:
        if u == w.root_block:
            F[:, u, 0] = 1.0
            continue
        for (m, e) in par[u]:
            if w.type[m] == W.PRODUCT:
                F[:, u, :] += F[:, m, :]
            else:
                T = th[w.param_blk[e] + 1]                                  # [i (parent row), j (child row)]
                with np.errstate(divide="ignore", invalid="ignore"):
                    ratio = np.exp(L[:, u, None, :] - L[:, m, :, None])     # [B, i, j] = p_c / p_n
                ratio = np.where(np.isfinite(ratio), ratio, 0.0)
                F[:, u, :] += np.einsum("ij,bij,bi->bj", T, ratio, F[:, m, :])
    return F.reshape(B, n * K)


SMALL = [
    lambda: W.hmm(4, 4, 5, 2, 6, 61),
    lambda: W.hclt(6, 4, 2, 5, 62, n_cats=4),
    lambda: W.pd(3, 1, 4, 2, 7, 63, n_cats=3, keep=0.5),
    lambda: W.pd(2, 2, 4, 4, 5, 64, n_cats=3),
    lambda: W.reduced(5),
]


@pytest.mark.parametrize("make", SMALL)
def test_root_flow_and_parent_sum(make):
    w = make()
    ll, lp, flow, _, _ = orc.backward(w, w.theta, w.tables, w.x)
    assert np.all(flow[:, w.root_block * w.K] == 1.0)
    ref = parents_gather_flows(w, w.theta, lp)
    assert np.allclose(flow, ref, rtol=1e-10, atol=1e-14)


@pytest.mark.parametrize("make", SMALL + [lambda: W.reduced(2), lambda: W.reduced(1)])
def test_flow_sums(make):
    w = make()
    ll, lp, flow, tf, gf = orc.backward(w, w.theta, w.tables, w.x)
    B, K = w.B, w.K
    # per variable, the flows into its input nodes add up to 1 for every sample (smooth + decomposable)
    per_var = np.zeros((B, w.n_vars))
    for u in np.nonzero(w.type == W.INPUT)[0]:
        per_var[:, w.in_var[u]] += flow[:, u * K:(u + 1) * K].sum(axis=1)
    assert np.allclose(per_var, 1.0, rtol=0, atol=1e-9)
    assert np.isclose(gf.sum(), B * w.n_vars, rtol=1e-10)
    # untied circuits: the edge flows of a sum node add up to its node flow (summed over the batch)
    if w.meta["kind"] != "hmm":
        for u in np.nonzero(w.type == W.SUM)[0]:
            row = np.zeros(K)
            for e in range(w.child_ptr[u], w.child_ptr[u + 1]):
                row += tf[w.param_blk[e] + 1].sum(axis=1)
            assert np.allclose(row, flow[:, u * K:(u + 1) * K].sum(axis=0), rtol=1e-9, atol=1e-12)
    else:
        T, H = w.meta["T"], w.meta["H"]
        nb = H // K
        assert np.isclose(tf[1:1 + nb * nb].sum(), B * (T - 1), rtol=1e-10)      # one transition per step
        assert np.isclose(tf[1 + nb * nb:].sum(), B, rtol=1e-10)                 # one initial state


def _hmm_dense_flows(w, tf, gf):
    K, H = w.K, w.meta["H"]
    nb = H // K
    GA = tf[1:1 + nb * nb].reshape(nb, nb, K, K).transpose(0, 2, 1, 3).reshape(H, H)
    Gpi = tf[1 + nb * nb:, 0, :].reshape(H)
    GE = gf.transpose(0, 2, 1).reshape(H, -1)
    return Gpi, GA, GE


@pytest.mark.parametrize("make", [
    lambda: W.hmm(5, 6, 7, 3, 9, 71),
    lambda: W.config(1),
    lambda: W.hmm(6, 8, 12, 4, 8, 72, alpha_trans=0.1, alpha_emis=0.1, tokens="zipf"),
])
def test_hmm_flows_are_gradients_and_baum_welch_counts(make):
    w = make()
    _, _, _, tf, gf = orc.backward(w, w.theta, w.tables, w.x)
    Gpi, GA, GE = _hmm_dense_flows(w, tf, gf)
    pi = w.meta["pi"].astype(np.float64); A = w.meta["A"].astype(np.float64)
    E = W.hmm_emission(w).astype(np.float64)
    # (a) autograd through the textbook forward algorithm: d sum_b log p / d log(param)
    lpi = torch.tensor(np.log(pi), requires_grad=True)
    lA = torch.tensor(np.log(A), requires_grad=True)
    lE = torch.tensor(np.log(E), requires_grad=True)
    refs.hmm_loglik_torch(lpi, lA, lE, torch.tensor(w.x, dtype=torch.long)).sum().backward()
    assert np.allclose(Gpi, lpi.grad.numpy(), rtol=1e-9, atol=1e-12)
    assert np.allclose(GA, lA.grad.numpy(), rtol=1e-9, atol=1e-12)
    assert np.allclose(GE, lE.grad.numpy(), rtol=1e-9, atol=1e-12)
    # (b) alpha-beta expected counts
    g0, xi, em, _ = refs.hmm_baum_welch_counts(pi, A, E, w.x)
    assert np.allclose(Gpi, g0, rtol=1e-9, atol=1e-12)
    assert np.allclose(GA, xi, rtol=1e-9, atol=1e-12)
    assert np.allclose(GE, em, rtol=1e-9, atol=1e-12)


@pytest.mark.parametrize("make", [lambda: W.hclt(7, 4, 2, 6, 73, n_cats=5), lambda: W.reduced(2)])
def test_hclt_flows_are_gradients(make):
    w = make()
    _, _, _, tf, gf = orc.backward(w, w.theta, w.tables, w.x)
    D, M, K = w.meta["D"], w.meta["M"], w.K
    nb = M // K
    lW = [None] + [torch.tensor(np.log(W.hclt_edge_weights(w, c).astype(np.float64)), requires_grad=True)
                   for c in range(1, D)]
    lT = [torch.tensor(np.log(W.hclt_table(w, v).astype(np.float64)), requires_grad=True) for v in range(D)]
    lpi = torch.tensor(np.log(w.meta["pi"].astype(np.float64)), requires_grad=True)
    refs.latent_tree_loglik_torch(w.meta["parent"], w.meta["order"], lpi, lW, lT,
                                  torch.tensor(w.x, dtype=torch.long)).sum().backward()
    for c in range(1, D):
        base = 1 + (c - 1) * nb * nb
        G = tf[base:base + nb * nb].reshape(nb, nb, K, K).transpose(0, 2, 1, 3).reshape(M, M)
        assert np.allclose(G, lW[c].grad.numpy(), rtol=1e-9, atol=1e-12)
    for v in range(D):
        G = gf[v * nb:(v + 1) * nb].transpose(0, 2, 1).reshape(M, -1)
        assert np.allclose(G, lT[v].grad.numpy(), rtol=1e-9, atol=1e-12)
    assert np.allclose(tf[1 + (D - 1) * nb * nb:, 0, :].reshape(M), lpi.grad.numpy(), rtol=1e-9, atol=1e-12)


def test_pd_edge_flows_match_finite_differences():
    w = W.pd(3, 1, 4, 2, 1, 81, n_cats=3, keep=0.6)
    ll, lp, flow, tf, gf = orc.backward(w, w.theta, w.tables, w.x)
    rng = np.random.default_rng(9)
    nz = np.argwhere(w.theta > 0)
    picks = nz[rng.choice(len(nz), size=40, replace=False)]
    h = 1e-2
    for p, i, j in picks:
        tp = w.theta.copy(); tm = w.theta.copy()
        tp[p, i, j] = np.float32(w.theta[p, i, j] * (1 + h)); tm[p, i, j] = np.float32(w.theta[p, i, j] * (1 - h))
        d = np.log(np.float64(tp[p, i, j])) - np.log(np.float64(tm[p, i, j]))
        _, lp_ = orc.forward(w, tp, w.tables, w.x); _, lm_ = orc.forward(w, tm, w.tables, w.x)
        fd = (lp_[0] - lm_[0]) / d
        assert np.isclose(tf[p, i, j], fd, rtol=2e-3, atol=1e-7), (p, i, j, tf[p, i, j], fd)
    # table flows: d log p / d log table entry, same recipe
    nzt = np.argwhere(gf > 0)
    for t, c, k in nzt[rng.choice(len(nzt), size=min(20, len(nzt)), replace=False)]:
        tp = w.tables.copy(); tm = w.tables.copy()
        tp[t, c, k] = np.float32(w.tables[t, c, k] * (1 + h)); tm[t, c, k] = np.float32(w.tables[t, c, k] * (1 - h))
        d = np.log(np.float64(tp[t, c, k])) - np.log(np.float64(tm[t, c, k]))
        _, lp_ = orc.forward(w, w.theta, tp, w.x); _, lm_ = orc.forward(w, w.theta, tm, w.x)
        assert np.isclose(gf[t, c, k], (lp_[0] - lm_[0]) / d, rtol=2e-3, atol=1e-7)


def test_masked_variables_get_no_table_flow_and_zero_prob_samples_no_flow():
    w = W.hclt(5, 4, 2, 6, 91, n_cats=4)
    mask = np.zeros((w.B, w.n_vars), dtype=np.uint8); mask[:, 2] = 1
    _, _, flow, tf, gf = orc.backward(w, w.theta, w.tables, w.x, mask)
    nb = 2
    assert gf[2 * nb:3 * nb].sum() == 0.0
    assert np.isclose(gf.sum(), w.B * (w.n_vars - 1), rtol=1e-10)
    tables = w.tables.copy(); tables[:, 0, :] = 0.0
    x = np.where(w.x == 0, 1, w.x); x[3, 1] = 0
    ll, _, flow, tf, gf = orc.backward(w, w.theta, tables, x)
    assert ll[3] == -np.inf and np.all(flow[3] == 0.0)
    assert np.isclose(gf.sum(), (w.B - 1) * w.n_vars, rtol=1e-10) and np.all(np.isfinite(tf))


# ---------------------------------------------------------------------------------------- EM
def test_em_step_is_baum_welch_update_for_hmm():
    w = W.hmm(5, 6, 7, 3, 40, 101)
    _, _, _, tf, gf = orc.backward(w, w.theta, w.tables, w.x)
    th1, tb1 = orc.em_step(w, w.theta, w.tables, tf, gf, step=1.0, pseudocount=0.0)
    pi = w.meta["pi"].astype(np.float64); A = w.meta["A"].astype(np.float64); E = W.hmm_emission(w).astype(np.float64)
    g0, xi, em, _ = refs.hmm_baum_welch_counts(pi, A, E, w.x)
    w1 = w.with_batch(w.x); w1.theta = th1; w1.tables = tb1
    K, H = w.K, 6
    nb = H // K
    A1 = th1[1:1 + nb * nb].reshape(nb, nb, K, K).transpose(0, 2, 1, 3).reshape(H, H)
    assert np.allclose(A1, xi / xi.sum(axis=1, keepdims=True), rtol=1e-6)
    assert np.allclose(th1[1 + nb * nb:, 0, :].reshape(H), g0 / g0.sum(), rtol=1e-6)
    assert np.allclose(W.hmm_emission(w1), em / em.sum(axis=1, keepdims=True), rtol=1e-6, atol=1e-30)
    assert np.all(th1[1 + nb * nb:, 1:, :] == 0.0)          # placeholder rows of the root block untouched


@pytest.mark.parametrize("make", [lambda: W.reduced(2, B=40), lambda: W.reduced(5, B=30), lambda: W.reduced(1, B=50)])
def test_em_keeps_simplex_and_never_decreases_likelihood(make):
    w = make()
    theta, tables = w.theta, w.tables
    prev = -np.inf
    for it in range(3):
        ll, _, _, tf, gf = orc.backward(w, theta, tables, w.x)
        assert ll.sum() >= prev - 1e-6 * abs(ll.sum())
        prev = ll.sum()
        theta, tables = orc.em_step(w, theta, tables, tf, gf, step=1.0, pseudocount=0.0)
        for u in np.nonzero(w.type == W.SUM)[0]:
            rows = sum(theta[w.param_blk[e] + 1].astype(np.float64).sum(axis=1)
                       for e in range(w.child_ptr[u], w.child_ptr[u + 1]))
            assert np.allclose(rows[:w.n_real[u]], 1.0, atol=1e-5)
        assert np.allclose(tables.astype(np.float64).sum(axis=1), 1.0, atol=1e-5)


def test_em_step_size_and_pseudocount():
    w = W.hclt(5, 4, 2, 12, 111, n_cats=4)
    _, _, _, tf, gf = orc.backward(w, w.theta, w.tables, w.x)
    full, _ = orc.em_step(w, w.theta, w.tables, tf, gf, step=1.0, pseudocount=0.0)
    half, _ = orc.em_step(w, w.theta, w.tables, tf, gf, step=0.25, pseudocount=0.0)
    real = np.ones_like(w.theta, dtype=bool); real[0] = False
    real[-2:, 1:, :] = False                                  # root block rows 1.. are placeholders
    assert np.allclose(half[real], 0.75 * w.theta[real] + 0.25 * full[real], rtol=1e-6)
    # a huge pseudocount pulls every real row to uniform over its real children
    uni, tab = orc.em_step(w, w.theta, w.tables, tf, gf, step=1.0, pseudocount=1e12)
    assert np.allclose(uni[1:-2], 1.0 / 4, rtol=1e-5)
    assert np.allclose(tab, 1.0 / 4, rtol=1e-5)
    assert np.all(uni[-2:, 1:, :] == 0.0) and np.all(uni[0] == 0.0)


def two_component_mixture():
    """One sum node over two input nodes on the same variable (K = 1): p(x) = 0.25 f_0(x) + 0.75 f_1(x)."""
    i32 = lambda a: np.asarray(a, dtype=np.int32)
    theta = np.zeros((3, 1, 1), dtype=np.float32); theta[1] = 0.25; theta[2] = 0.75
    tables = np.array([[[0.5], [0.25], [0.25]], [[0.125], [0.125], [0.75]]], dtype=np.float32)
    return W.Workload(name="mixture2", K=1, n_blocks=3, root_block=2, type=np.asarray([W.INPUT, W.INPUT, W.SUM], dtype=np.uint8),
                      n_real=i32([1, 1, 1]), child_ptr=np.asarray([0, 0, 0, 2], dtype=np.int64), child=i32([0, 1]),
                      param_blk=i32([0, 1]), n_param_blocks=2, in_var=i32([0, 0, -1]), in_table=i32([0, 1, -1]),
                      n_vars=1, n_cats=3, n_tables=2, theta=theta, tables=tables, x=i32([[0], [2], [2], [1]]))


def test_em_pseudocount_is_one_total_mass_split_evenly_hand_computed():
    """The paper prints no formula for the smoothed update ("parity unpinned" by the paper); the reading pinned here is
    Laplace smoothing with a total mass `pseudocount` per sum node / table column, split evenly over the node's edges:
    theta_new = (flow + pc / n_edges) / (sum of flows + pc).  Values below are worked by hand; adding `pc` to every
    edge instead would give (5/8, 3/8) and (4/17, 5/17, 8/17)."""
    w = two_component_mixture()
    tf = np.zeros((3, 1, 1)); tf[1] = 3.0; tf[2] = 1.0
    gf = np.zeros((2, 3, 1)); gf[0, :, 0] = (1.0, 2.0, 5.0); gf[1, :, 0] = (0.0, 0.0, 4.0)
    th, tb = orc.em_step(w, w.theta, w.tables, tf, gf, step=1.0, pseudocount=2.0)
    assert np.allclose(th[1:, 0, 0], [(3 + 1) / 6, (1 + 1) / 6], rtol=1e-6)
    assert np.allclose(tb[0, :, 0], [(1 + 2 / 3) / 10, (2 + 2 / 3) / 10, (5 + 2 / 3) / 10], rtol=1e-6)
    assert np.allclose(tb[1, :, 0], [(2 / 3) / 6, (2 / 3) / 6, (4 + 2 / 3) / 6], rtol=1e-6)
    # the full loop on the same circuit: posterior responsibilities by hand (Def. 2 on a two-component mixture)
    _, _, _, tf, gf = orc.backward(w, w.theta, w.tables, w.x)
    f = w.tables.astype(np.float64)[:, w.x[:, 0], 0]                     # [component, sample]
    post = np.array([[0.25], [0.75]]) * f
    post /= post.sum(axis=0, keepdims=True)
    assert np.allclose(tf[1:, 0, 0], post.sum(axis=1), rtol=1e-12)
    th, _ = orc.em_step(w, w.theta, w.tables, tf, gf, step=0.5, pseudocount=1.0)
    want = 0.5 * np.array([0.25, 0.75]) + 0.5 * (post.sum(axis=1) + 0.5) / (4 + 1.0)
    assert np.allclose(th[1:, 0, 0], want, rtol=1e-6)


def test_category_outside_the_table_is_outside_the_support():
    """A value outside 0..n_cats-1 has probability 0 under a categorical distribution.  Pinned two ways: against the
    same circuit with its tables widened by zero-probability categories (where the value is in range), and against
    the batch without the offending samples (a sample of probability 0 adds no flow)."""
    w = W.hclt(6, 4, 2, 9, 171, n_cats=4)
    x = w.x.copy(); x[2, 1] = w.n_cats + 2; x[5, 0] = -3
    ll, lp, flow, tf, gf = orc.backward(w, w.theta, w.tables, x)
    assert ll[2] == -np.inf and ll[5] == -np.inf and np.all(flow[2, :] == 0.0) and np.all(flow[5, :] == 0.0)
    wide = w.with_batch(np.where(x < 0, w.n_cats + 3, x))                # the negative value becomes another zero category
    wide.n_cats = w.n_cats + 4
    wide.tables = np.concatenate([w.tables, np.zeros((w.n_tables, 4, w.K), dtype=np.float32)], axis=1)
    ll2, lp2, flow2, tf2, gf2 = orc.backward(wide, wide.theta, wide.tables, wide.x)
    assert np.array_equal(ll, ll2) and np.array_equal(lp, lp2) and np.array_equal(flow, flow2) and np.array_equal(tf, tf2)
    assert np.array_equal(gf, gf2[:, :w.n_cats]) and np.all(gf2[:, w.n_cats:] == 0.0)
    keep = np.array([b for b in range(w.B) if b not in (2, 5)])
    ll3, _, _, tf3, gf3 = orc.backward(w, w.theta, w.tables, x[keep])
    assert np.array_equal(ll[keep], ll3) and np.allclose(tf, tf3, rtol=1e-13) and np.allclose(gf, gf3, rtol=1e-13)
