"""Pins of the oracle's forward pass against what the paper and the mathematics fix.

* a circuit with simplex weights defines a normalised distribution (Def. 1): brute-force sum over all
  assignments equals 1;
* marginals are a forward pass with the marginalised inputs set to 1 (Sec. 2): equals the explicit sum;
* an HMM has an equivalent circuit (footnote, Sec. 1): the textbook forward algorithm gives the same
  log-likelihood; likewise the hidden Chow-Liu tree and sum-product message passing on its latent tree;
* a block-sparse circuit equals the dense circuit whose pruned parameter blocks are zero (Sec. 4.2).
"""
import itertools

import numpy as np
import pytest
import torch

from oracle import pc_oracle as orc
from paper_2406_00766_amd import workloads as W
from tests import refs


def all_assignments(n_vars, n_cats):
    return np.array(list(itertools.product(range(n_cats), repeat=n_vars)), dtype=np.int32)


TINY = [
    lambda: W.hmm(3, 2, 3, 1, 1, 11),
    lambda: W.hmm(3, 4, 3, 2, 1, 12),
    lambda: W.hmm(4, 4, 3, 4, 1, 13, alpha_trans=0.1, alpha_emis=0.1),
    lambda: W.hclt(4, 2, 1, 1, 14, n_cats=3),
    lambda: W.hclt(5, 4, 2, 1, 15, n_cats=3),
    lambda: W.hclt(6, 3, 3, 1, 16, n_cats=2),
    lambda: W.pd(2, 1, 2, 1, 1, 17, n_cats=3),
    lambda: W.pd(2, 1, 4, 2, 1, 18, n_cats=2),
    lambda: W.pd(2, 1, 4, 2, 1, 19, n_cats=3, keep=0.4),
    lambda: W.pd(3, 1, 2, 2, 1, 20, n_cats=2, keep=0.5),
    lambda: W.pd(1, 2, 2, 2, 1, 21, n_cats=3),
]


@pytest.mark.parametrize("make", TINY)
def test_bruteforce_normalisation(make):
    w = make()
    xs = all_assignments(w.n_vars, w.n_cats)
    _, ll = orc.forward(w, w.theta, w.tables, xs)
    total = np.exp(ll).sum()
    # fp32 parameters are normalised in float64 and then rounded: rows sum to 1 within ~1e-6
    assert abs(total - 1.0) < 2e-5, total


@pytest.mark.parametrize("make", TINY[:9])
def test_marginals_equal_explicit_sums(make):
    w = make()
    rng = np.random.default_rng(5)
    for _ in range(4):
        keep = rng.random(w.n_vars) < 0.5
        obs = rng.integers(0, w.n_cats, size=w.n_vars).astype(np.int32)
        mask = (~keep).astype(np.uint8)[None, :]
        _, ll_m = orc.forward(w, w.theta, w.tables, obs[None, :], mask)
        free = np.nonzero(~keep)[0]
        xs = np.repeat(obs[None, :], w.n_cats ** len(free), axis=0)
        if len(free):
            xs[:, free] = all_assignments(len(free), w.n_cats)
        _, ll = orc.forward(w, w.theta, w.tables, xs)
        # exact only when every table column sums to 1; the fp32-rounded tables do so within ~1e-7 each
        assert np.isclose(np.exp(ll_m[0]), np.exp(ll).sum(), rtol=2e-6, atol=0)


def test_all_marginalised_is_log_one():
    w = W.hclt(5, 4, 2, 3, 15, n_cats=3)
    mask = np.ones((3, w.n_vars), dtype=np.uint8)
    _, ll = orc.forward(w, w.theta, w.tables, w.x, mask)
    assert np.allclose(ll, 0.0, atol=2e-6)


@pytest.mark.parametrize("make", [
    lambda: W.config(1),
    lambda: W.config(1, K=16),
    lambda: W.reduced(1),
    lambda: W.reduced(4),
    lambda: W.hmm(7, 6, 9, 3, 10, 31, alpha_trans=0.1, alpha_emis=0.1, tokens="zipf"),
])
def test_hmm_forward_algorithm(make):
    w = make()
    pi = w.meta["pi"].astype(np.float64)
    A = w.meta["A"].astype(np.float64)
    E = W.hmm_emission(w).astype(np.float64)
    _, ll = orc.forward(w, w.theta, w.tables, w.x)
    ref = refs.hmm_loglik_scaled(pi, A, E, w.x)
    assert np.allclose(ll, ref, rtol=1e-11, atol=0)
    ref2 = refs.hmm_loglik_torch(torch.tensor(np.log(pi)), torch.tensor(np.log(A)), torch.tensor(np.log(E)),
                                 torch.tensor(w.x, dtype=torch.long)).numpy()
    assert np.allclose(ll, ref2, rtol=1e-11, atol=0)


def _hclt_ref(w):
    D = w.meta["D"]
    log_W = [None] + [torch.tensor(np.log(W.hclt_edge_weights(w, c).astype(np.float64))) for c in range(1, D)]
    log_tab = [torch.tensor(np.log(W.hclt_table(w, v).astype(np.float64))) for v in range(D)]
    log_pi = torch.tensor(np.log(w.meta["pi"].astype(np.float64)))
    return log_pi, log_W, log_tab


@pytest.mark.parametrize("make", [
    lambda: W.reduced(2),
    lambda: W.reduced(3),
    lambda: W.hclt(9, 6, 2, 12, 33, n_cats=5),
])
def test_hclt_message_passing(make):
    w = make()
    log_pi, log_W, log_tab = _hclt_ref(w)
    ref = refs.latent_tree_loglik_torch(w.meta["parent"], w.meta["order"], log_pi, log_W, log_tab,
                                        torch.tensor(w.x, dtype=torch.long)).numpy()
    _, ll = orc.forward(w, w.theta, w.tables, w.x)
    assert np.allclose(ll, ref, rtol=1e-11, atol=0)


def test_hclt_single_latent_state_factorises():
    w = W.hclt(7, 1, 1, 9, 34, n_cats=4)
    _, ll = orc.forward(w, w.theta, w.tables, w.x)
    ref = np.zeros(w.B)
    for v in range(7):
        ref += np.log(W.hclt_table(w, v).astype(np.float64)[0, w.x[:, v]])
    # theta is the 1x1 weight 1.0 everywhere
    assert np.allclose(ll, ref, rtol=1e-12, atol=0)


def test_pruned_equals_dense_with_zero_blocks():
    dense = W.pd(3, 1, 4, 2, 20, 41, n_cats=3)
    rng = np.random.default_rng(3)
    # drop a random subset of sum edges (keep the first edge of every sum block)
    drop = np.zeros(dense.n_edges, dtype=bool)
    for u in np.nonzero(dense.type == W.SUM)[0]:
        e0, e1 = dense.child_ptr[u], dense.child_ptr[u + 1]
        drop[e0 + 1:e1] = rng.random(e1 - e0 - 1) < 0.5
    theta_zero = dense.theta.copy()
    theta_zero[dense.param_blk[drop] + 1] = 0.0
    _, ll_zero = orc.forward(dense, theta_zero, dense.tables, dense.x)

    keep = ~drop
    new_ptr = np.zeros_like(dense.child_ptr)
    new_ptr[1:] = np.cumsum([keep[dense.child_ptr[u]:dense.child_ptr[u + 1]].sum() for u in range(dense.n_blocks)])
    pruned = dense.with_batch(dense.x)
    pruned.child_ptr = new_ptr
    pruned.child = dense.child[keep].copy()
    pruned.param_blk = dense.param_blk[keep].copy()
    _, ll_pruned = orc.forward(pruned, dense.theta, dense.tables, dense.x)
    assert np.allclose(ll_zero, ll_pruned, rtol=1e-13, atol=0)
    assert drop.sum() > 0


def test_zero_probability_sample_gives_minus_inf():
    w = W.hmm(3, 2, 3, 2, 4, 51)
    tables = w.tables.copy()
    tables[:, 0, :] = 0.0                       # token 0 impossible under every state
    x = w.x.copy(); x[0, 1] = 0; x[1:] = np.where(x[1:] == 0, 1, x[1:])
    _, ll = orc.forward(w, w.theta, tables, x)
    assert ll[0] == -np.inf and np.all(np.isfinite(ll[1:]))


def test_cycle_is_rejected():
    w = W.hmm(3, 2, 3, 2, 1, 52)
    # make the first product block a child of ... itself through its sum: add edge input<-? not allowed,
    # so rewire: product P_2 gets S_1 as child, which (through P_1 -> S_2 -> P_2) closes a cycle.
    bad = w.with_batch(w.x)
    child = w.child.copy()
    # locate P_{T-1} (single child) and point it at the root
    u = [b for b in range(w.n_blocks) if w.type[b] == W.PRODUCT and w.child_ptr[b + 1] - w.child_ptr[b] == 1][0]
    child[w.child_ptr[u]] = w.root_block
    bad.child = child
    with pytest.raises(ValueError):
        orc.forward(bad, w.theta, w.tables, w.x)
