"""RAT-SPN workload: the oracle against what holds for any normalised smooth and decomposable circuit.

No closed form exists for this structure, so the pins are brute force: probabilities of all assignments sum to one,
a marginalised forward pass equals the explicit sum over the marginalised variables, and per sample the input-node
flows of every variable sum to one (each variable is decided exactly once on every path from the root, Def. 2).
"""
import itertools

import numpy as np
import pytest

from oracle import compile_oracle as co
from oracle import pc_oracle as orc
from paper_2406_00766_amd import workloads as W


@pytest.mark.parametrize("D,depth,R,S,K,n_cats", [(4, 1, 2, 4, 2, 3), (8, 2, 2, 4, 2, 2), (8, 3, 1, 6, 3, 2), (6, 1, 3, 2, 1, 2)])
def test_all_assignments_sum_to_one(D, depth, R, S, K, n_cats):
    w = W.rat_spn(D, depth, R, S, K, 3, 11, n_cats=n_cats, data="uniform")
    xs = np.array(list(itertools.product(range(n_cats), repeat=D)), dtype=np.int32)
    _, ll = orc.forward(w.with_batch(xs), w.theta, w.tables, xs)
    assert abs(np.exp(ll).sum() - 1.0) < 1e-6


def test_marginal_equals_explicit_sum():
    w = W.rat_spn(6, 1, 2, 4, 2, 3, 12, n_cats=3, data="uniform")
    x = np.array([[0, 1, 2, 0, 1, 2]], dtype=np.int32)
    mask = np.array([[0, 1, 0, 0, 1, 0]], dtype=np.uint8)
    _, ll_m = orc.forward(w.with_batch(x), w.theta, w.tables, x, mask)
    tot = 0.0
    for a in range(3):
        for b in range(3):
            y = x.copy(); y[0, 1] = a; y[0, 4] = b
            tot += np.exp(orc.forward(w.with_batch(y), w.theta, w.tables, y)[1][0])
    np.testing.assert_allclose(np.exp(ll_m[0]), tot, rtol=2e-6)


def test_input_flows_of_each_variable_sum_to_one():
    w = W.rat_spn(8, 2, 3, 8, 4, 9, 13, n_cats=4, data="uniform")
    ll, lp, flow, tf, gf = orc.backward(w, w.theta, w.tables, w.x, None)
    K = w.K
    per_var = np.zeros((w.B, w.n_vars))
    for u in np.nonzero(w.type == W.INPUT)[0]:
        per_var[:, w.in_var[u]] += flow[:, u * K:(u + 1) * K].sum(axis=1)
    np.testing.assert_allclose(per_var, 1.0, rtol=1e-9)
    # the table flows hold exactly these flows, at the observed categories
    np.testing.assert_allclose(gf.sum(), w.B * w.n_vars, rtol=1e-9)


def test_structure_counts_and_compile():
    w = W.rat_spn(16, 2, 2, 8, 4, 2, 14, n_cats=3, draw=False)
    nb = 2
    # per replica: 1 top region (no sums) + 2 regions with sums; every region has nb^2 product blocks
    assert int((w.type == W.PRODUCT).sum()) == 2 * 3 * nb * nb
    assert int((w.type == W.SUM).sum()) == 2 * 2 * nb + 1
    tabs = co.compile_tables(w)
    kinds = [L["kind"] for L in tabs["layers"]]
    assert kinds == [0, 1, 2, 1, 2]                       # inputs, products, sums, top products, root
