"""The wide block-sparse sum layer (App. C.1) as a workload: the oracle against the closed form of that circuit.

The circuit is p(x) = sum_k pi[k] prod_s S_s[k](x_s) with S_s(x_s) = W_s e_s(x_s); W_s is the dense [M, M]
matrix with zeros where edge blocks were dropped and e_s(x_s)[j] the categorical table entry of input node j.
Forward values and all flows therefore have closed forms in dense linear algebra, written out here.
"""
import numpy as np
import pytest

from oracle import compile_oracle as co
from oracle import pc_oracle as orc
from paper_2406_00766_amd import workloads as W


def closed_form(w):
    K, M, n_sets = w.K, w.meta["M"], w.meta["n_sets"]
    nb = M // K
    B = w.B
    Ws = [W.sum_layer_dense(w, s) for s in range(n_sets)]
    e = []
    for s in range(n_sets):
        T = np.concatenate([w.tables[s * nb + j].astype(np.float64) for j in range(nb)], axis=1)   # [cats, M]
        e.append(T[w.x[:, s]])                                                                       # [B, M]
    S = [e[s] @ Ws[s].T for s in range(n_sets)]                                                       # [B, M]
    pi = np.concatenate([w.theta[w.n_param_blocks - nb + 1 + j][0] for j in range(nb)]).astype(np.float64)
    prod = np.ones((B, M))
    for s in range(n_sets):
        prod *= S[s]
    p = prod @ pi
    post = prod * pi[None, :] / p[:, None]                 # flow of T[k] = flow of every S_s[k]
    G = [np.einsum("bi,ij,bj->ij", post / S[s], Ws[s], e[s]) for s in range(n_sets)]
    return np.log(p), post, G, e, Ws, S


@pytest.mark.parametrize("K,keep", [(4, 1.0), (4, 0.4), (1, 0.5), (8, 0.2)])
def test_oracle_matches_dense_closed_form(K, keep):
    w = W.sum_layer(3, 16, K, 21, 77, keep=keep, n_cats=5)
    ll, lp, flow, tf, gf = orc.backward(w, w.theta, w.tables, w.x, None)
    ref_ll, post, G, e, Ws, S = closed_form(w)
    np.testing.assert_allclose(ll, ref_ll, rtol=1e-12, atol=1e-12)
    nb = 16 // K
    S0, P0 = w.meta["S0"], w.meta["P0"]
    for s in range(3):
        got_S = lp[:, (S0 + s * nb) * K:(S0 + (s + 1) * nb) * K]
        np.testing.assert_allclose(got_S, np.log(S[s]), rtol=1e-12, atol=1e-12)
        got_F = flow[:, (S0 + s * nb) * K:(S0 + (s + 1) * nb) * K]
        np.testing.assert_allclose(got_F, post, rtol=1e-10, atol=1e-14)
        # flow of product node j of set s: sum_i post[i] W[i, j] e[j] / S[i]
        ref_P = np.einsum("bi,ij,bj->bj", post / S[s], Ws[s], e[s])
        got_P = flow[:, (P0 + s * nb) * K:(P0 + (s + 1) * nb) * K]
        np.testing.assert_allclose(got_P, ref_P, rtol=1e-10, atol=1e-14)
        # parameter flows, block by block
        for i in range(nb):
            u = S0 + s * nb + i
            for ed in range(int(w.child_ptr[u]), int(w.child_ptr[u + 1])):
                j = int(w.child[ed]) - P0 - s * nb
                np.testing.assert_allclose(tf[int(w.param_blk[ed]) + 1], G[s][i * K:(i + 1) * K, j * K:(j + 1) * K],
                                           rtol=1e-10, atol=1e-14)


def test_every_sum_node_keeps_a_child_and_edge_count():
    w = W.sum_layer(7, 64, 8, 3, 5, keep=0.05, n_cats=4)
    nb = 8
    S0 = w.meta["S0"]
    deg = np.diff(w.child_ptr)[S0:S0 + 7 * nb]
    assert deg.min() >= 1
    assert w.meta["n_layer_edges"] == int(deg.sum()) * 64
    dense = W.sum_layer(7, 64, 8, 3, 5, n_cats=4)
    assert dense.meta["n_layer_edges"] == 7 * 64 * 64
    # rows of every set are normalised over the kept blocks
    for s in range(7):
        np.testing.assert_allclose(W.sum_layer_dense(w, s).sum(axis=1), 1.0, rtol=1e-5)


def test_compile_groups_follow_child_counts():
    w = W.sum_layer(6, 128, 8, 4, 9, keep=0.3, draw=False)
    tabs = co.compile_tables(w)
    layer = [L for L in tabs["layers"] if L["kind"] == 2][0]          # the wide sum layer
    widths = [np.asarray(g[1]).shape[1] for g in layer["fwd"]]
    assert widths == sorted(widths) and len(widths) >= 2
    counts = np.diff(w.child_ptr)[w.meta["S0"]:w.meta["T0"]]
    assert widths[-1] == counts.max()
    total = sum(np.asarray(g[1]).size for g in layer["fwd"])
    assert total <= counts.sum() + -(-counts.sum() * w.tol_permille // 1000)
