"""Collapse of consecutive sum / sum and product / product blocks (footnote to Def. 2).

Pins of the oracle's collapse (oracle/compile_oracle.collapse): the collapsed circuit computes the same function as
the original DAG -- checked by brute force over every assignment with the node-by-node oracle forward pass, which
evaluates any DAG of sum, product and input nodes straight from Def. 1 --, a hand-computed two-level example, and the
result alternates.  The library's pc_collapse (host C++) must produce the same DAG bit for bit.
"""
import itertools
import types

import numpy as np
import pytest

from oracle import compile_oracle as co
from oracle import pc_oracle as orc
from paper_2406_00766_amd import binding as pcb
from paper_2406_00766_amd import workloads as W


def alternates(c):
    for u in range(c.n_blocks):
        for e in range(int(c.child_ptr[u]), int(c.child_ptr[u + 1])):
            k = c.type[c.child[e]]
            if (c.type[u] == W.SUM and k != W.PRODUCT) or (c.type[u] == W.PRODUCT and k == W.PRODUCT):
                return False
    return True


def all_assignments(n_vars, n_cats):
    return np.array(list(itertools.product(range(n_cats), repeat=n_vars)), dtype=np.int32)


@pytest.mark.parametrize("seed,K", [(900, 1), (901, 2), (904, 2), (905, 3), (911, 1), (912, 4)])
def test_collapsed_random_dag_computes_the_same_function(seed, K):
    w = W.non_alternating(3, 4, 4, K, 4, seed, n_cats=3)
    assert not alternates(w)
    c = co.collapse(w, w.theta)
    assert alternates(c)
    X = all_assignments(3, 3)
    ll0 = orc.forward(w, w.theta, w.tables, X)[1]
    ll1 = orc.forward(c, c.theta, w.tables, X)[1]
    assert np.allclose(ll0, ll1, rtol=0, atol=1e-6)          # the merged weights are rounded to fp32 once


def test_collapsed_tree_circuit_stays_normalised():
    base = W.hclt(4, 4, 2, 5, 77, n_cats=3)
    w = W.non_alternating_from(base, 5)
    c = co.collapse(w, w.theta)
    X = all_assignments(4, 3)
    p0 = np.exp(orc.forward(w, w.theta, w.tables, X)[1])
    p1 = np.exp(orc.forward(c, c.theta, w.tables, X)[1])
    assert abs(p0.sum() - 1.0) < 1e-6 and abs(p1.sum() - 1.0) < 1e-6
    assert np.allclose(p0, p1, rtol=1e-6)


def test_two_level_example_by_hand():
    """K = 1.  root = 0.25 a + 0.75 t,  t = 0.4 a + 0.6 b  (a, b products over one input each, t a sum under a sum):
    collapsed root = (0.25 + 0.75 * 0.4) a + (0.75 * 0.6) b = 0.55 a + 0.45 b."""
    w = types.SimpleNamespace(
        K=1, n_blocks=6, root_block=5, type=np.array([0, 0, 1, 1, 2, 2], dtype=np.uint8), n_real=np.ones(6, dtype=np.int32),
        child_ptr=np.array([0, 0, 0, 1, 2, 4, 6], dtype=np.int64), child=np.array([0, 1, 2, 3, 2, 4], dtype=np.int32),
        param_blk=np.array([-1, -1, 0, 1, 2, 3], dtype=np.int32), n_param_blocks=4,
        in_var=np.array([0, 1, -1, -1, -1, -1], dtype=np.int32), in_table=np.array([0, 1, -1, -1, -1, -1], dtype=np.int32),
        n_vars=2, n_cats=2, n_tables=2, max_groups=8, tol_permille=250,
        theta=np.array([0, 0.4, 0.6, 0.25, 0.75], dtype=np.float32).reshape(5, 1, 1))
    c = co.collapse(w, w.theta)
    assert c.n_blocks == 5 and list(c.block_map) == [0, 1, 2, 3, -1, 4]
    assert list(c.child[c.child_ptr[4]:c.child_ptr[5]]) == [2, 3]
    got = [float(c.theta[p + 1, 0, 0]) for p in c.param_blk[c.child_ptr[4]:c.child_ptr[5]]]
    assert np.allclose(got, [0.55, 0.45], rtol=1e-6)


@pytest.mark.parametrize("make", [
    lambda: W.non_alternating(4, 4, 4, 4, 5, 900),
    lambda: W.non_alternating(5, 5, 5, 32, 5, 913),
    lambda: W.non_alternating_from(W.reduced(2), 6),
    lambda: W.non_alternating_from(W.reduced(5), 7),
    lambda: W.reduced(1),                                     # already alternating and tied: nothing changes, ties kept
])
def test_library_collapse_equals_the_oracle_collapse(make):
    w = make()
    a, b = co.collapse(w, w.theta), pcb.pc_collapse(w)
    for k in ("type", "n_real", "child_ptr", "child", "param_blk", "in_var", "in_table", "block_map"):
        assert np.array_equal(getattr(a, k), getattr(b, k)), k
    assert (a.n_blocks, a.root_block, a.n_param_blocks) == (b.n_blocks, b.root_block, b.n_param_blocks)
    assert np.allclose(a.theta, b.theta, rtol=1e-6, atol=0)
    if w.meta.get("kind") != "non_alternating":
        assert np.array_equal(b.child, w.child) and np.array_equal(b.param_blk, w.param_blk) and np.array_equal(b.theta, w.theta)
    # the default compile refuses the original and takes the collapsed DAG
    if not alternates(w):
        with pytest.raises(pcb.PcError) as e:
            pcb.pc_compile(w, host_only=True)
        assert e.value.status_name == "PC_ERR_NOT_ALTERNATING"
    pcb.pc_destroy(pcb.pc_compile(b, host_only=True))


def test_collapse_error_paths():
    w = W.non_alternating(3, 3, 3, 2, 4, 901)
    # a product block that reaches the same child through two product children
    p = [u for u in range(w.n_blocks) if w.type[u] == W.INPUT][0]
    n = w.n_blocks
    w2 = w.with_batch(w.x)
    w2.n_blocks = n + 3
    w2.type = np.append(w.type, np.array([W.PRODUCT] * 3, dtype=np.uint8))
    w2.n_real = np.append(w.n_real, np.full(3, w.K, dtype=np.int32))
    w2.in_var = np.append(w.in_var, np.full(3, -1, dtype=np.int32)); w2.in_table = np.append(w.in_table, np.full(3, -1, dtype=np.int32))
    w2.child_ptr = np.append(w.child_ptr, w.child_ptr[-1] + np.array([1, 2, 4]))
    w2.child = np.append(w.child, np.array([p, p, n, n + 1], dtype=np.int32))
    w2.param_blk = np.append(w.param_blk, np.full(4, -1, dtype=np.int32))
    w2.root_block = n + 2                                     # a product root is enough for the collapse itself
    with pytest.raises(pcb.PcError) as e:
        pcb.pc_collapse(w2)
    assert e.value.status_name == "PC_ERR_NOT_BLOCK_SPARSE"
    with pytest.raises(co.CompileError):
        co.collapse(w2, w2.theta)
    # a cycle: a sum block that is its own child
    w3 = w.with_batch(w.x)
    w3.child = w.child.copy()
    s = [u for u in range(w.n_blocks) if w.type[u] == W.SUM and w.child_ptr[u + 1] > w.child_ptr[u]][0]
    w3.child[w.child_ptr[s]] = s
    with pytest.raises(pcb.PcError) as e:
        pcb.pc_collapse(w3)
    assert e.value.status_name == "PC_ERR_CYCLE"
