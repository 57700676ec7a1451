"""Pins of the compile oracle: Alg. 2 (App. A.1) and the index tensors (Sec. 4.3, App. A.2)."""
import itertools
import json
import os

import numpy as np
import pytest

from oracle import compile_oracle as co
from paper_2406_00766_amd import workloads as W

HERE = os.path.dirname(os.path.abspath(__file__))


def brute_force_best(nchs, n_groups):
    """Optimal overhead with at most n_groups capacities, by enumeration (App. A.1's optimality claim)."""
    uni = sorted(set(nchs))
    best = None
    for r in range(1, min(n_groups, len(uni)) + 1):
        for caps in itertools.combinations(uni, r):
            if caps[-1] != uni[-1]:
                continue
            c = co.overhead(nchs, caps)
            best = c if best is None else min(best, c)
    return best


def test_alg2_matches_brute_force():
    rng = np.random.default_rng(0)
    for trial in range(300):
        n = int(rng.integers(1, 30))
        nchs = rng.integers(1, int(rng.integers(2, 12)), size=n).tolist()
        G = int(rng.integers(1, 7))
        tol = int(rng.choice([0, 50, 100, 250, 500, 1000]))
        caps = co.partition_groups(nchs, G, tol)
        total = sum(nchs)
        target = total + -(-total * tol // 1000)
        assert caps == sorted(set(caps)) and caps[-1] == max(nchs) and len(caps) <= G
        got = co.overhead(nchs, caps)
        # the fewest groups that meet the target, at that group count's optimal overhead
        feasible = [g for g in range(1, G + 1) if brute_force_best(nchs, g) <= target]
        if feasible:
            g = feasible[0]
            assert got <= target
            assert got == brute_force_best(nchs, g), (nchs, G, tol, caps)
            assert len(caps) <= g
            if g > 1:
                assert brute_force_best(nchs, g - 1) > target
        else:
            assert got == brute_force_best(nchs, G)


def test_alg2_special_cases():
    assert co.partition_groups([5] * 9, 8, 250) == [5]
    assert co.partition_groups([1, 2, 3, 9], 1, 0) == [9]
    assert co.partition_groups([1, 1, 1, 100], 8, 250) == [1, 100]
    assert co.partition_groups([3, 1, 2], 8, 0) == [1, 2, 3]
    assert co.partition_groups([], 8, 250) == []
    # tolerance large enough for one group
    assert co.partition_groups([1, 2], 8, 1000) == [2]


def _fig4_workload():
    spec = json.load(open(os.path.join(HERE, "golden", "fig4_layer.json")))
    K = spec["K"]
    from paper_2406_00766_amd.workloads import _Builder, _make, INPUT, PRODUCT, SUM
    bld = _Builder(K)
    ids = {}
    for i, name in enumerate(spec["product_blocks"]):
        e = bld.add(INPUT, var=i, table=i)
        ids[name] = bld.add(PRODUCT)
        bld.link(ids[name], e)
    p = 0
    for name, chs in spec["sum_blocks"].items():
        ids[name] = bld.add(SUM)
        for c in chs:
            bld.link(ids[name], ids[c], p)
            p += 1
    # a root on top so that the DAG is a legal circuit: products over each sum block, then one sum
    tops = []
    for name in spec["sum_blocks"]:
        t = bld.add(PRODUCT)
        bld.link(t, ids[name])
        tops.append(t)
    root = bld.add(SUM, n_real=1)
    for t in tops:
        bld.link(root, t, p)
        p += 1
    theta = np.zeros((p + 1, K, K), dtype=np.float32)
    tables = np.full((3, 2, K), 0.5, dtype=np.float32)
    w = _make("fig4", bld, root, p, 3, 2, 3, theta, tables, np.zeros((1, 3), dtype=np.int32), {})
    return spec, ids, w


def test_fig4_example_groups_and_index_tensors():
    spec, ids, w = _fig4_workload()
    K = spec["K"]
    comp = co.compile_tables(w)
    off = {name: (u + 1) * K for name, u in ids.items()}
    layer = [l for l in comp["layers"] if l["kind"] == co.SUM and l["depth"] == 2][0]
    assert len(layer["fwd"]) == len(spec["expected_groups"])
    for (sum_ids, prod_ids, param_ids), exp in zip(layer["fwd"], spec["expected_groups"]):
        assert prod_ids.shape == (len(exp["sum_ids"]), exp["capacity"])
        assert sum_ids.tolist() == [off[n] for n in exp["sum_ids"]]
        assert prod_ids.tolist() == [[off[n] for n in row] for row in exp["prod_ids"]]
        assert np.all(param_ids > 0) and len(set(param_ids.ravel().tolist())) == param_ids.size
    # backward compilation by parent count (App. A.2): n01 has two parents, n23 and n45 one each
    bwd = layer["bwd"]
    assert [g[1].shape for g in bwd] == [(2, 1), (1, 2)]
    assert bwd[0][0].tolist() == [off["n23"], off["n45"]] and bwd[1][0].tolist() == [off["n01"]]
    assert bwd[0][1].tolist() == [[off["m23"]], [off["m45"]]] and bwd[1][1].tolist() == [[off["m01"], off["m23"]]]


def _edges_from_tables(groups, with_params):
    out = []
    for ids, nbr, par in groups:
        assert nbr.shape == par.shape and nbr.shape[0] == len(ids)
        for r in range(len(ids)):
            row = nbr[r]
            real = row[row > 0]
            assert np.all(np.diff(real) > 0), "neighbours ascending"
            assert np.all(row[len(real):] == 0) and np.all(par[r, len(real):] == 0), "padding at the end, zeros"
            for j in range(len(real)):
                out.append((int(ids[r]), int(row[j]), int(par[r, j]) if with_params else 0))
        assert np.all(np.diff(ids) > 0), "rows ascending inside a group"
    return out


@pytest.mark.parametrize("make", [lambda: W.reduced(i) for i in range(1, 6)] + [lambda: W.config(1), lambda: W.config(2)])
def test_table_invariants(make):
    w = make()
    K = w.K
    comp = co.compile_tables(w)
    depth = co.block_depths(w)
    seen = set()
    for layer in comp["layers"]:
        if layer["kind"] == co.INPUT:
            ids, var, tab = layer["fwd"][0]
            us = ids // K - 1
            assert np.all(w.type[us] == W.INPUT) and np.all(np.diff(ids) > 0)
            assert np.array_equal(var, w.in_var[us]) and np.array_equal(tab, w.in_table[us])
            assert len(ids) == int((w.type == W.INPUT).sum())
            continue
        is_sum = layer["kind"] == co.SUM
        fwd = _edges_from_tables(layer["fwd"], is_sum)
        bwd = _edges_from_tables(layer["bwd"], is_sum)
        # every real block edge of the layer exactly once in the forward and once in the backward tables
        truth = []
        for u in range(w.n_blocks):
            if depth[u] == layer["depth"] and w.type[u] == layer["kind"]:
                for e in range(w.child_ptr[u], w.child_ptr[u + 1]):
                    truth.append(((u + 1) * K, (int(w.child[e]) + 1) * K,
                                  (int(w.param_blk[e]) + 1) * K * K if is_sum else 0))
        assert sorted(fwd) == sorted(truth)
        assert sorted((p, c, t) for (c, p, t) in bwd) == sorted(truth)
        assert len(set(truth)) == len(truth)
        # padding stays within the tolerance whenever fewer than max_groups groups were needed
        for groups in (layer["fwd"], layer["bwd"]):
            cells = sum(g[1].size for g in groups)
            real = sum(int((g[1] > 0).sum()) for g in groups)
            if len(groups) < w.max_groups:
                assert cells <= real + -(-real * w.tol_permille // 1000)
            caps = [g[1].shape[1] for g in groups]
            assert caps == sorted(set(caps))
        key = (layer["kind"], layer["depth"])
        assert key not in seen
        seen.add(key)
    kinds = [(l["depth"], l["kind"]) for l in comp["layers"]]
    assert kinds == sorted(kinds)
    assert comp["n_rows"] == (w.n_blocks + 1) * K


@pytest.mark.parametrize("make", [lambda: W.reduced(i) for i in range(1, 7)] +
                         [lambda: W.random_circuit(5, 4, 3, 2, 3, 311), lambda: W.random_circuit(6, 6, 4, 4, 3, 312),
                          lambda: W.config(2, draw=False)])
def test_depth_is_the_longest_path_and_children_run_in_earlier_layers(make):
    """Sec. 3 layering: a block can be evaluated once all its children have been, so every child must sit in a layer
    that runs earlier.  The depth itself is pinned against a brute-force longest path to an input block (memoised
    recursion over the children lists, written independently of the oracle's pass)."""
    import functools
    import sys
    w = make()
    depth = co.block_depths(w)
    sys.setrecursionlimit(max(sys.getrecursionlimit(), 4 * w.n_blocks + 1000))

    @functools.lru_cache(maxsize=None)
    def longest(u):
        ch = w.child[w.child_ptr[u]:w.child_ptr[u + 1]]
        return 0 if len(ch) == 0 else 1 + max(longest(int(c)) for c in ch)

    assert [longest(u) for u in range(w.n_blocks)] == [int(d) for d in depth]
    comp = co.compile_tables(w)
    position = {(l["kind"], l["depth"]): i for i, l in enumerate(comp["layers"])}
    for u in range(w.n_blocks):
        mine = position[(int(w.type[u]), int(depth[u]) if w.type[u] != W.INPUT else comp["layers"][0]["depth"])]
        for c in w.child[w.child_ptr[u]:w.child_ptr[u + 1]]:
            kind_c = int(w.type[c])
            theirs = position[(kind_c, int(depth[c]) if kind_c != W.INPUT else comp["layers"][0]["depth"])]
            assert depth[c] < depth[u] and theirs < mine


def test_validation_errors():
    w = W.hmm(3, 2, 3, 2, 1, 52)
    bad = w.with_batch(w.x)
    child = w.child.copy()
    u = [b for b in range(w.n_blocks) if w.type[b] == W.PRODUCT and w.child_ptr[b + 1] - w.child_ptr[b] == 1][0]
    child[w.child_ptr[u]] = w.root_block
    bad.child = child
    with pytest.raises(co.CompileError):
        co.compile_tables(bad)
    # a sum block whose child is an input block breaks the sum/product alternation (Def. 2's assumption)
    bad2 = w.with_batch(w.x)
    child2 = w.child.copy()
    s = int(np.nonzero(w.type == W.SUM)[0][0])
    child2[w.child_ptr[s]] = int(np.nonzero(w.type == W.INPUT)[0][0])
    bad2.child = child2
    with pytest.raises(co.CompileError):
        co.compile_tables(bad2)
