"""TEST INFRASTRUCTURE ONLY: plain-Python oracle of the layer compiler (integer results).

What the paper fixes:  nodes are layered by topological depth, leaves first (Sec. 3); the node
blocks of a layer are partitioned into groups of similar child-block count by the dynamic
programme of App. A.1 (Alg. 2), padded with pseudo blocks of probability 0 (Sec. 4.3); per group
the index tensors sum_ids [C_M], prod_ids / param_ids [C_M, C_N] are recorded (Sec. 4.3), and a
second compilation by parent count gives ch_ids [C_N], par_ids / par_param_ids [C_N, C_M] for the
backward pass (App. A.2).

What the paper leaves open is fixed here as one canonical form (the GPU library follows the same
written rules; the two share no code):
  * node offset of block u is (u+1)*K; offset 0 is a null block (log-prob 0, flow 0);
    parameter block p starts at (p+1)*K*K; parameter offset 0 is an all-zero block; padding
    entries are node offset 0 / parameter offset 0.
  * depth(input) = 0, depth(n) = 1 + max depth(children) (longest path).  Layers: all input
    blocks; then for d = 1, 2, ...: the product blocks of depth d, then the sum blocks of depth d.
  * inside a layer blocks ascend by id; a block joins the smallest group capacity >= its count;
    inside a group blocks keep ascending; a row lists its neighbours in ascending node offset.
  * product layers get the same two table sets as sum layers (children per product block,
    product parents per child block), without parameter ids.
  * Alg. 2 as printed returns the largest feasible group count, never tries a single group and
    backtracks along one column; the reading used here: try n = 1, 2, ..., G and stop at the first
    n whose optimal overhead is <= sum + ceil(sum * tol), else use G; backtrack through columns
    n, n-1, ...; capacities are the distinct values found; all arithmetic in integers; ties keep
    the smallest split index (strict '<' in the printed inner loop).
"""
from __future__ import annotations

import numpy as np

INPUT, PRODUCT, SUM = 0, 1, 2


class CompileError(ValueError):
    pass


def partition_groups(nchs, max_groups: int, tol_permille: int) -> list[int]:
    """App. A.1, Alg. 2: group capacities (ascending) for a layer with child counts `nchs`."""
    nchs = [int(v) for v in nchs]
    if not nchs:
        return []
    uni = sorted(set(nchs))
    counts = [0] * len(uni)
    pos = {v: i for i, v in enumerate(uni)}
    for v in nchs:
        counts[pos[v]] += 1
    L = len(uni)
    G = max(1, int(max_groups))
    total = sum(u * c for u, c in zip(uni, counts))
    target = total + (total * int(tol_permille) + 999) // 1000
    cum = []
    s = 0
    for c in counts:
        s += c
        cum.append(s)

    dp = [[0] * (G + 1) for _ in range(L)]
    bt = [[0] * (G + 1) for _ in range(L)]
    for i in range(L):
        dp[i][1] = uni[i] * cum[i]
    n_sel = G
    if dp[L - 1][1] <= target:
        n_sel = 1
    else:
        for n in range(2, G + 1):
            dp[0][n] = uni[0] * cum[0]
            bt[0][n] = 0
            for i in range(1, L):
                best, best_j = None, -1
                for j in range(i):
                    cur = dp[j][n - 1] + uni[i] * (cum[i] - cum[j])
                    if best is None or cur < best:
                        best, best_j = cur, j
                dp[i][n] = best
                bt[i][n] = best_j
            if dp[L - 1][n] <= target:
                n_sel = n
                break
    caps = set()
    i = L - 1
    for n in range(n_sel, 0, -1):
        caps.add(uni[i])
        if n > 1:
            i = bt[i][n]
    return sorted(caps)


def overhead(nchs, caps) -> int:
    """Cost of a partitioning (App. A.1): every count is padded to the smallest capacity holding it."""
    tot = 0
    for v in nchs:
        tot += min(c for c in caps if c >= v)
    return tot


def block_depths(w) -> np.ndarray:
    """Longest-path depth of every block; validates the DAG (acyclic, sum/product alternation)."""
    n = w.n_blocks
    typ, ptr, child = w.type, w.child_ptr, w.child
    depth = np.full(n, -1, dtype=np.int64)
    state = np.zeros(n, dtype=np.int8)
    for s in range(n):
        if state[s]:
            continue
        stack = [(s, int(ptr[s]))]
        state[s] = 1
        while stack:
            u, e = stack[-1]
            if e < ptr[u + 1]:
                stack[-1] = (u, e + 1)
                c = int(child[e])
                if c < 0 or c >= n:
                    raise CompileError("child id out of range")
                if state[c] == 1:
                    raise CompileError("cycle")
                if state[c] == 0:
                    state[c] = 1
                    stack.append((c, int(ptr[c])))
            else:
                stack.pop()
                state[u] = 2
                ch = child[ptr[u]:ptr[u + 1]]
                if typ[u] == INPUT:
                    if len(ch):
                        raise CompileError("input block with children")
                    depth[u] = 0
                else:
                    if len(ch) == 0:
                        raise CompileError("inner block without children")
                    if len(set(int(c) for c in ch)) != len(ch):
                        raise CompileError("duplicate child block")
                    if typ[u] == SUM and any(typ[c] != PRODUCT for c in ch):
                        raise CompileError("sum block with a non-product child")
                    if typ[u] == PRODUCT and any(typ[c] == PRODUCT for c in ch):
                        raise CompileError("product block with a product child")
                    depth[u] = 1 + max(int(depth[c]) for c in ch)
    return depth


def _grouped_tables(rows, max_groups, tol_permille):
    """rows: list of (row_id_offset, [(nbr_offset, param_offset), ...]) in ascending row id.
    Returns a list of groups, each (ids[R], nbr[R, C], par[R, C]) int32, ascending capacity."""
    caps = partition_groups([len(r[1]) for r in rows], max_groups, tol_permille)
    groups = []
    for cap in caps:
        lower = max([c for c in caps if c < cap], default=0)
        sel = [r for r in rows if lower < len(r[1]) <= cap]
        ids = np.array([r[0] for r in sel], dtype=np.int64)
        nbr = np.zeros((len(sel), cap), dtype=np.int64)
        par = np.zeros((len(sel), cap), dtype=np.int64)
        for i, (_, lst) in enumerate(sel):
            lst = sorted(lst)
            for j, (a, p) in enumerate(lst):
                nbr[i, j] = a
                par[i, j] = p
        for arr in (ids, nbr, par):
            if arr.size and arr.max() > np.iinfo(np.int32).max:
                raise CompileError("index overflow")
        groups.append((ids.astype(np.int32), nbr.astype(np.int32), par.astype(np.int32)))
    return groups


def compile_tables(w) -> dict:
    """Returns {'K', 'n_rows', 'layers': [ {kind, depth, fwd: [...], bwd: [...]} ]}.

    Input layer: fwd = [(ids, var, table)], bwd = [].
    Product / sum layer: fwd groups (ids, nbr_ids, param_ids) by child count, bwd groups
    (ch_ids, par_ids, par_param_ids) by parent count (param ids all 0 for product layers).
    """
    K = int(w.K)
    depth = block_depths(w)
    if w.type[w.root_block] != SUM:
        raise CompileError("root must be a sum block")
    if int(getattr(w, "product_scratch", 0)):
        # Sec. 5, product values recomputed: a product block is evaluated as late as possible, in the layer right before
        # the sum blocks that read it (all of one depth d: the block moves to depth d, and product layers come before
        # sum layers inside a depth); product blocks nobody reads form a last layer of their own
        readers: dict[int, set] = {}
        for u in range(w.n_blocks):
            if w.type[u] == SUM:
                for e in range(int(w.child_ptr[u]), int(w.child_ptr[u + 1])):
                    readers.setdefault(int(w.child[e]), set()).add(int(depth[u]))
        last = int(depth.max()) + 1
        for u in range(w.n_blocks):
            if w.type[u] == PRODUCT:
                ds = readers.get(u, {last})
                if len(ds) != 1:
                    raise CompileError("product block read by sum blocks of different depths")
                depth[u] = next(iter(ds))
    node_off = lambda u: (int(u) + 1) * K
    par_off = lambda p: (int(p) + 1) * K * K
    layers = []
    inputs = [u for u in range(w.n_blocks) if w.type[u] == INPUT]
    layers.append({
        "kind": INPUT, "depth": 0,
        "fwd": [(np.array([node_off(u) for u in inputs], dtype=np.int32),
                 np.array([w.in_var[u] for u in inputs], dtype=np.int32),
                 np.array([w.in_table[u] for u in inputs], dtype=np.int32))],
        "bwd": []})
    by_layer: dict[tuple[int, int], list[int]] = {}
    for u in range(w.n_blocks):                       # ascending u inside every bucket
        if w.type[u] != INPUT:
            by_layer.setdefault((int(depth[u]), int(w.type[u])), []).append(u)
    for d in range(1, int(depth.max()) + 1):
        for kind in (PRODUCT, SUM):
            blocks = by_layer.get((d, kind))
            if not blocks:
                continue
            fwd_rows = []
            parents: dict[int, list] = {}
            for u in blocks:
                lst = []
                for e in range(int(w.child_ptr[u]), int(w.child_ptr[u + 1])):
                    c = int(w.child[e])
                    p = par_off(w.param_blk[e]) if kind == SUM else 0
                    lst.append((node_off(c), p))
                    parents.setdefault(c, []).append((node_off(u), p))
                fwd_rows.append((node_off(u), lst))
            bwd_rows = [(node_off(c), parents[c]) for c in sorted(parents)]
            layers.append({
                "kind": kind, "depth": d,
                "fwd": _grouped_tables(fwd_rows, w.max_groups, w.tol_permille),
                "bwd": _grouped_tables(bwd_rows, w.max_groups, w.tol_permille)})
    return {"K": K, "n_rows": (w.n_blocks + 1) * K, "layers": layers}


# ------------------------------------------------------------------------------------------------
# Collapse of consecutive sum / sum and product / product blocks (footnote to Def. 2)
# ------------------------------------------------------------------------------------------------
def collapse(w, theta):
    """Rewrite a block DAG so that it alternates: a product block takes over the children of its product children
    (a product of products is one product), a sum block takes over the children of its sum children with the weight
    blocks multiplied (sum_j A[i,j] sum_k B[j,k] c_k = sum_k (A B)[i,k] c_k); several paths to one child add up.

    Canonical form of the result (the library follows the same written rules):
      * edges keep the order of the original edges, a replaced edge expanding in place into its child's edges; a
        child reached twice keeps its first position (sum blocks: the weight blocks add; product blocks: an error);
      * blocks no longer reachable from the root are dropped, the others keep their order and are renumbered 0, 1, ...;
      * a sum block none of whose edges changed keeps its parameter blocks (and its ties); a changed one gets fresh
        blocks for all its edges; parameter blocks are renumbered in order of first use (blocks ascending, edges in order).
    Returns a namespace with the DAG fields of a workload, `theta` (float32) and `block_map` (old id -> new id or -1)."""
    from types import SimpleNamespace
    K, n = int(w.K), int(w.n_blocks)
    typ = np.asarray(w.type)
    th = np.asarray(theta, dtype=np.float64)
    prod_list: dict[int, list[int]] = {}
    sum_list: dict[int, tuple[list[int], list, bool]] = {}

    def flat_product(u):
        if u not in prod_list:
            out = []
            for e in range(int(w.child_ptr[u]), int(w.child_ptr[u + 1])):
                c = int(w.child[e])
                out.extend(flat_product(c) if typ[c] == PRODUCT else [c])
            if len(set(out)) != len(out):
                raise CompileError(f"product block {u} reaches a child twice")
            prod_list[u] = out
        return prod_list[u]

    def flat_sum(u):
        """(children, per child: original parameter block id or matrix, changed)"""
        if u not in sum_list:
            order, entry, changed = [], {}, False
            for e in range(int(w.child_ptr[u]), int(w.child_ptr[u + 1])):
                c, pb = int(w.child[e]), int(w.param_blk[e])
                if typ[c] == SUM:
                    changed = True
                    cc, ce, _ = flat_sum(c)
                    parts = [(k2, th[pb + 1] @ (th[m + 1] if isinstance(m, int) else m)) for k2, m in zip(cc, ce)]
                else:
                    parts = [(c, pb)]
                for k2, m in parts:
                    if k2 in entry:
                        changed = True
                        old = entry[k2]
                        entry[k2] = (th[old + 1] if isinstance(old, int) else old) + (th[m + 1] if isinstance(m, int) else m)
                    else:
                        entry[k2] = m
                        order.append(k2)
            sum_list[u] = (order, [entry[k2] for k2 in order], changed)
        return sum_list[u]

    import sys
    sys.setrecursionlimit(max(10000, 4 * n))
    new_children: dict[int, list[int]] = {}
    reach, stack = set(), [int(w.root_block)]
    while stack:
        u = stack.pop()
        if u in reach:
            continue
        reach.add(u)
        new_children[u] = flat_product(u) if typ[u] == PRODUCT else flat_sum(u)[0] if typ[u] == SUM else []
        stack.extend(new_children[u])
    keep = sorted(reach)
    block_map = np.full(n, -1, dtype=np.int32)
    block_map[keep] = np.arange(len(keep), dtype=np.int32)
    child_ptr, child, param, mats, pb_new = [0], [], [], [], {}
    for u in keep:
        if typ[u] == SUM:
            order, ent, changed = flat_sum(u)
            for c, m in zip(order, ent):
                if not changed and isinstance(m, int):
                    if m not in pb_new:
                        pb_new[m] = len(mats)
                        mats.append(th[m + 1])
                    param.append(pb_new[m])
                else:
                    param.append(len(mats))
                    mats.append(th[m + 1] if isinstance(m, int) else m)
                child.append(int(block_map[c]))
        else:
            for c in new_children[u]:
                child.append(int(block_map[c]))
                param.append(-1)
        child_ptr.append(len(child))
    theta_new = np.zeros((len(mats) + 1, K, K), dtype=np.float32)
    for p, M in enumerate(mats):
        theta_new[p + 1] = M.astype(np.float32)
    keep = np.asarray(keep, dtype=np.int64)
    return SimpleNamespace(
        K=K, n_blocks=len(keep), root_block=int(block_map[int(w.root_block)]), type=typ[keep].astype(np.uint8),
        n_real=np.asarray(w.n_real)[keep].astype(np.int32), child_ptr=np.asarray(child_ptr, dtype=np.int64),
        child=np.asarray(child, dtype=np.int32), param_blk=np.asarray(param, dtype=np.int32), n_param_blocks=len(mats),
        in_var=np.asarray(w.in_var)[keep].astype(np.int32), in_table=np.asarray(w.in_table)[keep].astype(np.int32),
        n_vars=int(w.n_vars), n_cats=int(w.n_cats), n_tables=int(w.n_tables), max_groups=int(w.max_groups),
        tol_permille=int(w.tol_permille), theta=theta_new, block_map=block_map)
