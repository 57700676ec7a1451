"""Seeded synthetic workloads: block-level circuit structures, fp32 parameters and data.

This module only *describes* inputs (structure, random parameters, random data).  It holds
none of the method's arithmetic (no forward pass, no flows, no table compilation) and is the
one module both the CPU oracle's tests and the GPU path's tests / benchmark draw inputs from.

Structures follow the experimental section of the paper (Sec. 6, App. C): homogeneous HMMs
written as circuits (footnote to Sec. 1), hidden Chow-Liu trees, and a Poon-Domingos grid
structure with axis-aligned splits (App. C.4), optionally with whole child blocks pruned at
random as in the block-sparse experiment (App. C.1), a random tensorised structure (RAT-SPN), and the
single wide block-sparse sum layer of that experiment (also the shape of the layer analysed in Sec. 4.2).

Block-level DAG convention (one "block" = K consecutive node slots):
  type[u]        0 input, 1 product, 2 sum
  n_real[u]      number of real nodes in the block (rows >= n_real are placeholders, Sec. 4.1 footnote)
  child_ptr/child  CSR list of child blocks per block
  param_blk[e]   for an edge out of a sum block: id of its K x K parameter block (equal ids = tied,
                 App. A.3); -1 otherwise.  Parameter block p is stored at theta[p + 1]; theta[0] is an
                 all-zero block used by table padding.  theta[p + 1][i][j] is the weight from sum node i
                 of the parent block to node j of the child block.
  in_var/in_table  for an input block: the variable it reads and its categorical table;
                 tables[t][c][k] = P(X = c) under node k of the block (category-major).
A product block multiplies its child blocks element-wise: node k of the block has node k of every
child block as children.
"""
from __future__ import annotations

import heapq
from dataclasses import dataclass, field

import numpy as np

SEED_BASE = 240600766
FLT_MIN = np.float32(np.finfo(np.float32).tiny)

INPUT, PRODUCT, SUM = 0, 1, 2


@dataclass
class Workload:
    name: str
    K: int
    n_blocks: int
    root_block: int
    type: np.ndarray
    n_real: np.ndarray
    child_ptr: np.ndarray
    child: np.ndarray
    param_blk: np.ndarray
    n_param_blocks: int
    in_var: np.ndarray
    in_table: np.ndarray
    n_vars: int
    n_cats: int
    n_tables: int
    theta: np.ndarray          # float32 [n_param_blocks + 1, K, K], block 0 all zero
    tables: np.ndarray         # float32 [n_tables, n_cats, K]
    x: np.ndarray              # int32 [B, n_vars]
    max_groups: int = 8
    tol_permille: int = 250
    meta: dict = field(default_factory=dict)
    product_scratch: int = 0   # 1: compile in the memory-saving mode of Sec. 5 (needs the block order of pc_order_for_scratch)

    @property
    def B(self) -> int:
        return int(self.x.shape[0])

    @property
    def n_edges(self) -> int:
        return int(self.child.shape[0])

    def n_sum_edges(self) -> int:
        """Node-level number of sum edges with a real parent row (the paper's circuit size)."""
        tot = 0
        for u in np.nonzero(self.type == SUM)[0]:
            ch = self.child[self.child_ptr[u]:self.child_ptr[u + 1]]
            tot += int(self.n_real[u]) * int(self.n_real[ch].sum())
        return tot

    def with_batch(self, x: np.ndarray) -> "Workload":
        w = Workload(**{k: getattr(self, k) for k in self.__dataclass_fields__})
        w.x = np.ascontiguousarray(x, dtype=np.int32)
        return w


class _Builder:
    def __init__(self, K: int):
        self.K = K
        self.type: list[int] = []
        self.n_real: list[int] = []
        self.children: list[list[int]] = []
        self.params: list[list[int]] = []
        self.var: list[int] = []
        self.table: list[int] = []

    def add(self, typ: int, *, n_real: int | None = None, var: int = -1, table: int = -1) -> int:
        self.type.append(typ)
        self.n_real.append(self.K if n_real is None else n_real)
        self.children.append([])
        self.params.append([])
        self.var.append(var)
        self.table.append(table)
        return len(self.type) - 1

    def link(self, parent: int, child: int, param: int = -1) -> None:
        self.children[parent].append(child)
        self.params[parent].append(param)

    def arrays(self):
        n = len(self.type)
        ptr = np.zeros(n + 1, dtype=np.int64)
        for u in range(n):
            ptr[u + 1] = ptr[u] + len(self.children[u])
        child = np.fromiter((c for cs in self.children for c in cs), dtype=np.int32, count=int(ptr[-1]))
        param = np.fromiter((p for ps in self.params for p in ps), dtype=np.int32, count=int(ptr[-1]))
        return (np.asarray(self.type, dtype=np.uint8), np.asarray(self.n_real, dtype=np.int32), ptr, child, param,
                np.asarray(self.var, dtype=np.int32), np.asarray(self.table, dtype=np.int32))


def _f32_floor(a: np.ndarray) -> np.ndarray:
    """Cast probabilities to fp32; exact zeros and subnormals become the smallest normal float."""
    out = a.astype(np.float32)
    np.maximum(out, FLT_MIN, out=out)
    return out


def _dirichlet_rows(rng: np.random.Generator, alpha: float, shape: tuple[int, int]) -> np.ndarray:
    """Rows drawn from a symmetric Dirichlet(alpha), float64, each row normalised to sum 1."""
    if alpha == 1.0:
        g = rng.standard_exponential(shape)
    else:
        g = rng.standard_gamma(alpha, shape)
    s = g.sum(axis=1, keepdims=True)
    bad = (s <= 0).ravel()
    if bad.any():                      # all draws underflowed: fall back to a uniform row
        g[bad] = 1.0
        s = g.sum(axis=1, keepdims=True)
    return g / s


def _dense_to_blocks(W: np.ndarray, K: int) -> np.ndarray:
    """[R, C] -> [R/K * C/K, K, K], block (ib, jb) at index ib * (C/K) + jb."""
    R, C = W.shape
    return W.reshape(R // K, K, C // K, K).transpose(0, 2, 1, 3).reshape(-1, K, K)


def _make(name, bld: _Builder, root, n_param_blocks, n_vars, n_cats, n_tables, theta, tables, x, meta,
          max_groups=8, tol_permille=250) -> Workload:
    typ, n_real, ptr, child, param, var, table = bld.arrays()
    return Workload(name=name, K=bld.K, n_blocks=len(typ), root_block=root, type=typ, n_real=n_real,
                    child_ptr=ptr, child=child, param_blk=param, n_param_blocks=n_param_blocks,
                    in_var=var, in_table=table, n_vars=n_vars, n_cats=n_cats, n_tables=n_tables,
                    theta=theta, tables=tables, x=np.ascontiguousarray(x, dtype=np.int32),
                    max_groups=max_groups, tol_permille=tol_permille, meta=meta)


# --------------------------------------------------------------------------------------------
# HMM written as a circuit (footnote to Sec. 1; parameter tying across time, App. A.3)
# --------------------------------------------------------------------------------------------
def hmm(T: int, H: int, V: int, K: int, B: int, seed: int, *, alpha_init=1.0, alpha_trans=1.0,
        alpha_emis=1.0, tokens="uniform", keep_dense=True, draw=True, name=None) -> Workload:
    """Hidden z_0..z_{T-1}, tokens x_0..x_{T-1}.

    E_t[h]  input node on variable t with P(x_t = v | z_t = h), tied over t
    P_t[h]  = E_t[h] * S_{t+1}[h]      (P_{T-1}[h] = E_{T-1}[h])
    S_t[h]  = sum_h' A[h, h'] P_t[h']  for t = 1..T-1, tied over t
    root    = sum_h pi[h] P_0[h]
    """
    assert H % K == 0 and T >= 1
    nb = H // K
    rng = np.random.Generator(np.random.PCG64(seed))
    bld = _Builder(K)
    E = [[bld.add(INPUT, var=t, table=j) for j in range(nb)] for t in range(T)]
    P = [[bld.add(PRODUCT) for _ in range(nb)] for _ in range(T)]
    S = [None] + [[bld.add(SUM) for _ in range(nb)] for _ in range(1, T)]
    root = bld.add(SUM, n_real=1)
    for t in range(T):
        for j in range(nb):
            bld.link(P[t][j], E[t][j])
            if t + 1 < T:
                bld.link(P[t][j], S[t + 1][j])
    for t in range(1, T):
        for i in range(nb):
            for j in range(nb):
                bld.link(S[t][i], P[t][j], i * nb + j)
    n_A = nb * nb if T > 1 else 0
    for j in range(nb):
        bld.link(root, P[0][j], n_A + j)
    n_param_blocks = n_A + nb

    theta = np.zeros((n_param_blocks + 1, K, K), dtype=np.float32)
    if not draw:                                   # structure only: parameters and data left at zero
        return _make(name or f"hmm_T{T}_H{H}_V{V}_K{K}_B{B}", bld, root, n_param_blocks, T, V, nb, theta,
                     np.zeros((nb, V, K), dtype=np.float32), np.zeros((B, T), dtype=np.int32), {"kind": "hmm", "T": T, "H": H, "V": V})
    pi = _f32_floor(_dirichlet_rows(rng, alpha_init, (1, H)))[0]
    A = None
    if T > 1:
        A = np.empty((H, H), dtype=np.float32)
        step = max(1, min(H, (1 << 22) // H))
        for r0 in range(0, H, step):
            A[r0:r0 + step] = _f32_floor(_dirichlet_rows(rng, alpha_trans, (min(step, H - r0), H)))
        theta[1:1 + n_A] = _dense_to_blocks(A, K)
    theta[1 + n_A:, 0, :] = pi.reshape(nb, K)

    tables = np.empty((nb, V, K), dtype=np.float32)
    for j in range(nb):
        Ej = _f32_floor(_dirichlet_rows(rng, alpha_emis, (K, V)))   # [K hidden states, V]
        tables[j] = Ej.T

    if tokens == "uniform":
        x = rng.integers(0, V, size=(B, T))
    elif tokens == "zipf":
        w = (np.arange(V, dtype=np.float64) + 1.0) ** -1.1
        cdf = np.cumsum(w / w.sum())
        x = np.minimum(np.searchsorted(cdf, rng.random((B, T)), side="right"), V - 1)
    else:
        raise ValueError(tokens)

    meta = {"kind": "hmm", "T": T, "H": H, "V": V, "pi": pi}
    if keep_dense:
        meta["A"] = A
    return _make(name or f"hmm_T{T}_H{H}_V{V}_K{K}_B{B}", bld, root, n_param_blocks, T, V, nb, theta, tables, x, meta)


def hmm_emission(w: Workload) -> np.ndarray:
    """Emission matrix [H, V] (fp32) read back from the block tables of an HMM workload."""
    nb, V, K = w.tables.shape
    return w.tables.transpose(0, 2, 1).reshape(nb * K, V)


# --------------------------------------------------------------------------------------------
# Hidden Chow-Liu tree over a random spanning tree
# --------------------------------------------------------------------------------------------
def _prufer_tree(seq: np.ndarray, D: int) -> list[tuple[int, int]]:
    degree = np.ones(D, dtype=np.int64)
    for v in seq:
        degree[v] += 1
    leaves = [i for i in range(D) if degree[i] == 1]
    heapq.heapify(leaves)
    edges = []
    for v in seq:
        leaf = heapq.heappop(leaves)
        edges.append((int(leaf), int(v)))
        degree[v] -= 1
        if degree[v] == 1:
            heapq.heappush(leaves, int(v))
    a = heapq.heappop(leaves)
    b = heapq.heappop(leaves)
    edges.append((int(a), int(b)))
    return edges


def random_tree(rng: np.random.Generator, D: int):
    """Uniform random labelled tree on D vertices, rooted at 0.  Returns (parent[], bfs order)."""
    if D == 1:
        return np.array([-1]), [0]
    if D == 2:
        edges = [(0, 1)]
    else:
        edges = _prufer_tree(rng.integers(0, D, size=D - 2), D)
    adj = [[] for _ in range(D)]
    for a, b in edges:
        adj[a].append(b)
        adj[b].append(a)
    parent = np.full(D, -1, dtype=np.int64)
    order = [0]
    seen = np.zeros(D, dtype=bool)
    seen[0] = True
    for v in order:
        for c in sorted(adj[v]):
            if not seen[c]:
                seen[c] = True
                parent[c] = v
                order.append(c)
    assert len(order) == D
    return parent, order


def hclt(D: int, M: int, K: int, B: int, seed: int, *, n_cats=256, data="gauss", draw=True, name=None) -> Workload:
    """Latent tree: each variable v has a latent z_v with M states.

    E_v[k]  input node on variable v, own table per variable
    P_v[k]  = E_v[k] * prod_{c child of v} S_c[k]
    S_c[k]  = sum_k' W_c[k, k'] P_c[k']     for every non-root variable c
    root    = sum_k pi[k] P_0[k]
    """
    assert M % K == 0
    nb = M // K
    rng = np.random.Generator(np.random.PCG64(seed))
    parent, order = random_tree(rng, D)
    kids = [[] for _ in range(D)]
    for v in order[1:]:
        kids[parent[v]].append(v)

    bld = _Builder(K)
    E = [[bld.add(INPUT, var=v, table=v * nb + j) for j in range(nb)] for v in range(D)]
    P = [[bld.add(PRODUCT) for _ in range(nb)] for _ in range(D)]
    S = [None] + [[bld.add(SUM) for _ in range(nb)] for _ in range(1, D)]
    root = bld.add(SUM, n_real=1)
    for v in range(D):
        for j in range(nb):
            bld.link(P[v][j], E[v][j])
            for c in kids[v]:
                bld.link(P[v][j], S[c][j])
    for c in range(1, D):
        base = (c - 1) * nb * nb
        for i in range(nb):
            for j in range(nb):
                bld.link(S[c][i], P[c][j], base + i * nb + j)
    n_W = (D - 1) * nb * nb
    for j in range(nb):
        bld.link(root, P[0][j], n_W + j)
    n_param_blocks = n_W + nb

    theta = np.zeros((n_param_blocks + 1, K, K), dtype=np.float32)
    if not draw:
        return _make(name or f"hclt_D{D}_M{M}_K{K}_B{B}", bld, root, n_param_blocks, D, n_cats, D * nb, theta,
                     np.zeros((D * nb, n_cats, K), dtype=np.float32), np.zeros((B, D), dtype=np.int32),
                     {"kind": "hclt", "D": D, "M": M, "parent": parent, "order": order})
    for c in range(1, D):
        W = _f32_floor(_dirichlet_rows(rng, 1.0, (M, M)))
        base = 1 + (c - 1) * nb * nb
        theta[base:base + nb * nb] = _dense_to_blocks(W, K)
    pi = _f32_floor(_dirichlet_rows(rng, 1.0, (1, M)))[0]
    theta[1 + n_W:, 0, :] = pi.reshape(nb, K)

    tables = np.empty((D * nb, n_cats, K), dtype=np.float32)
    for v in range(D):
        Tv = _f32_floor(_dirichlet_rows(rng, 1.0, (M, n_cats)))          # [latent state, category]
        tables[v * nb:(v + 1) * nb] = Tv.reshape(nb, K, n_cats).transpose(0, 2, 1)

    hi = n_cats - 1
    mu = rng.uniform(0.0, float(hi), size=D)
    std = 40.0 * n_cats / 256.0
    if data == "gauss":
        x = np.clip(np.rint(rng.normal(mu[None, :], std, size=(B, D))), 0, hi)
    elif data == "gauss_corr":
        amp = 16.0 * n_cats / 256.0
        off = np.empty((B, D))
        off[:, 0] = np.where(rng.random(B) < 0.5, -amp, amp)
        flip = rng.random((B, D)) >= 0.75
        for v in order[1:]:
            off[:, v] = np.where(flip[:, v], -off[:, parent[v]], off[:, parent[v]])
        x = np.clip(np.rint(rng.normal(mu[None, :] + off, std)), 0, hi)
    elif data == "uniform":
        x = rng.integers(0, n_cats, size=(B, D))
    else:
        raise ValueError(data)

    meta = {"kind": "hclt", "D": D, "M": M, "parent": parent, "order": order, "pi": pi}
    return _make(name or f"hclt_D{D}_M{M}_K{K}_B{B}", bld, root, n_param_blocks, D, n_cats, D * nb, theta, tables, x, meta)


def hclt_edge_weights(w: Workload, c: int) -> np.ndarray:
    """W_c [M, M] (fp32) of tree edge parent(c) -> c, read back from theta."""
    M, K = w.meta["M"], w.K
    nb = M // K
    base = 1 + (c - 1) * nb * nb
    return w.theta[base:base + nb * nb].reshape(nb, nb, K, K).transpose(0, 2, 1, 3).reshape(M, M)


def hclt_table(w: Workload, v: int) -> np.ndarray:
    """Emission table [M, n_cats] (fp32) of variable v."""
    M, K = w.meta["M"], w.K
    nb = M // K
    return w.tables[v * nb:(v + 1) * nb].transpose(0, 2, 1).reshape(M, -1)


# --------------------------------------------------------------------------------------------
# Poon-Domingos region structure with axis-aligned splits, optional block pruning
# --------------------------------------------------------------------------------------------
def pd(grid: int, cell: int, M: int, K: int, B: int, seed: int, *, keep=1.0, n_cats=256, draw=True, name=None) -> Workload:
    """grid x grid coarse cells of cell x cell pixels.  Regions = all coarse rectangles.

    leaf cell:   L[k] = prod_{pixels} E_pixel[k]; its region's sums range over L
    other region: one block of M product nodes per two-way split, P[k] = S_left[k] * S_right[k];
                  the region's M sums (root: one) range over the product nodes of all its splits
    keep < 1:    each (sum block, child block) pair survives with probability `keep`
                 (at least one child block per sum block always survives)
    """
    assert M % K == 0
    nb = M // K
    side = grid * cell
    D = side * side
    rng = np.random.Generator(np.random.PCG64(seed))
    bld = _Builder(K)

    E = [[bld.add(INPUT, var=v, table=v * nb + j) for j in range(nb)] for v in range(D)]
    regions = [(x0, x1, y0, y1) for x0 in range(grid) for x1 in range(x0 + 1, grid + 1)
               for y0 in range(grid) for y1 in range(y0 + 1, grid + 1)]
    regions.sort(key=lambda r: ((r[1] - r[0]) + (r[3] - r[2]), r))
    full = (0, grid, 0, grid)
    S = {}
    for r in regions:
        if r == full:
            S[r] = [bld.add(SUM, n_real=1)]
        else:
            S[r] = [bld.add(SUM) for _ in range(nb)]
    root = S[full][0]

    sum_children: dict = {}
    for r in regions:
        x0, x1, y0, y1 = r
        prods = []
        if x1 - x0 == 1 and y1 - y0 == 1:
            L = [bld.add(PRODUCT) for _ in range(nb)]
            for py in range(y0 * cell, (y0 + 1) * cell):
                for px in range(x0 * cell, (x0 + 1) * cell):
                    for j in range(nb):
                        bld.link(L[j], E[py * side + px][j])
            prods.extend(L)
        else:
            splits = [((x0, c, y0, y1), (c, x1, y0, y1)) for c in range(x0 + 1, x1)]
            splits += [((x0, x1, y0, c), (x0, x1, c, y1)) for c in range(y0 + 1, y1)]
            for a, b in splits:
                Pb = [bld.add(PRODUCT) for _ in range(nb)]
                for j in range(nb):
                    bld.link(Pb[j], S[a][j])
                    bld.link(Pb[j], S[b][j])
                prods.extend(Pb)
        sum_children[r] = prods

    n_param_blocks = 0
    kept: list[tuple[int, list[int]]] = []
    for r in regions:
        prods = sum_children[r]
        for s in S[r]:
            if keep >= 1.0:
                ks = list(prods)
            else:
                m = rng.random(len(prods)) < keep
                if not m.any():
                    m[rng.integers(0, len(prods))] = True
                ks = [p for p, f in zip(prods, m) if f]
            for p in ks:
                bld.link(s, p, n_param_blocks)
                n_param_blocks += 1
            kept.append((s, ks))

    theta = np.zeros((n_param_blocks + 1, K, K), dtype=np.float32)
    if not draw:
        return _make(name or f"pd_g{grid}_c{cell}_M{M}_K{K}_keep{keep}_B{B}", bld, root, n_param_blocks, D, n_cats,
                     D * nb, theta, np.zeros((D * nb, n_cats, K), dtype=np.float32), np.zeros((B, D), dtype=np.int32),
                     {"kind": "pd", "grid": grid, "cell": cell, "M": M, "keep": keep})
    pos = 1
    for s, ks in kept:
        nk = len(ks)
        rows = 1 if s == root else K
        W = _f32_floor(_dirichlet_rows(rng, 1.0, (rows, nk * K)))
        theta[pos:pos + nk, :rows, :] = W.reshape(rows, nk, K).transpose(1, 0, 2)
        pos += nk

    tables = np.empty((D * nb, n_cats, K), dtype=np.float32)
    for v in range(D):
        Tv = _f32_floor(_dirichlet_rows(rng, 1.0, (M, n_cats)))
        tables[v * nb:(v + 1) * nb] = Tv.reshape(nb, K, n_cats).transpose(0, 2, 1)

    x = rng.integers(0, n_cats, size=(B, D))
    meta = {"kind": "pd", "grid": grid, "cell": cell, "M": M, "keep": keep}
    return _make(name or f"pd_g{grid}_c{cell}_M{M}_K{K}_keep{keep}_B{B}", bld, root, n_param_blocks, D, n_cats,
                 D * nb, theta, tables, x, meta)


# --------------------------------------------------------------------------------------------
# Random tensorised structure (RAT-SPN, the fourth structure of Sec. 6.1)
# --------------------------------------------------------------------------------------------
def rat_spn(D: int, depth: int, R: int, S: int, K: int, B: int, seed: int, *, n_cats=256, data="gauss", draw=True,
            name=None) -> Workload:
    """R replicas of a random region tree over D variables, joined under one root.

    replica r:  a random permutation of the variables is split into two halves, recursively, `depth` times
    leaf region (variable set V):  S factorised distributions, distribution k = prod_{v in V} E_{r,v}[k]
                (one table per replica and variable)
    region with halves (left, right), each offering S / K node blocks: one product block per PAIR of blocks,
                P_{a,b}[k] = left_a[k] * right_b[k]   (the cross product taken block-wise; a leaf half
                contributes the input blocks of its variables directly, so products never feed products);
                the region's S sum nodes range over all (S / K)^2 * K product nodes
    root:       one sum node over the product nodes of the R top regions
    The paper gives sizes only (nodes / edges); depth, R and S are free parameters chosen to match them.
    """
    assert S % K == 0 and depth >= 1 and D >= 2 ** depth
    nb = S // K
    rng = np.random.Generator(np.random.PCG64(seed))
    bld = _Builder(K)
    n_tables = R * D * nb
    E = [[[bld.add(INPUT, var=v, table=(r * D + v) * nb + j) for j in range(nb)] for v in range(D)] for r in range(R)]
    sums: list[tuple[int, list[int]]] = []                 # (sum block, its product blocks), creation order
    top_products: list[int] = []

    def region(r: int, vs: np.ndarray, level: int):
        """-> per node block of the region, the list of blocks a product above has to multiply"""
        if level == depth:
            return [[E[r][int(v)][j] for v in vs] for j in range(nb)]
        half = len(vs) // 2
        left, right = region(r, vs[:half], level + 1), region(r, vs[half:], level + 1)
        prods = []
        for a in range(nb):
            for b in range(nb):
                p = bld.add(PRODUCT)
                for ch in left[a] + right[b]:
                    bld.link(p, ch)
                prods.append(p)
        if level == 0:
            top_products.extend(prods)
            return None
        blocks = [bld.add(SUM) for _ in range(nb)]
        for sblk in blocks:
            sums.append((sblk, prods))
        return [[sblk] for sblk in blocks]

    for r in range(R):
        region(r, rng.permutation(D), 0)
    root = bld.add(SUM, n_real=1)
    sums.append((root, top_products))
    n_param_blocks = 0
    for sblk, prods in sums:
        for p in prods:
            bld.link(sblk, p, n_param_blocks)
            n_param_blocks += 1

    meta = {"kind": "rat_spn", "D": D, "depth": depth, "R": R, "S": S}
    nm = name or f"rat_D{D}_d{depth}_R{R}_S{S}_K{K}_B{B}"
    theta = np.zeros((n_param_blocks + 1, K, K), dtype=np.float32)
    if not draw:
        return _make(nm, bld, root, n_param_blocks, D, n_cats, n_tables, theta,
                     np.zeros((n_tables, n_cats, K), dtype=np.float32), np.zeros((B, D), dtype=np.int32), meta)
    pos = 1
    for sblk, prods in sums:
        rows = 1 if sblk == root else K
        nk = len(prods)
        Wt = _f32_floor(_dirichlet_rows(rng, 1.0, (rows, nk * K)))
        theta[pos:pos + nk, :rows, :] = Wt.reshape(rows, nk, K).transpose(1, 0, 2)
        pos += nk
    tables = np.empty((n_tables, n_cats, K), dtype=np.float32)
    for t in range(R * D):
        Tv = _f32_floor(_dirichlet_rows(rng, 1.0, (S, n_cats)))
        tables[t * nb:(t + 1) * nb] = Tv.reshape(nb, K, n_cats).transpose(0, 2, 1)
    hi = n_cats - 1
    if data == "gauss":
        mu = rng.uniform(0.0, float(hi), size=D)
        x = np.clip(np.rint(rng.normal(mu[None, :], 40.0 * n_cats / 256.0, size=(B, D))), 0, hi)
    else:
        x = rng.integers(0, n_cats, size=(B, D))
    return _make(nm, bld, root, n_param_blocks, D, n_cats, n_tables, theta, tables, x, meta)


# --------------------------------------------------------------------------------------------
# One wide sum layer (App. C.1: independent fully-connected node sets; Sec. 4.2 analysis layer)
# --------------------------------------------------------------------------------------------
def sum_layer(n_sets: int, M: int, K: int, B: int, seed: int, *, keep=1.0, n_cats=256, draw=True, name=None) -> Workload:
    """`n_sets` independent sets of M sum nodes fully connected to M product nodes, wrapped into a circuit.

    set s (variable s):  E_s = M categorical input nodes, P_s[k] = E_s[k] (single child),
                         S_s[i] = sum_j W_s[i, j] P_s[j]   -- the layer under study, n_sets * M * M edges
    on top:              T[k] = prod_s S_s[k],  root = sum_k pi[k] T[k]
    keep < 1:  each K x K edge block of a set survives with probability `keep`; every sum block keeps at
               least one child block, so every sum node keeps at least one child (App. C.1).
    Built with array operations only, so that K = 1 (one block per node) stays affordable.
    """
    assert M % K == 0
    nb = M // K
    rng = np.random.Generator(np.random.PCG64(seed))
    nE = n_sets * nb
    E0, P0, S0, T0 = 0, nE, 2 * nE, 3 * nE
    root = T0 + nb
    n_blocks = root + 1

    masks = np.ones((n_sets, nb, nb), dtype=bool)
    if keep < 1.0:
        masks = rng.random((n_sets, nb, nb)) < keep
        empty = ~masks.any(axis=2)
        pick = rng.integers(0, nb, size=(n_sets, nb))
        s_i, r_i = np.nonzero(empty)
        masks[s_i, r_i, pick[s_i, r_i]] = True
    n_kept = masks.sum(axis=2).astype(np.int64)                        # [n_sets, nb] child blocks per sum block
    n_sum_edges = int(n_kept.sum())

    typ = np.empty(n_blocks, dtype=np.uint8)
    typ[E0:P0], typ[P0:S0], typ[S0:T0], typ[T0:root], typ[root] = INPUT, PRODUCT, SUM, PRODUCT, SUM
    n_real = np.full(n_blocks, K, dtype=np.int32)
    n_real[root] = 1
    deg = np.zeros(n_blocks, dtype=np.int64)
    deg[P0:S0] = 1
    deg[S0:T0] = n_kept.ravel()
    deg[T0:root] = n_sets
    deg[root] = nb
    ptr = np.zeros(n_blocks + 1, dtype=np.int64)
    np.cumsum(deg, out=ptr[1:])
    child = np.empty(int(ptr[-1]), dtype=np.int32)
    param = np.full(int(ptr[-1]), -1, dtype=np.int32)
    child[ptr[P0]:ptr[S0]] = np.arange(E0, P0, dtype=np.int32)
    set_of, _, col = np.nonzero(masks)                                 # row-major: set, sum block, child block ascending
    child[ptr[S0]:ptr[T0]] = (P0 + set_of * nb + col).astype(np.int32)
    param[ptr[S0]:ptr[T0]] = np.arange(n_sum_edges, dtype=np.int32)
    child[ptr[T0]:ptr[root]] = (S0 + np.arange(n_sets)[None, :] * nb + np.arange(nb)[:, None]).ravel().astype(np.int32)
    child[ptr[root]:] = np.arange(T0, root, dtype=np.int32)
    param[ptr[root]:] = n_sum_edges + np.arange(nb, dtype=np.int32)
    n_param_blocks = n_sum_edges + nb

    in_var = np.full(n_blocks, -1, dtype=np.int32)
    in_table = np.full(n_blocks, -1, dtype=np.int32)
    in_var[E0:P0] = np.repeat(np.arange(n_sets, dtype=np.int32), nb)
    in_table[E0:P0] = np.arange(nE, dtype=np.int32)

    theta = np.zeros((n_param_blocks + 1, K, K), dtype=np.float32)
    tables = np.zeros((nE, n_cats, K), dtype=np.float32)
    x = np.zeros((B, n_sets), dtype=np.int32)
    if draw:
        pos = 1
        for s in range(n_sets):
            Wd = rng.standard_exponential((M, M))
            dense_mask = np.repeat(np.repeat(masks[s], K, axis=0), K, axis=1)
            Wd *= dense_mask
            Wd /= Wd.sum(axis=1, keepdims=True)
            Wf = _f32_floor(Wd) * dense_mask
            nk = int(n_kept[s].sum())
            theta[pos:pos + nk] = _dense_to_blocks(Wf, K)[masks[s].ravel()]
            pos += nk
            Tv = _f32_floor(_dirichlet_rows(rng, 1.0, (M, n_cats)))
            tables[s * nb:(s + 1) * nb] = Tv.reshape(nb, K, n_cats).transpose(0, 2, 1)
        pi = _f32_floor(_dirichlet_rows(rng, 1.0, (1, M)))
        theta[pos:pos + nb, 0, :] = pi.reshape(nb, K)
        x = rng.integers(0, n_cats, size=(B, n_sets))
    meta = {"kind": "sum_layer", "n_sets": n_sets, "M": M, "keep": keep, "n_layer_edges": n_sum_edges * K * K,
            "S0": S0, "P0": P0, "T0": T0}
    return Workload(name=name or f"layer_S{n_sets}_M{M}_K{K}_keep{keep}_B{B}", K=K, n_blocks=n_blocks, root_block=root,
                    type=typ, n_real=n_real, child_ptr=ptr, child=child, param_blk=param, n_param_blocks=n_param_blocks,
                    in_var=in_var, in_table=in_table, n_vars=n_sets, n_cats=n_cats, n_tables=nE, theta=theta,
                    tables=tables, x=np.ascontiguousarray(x, dtype=np.int32), meta=meta)


def sum_layer_dense(w: Workload, s: int) -> np.ndarray:
    """float64 [M, M] weight matrix of set s of a `sum_layer` workload (zeros where edge blocks were dropped)."""
    K, nb, M = w.K, w.meta["M"] // w.K, w.meta["M"]
    out = np.zeros((M, M))
    for i in range(nb):
        u = w.meta["S0"] + s * nb + i
        for e in range(int(w.child_ptr[u]), int(w.child_ptr[u + 1])):
            j = int(w.child[e]) - w.meta["P0"] - s * nb
            out[i * K:(i + 1) * K, j * K:(j + 1) * K] = w.theta[int(w.param_blk[e]) + 1]
    return out


# --------------------------------------------------------------------------------------------
# Random alternating DAGs (test inputs: skip connections, tying, placeholders, unused blocks)
# --------------------------------------------------------------------------------------------
def random_circuit(n_vars: int, n_levels: int, width: int, K: int, B: int, seed: int, *, n_cats=5, tie_prob=0.3,
                   alpha=0.5, name=None) -> Workload:
    """A random block DAG that alternates product and sum levels above one input level.

    Children are drawn from ALL lower levels of the right kind (products take sum and input blocks, sums take
    product blocks), so blocks collect parents from several layers; some sum blocks reuse the whole parameter-block
    list of an earlier sum block with as many children (tying); some sum blocks have fewer than K real nodes; blocks
    that nothing refers to stay in the DAG.  Not smooth or decomposable in general -- the forward and backward
    passes are plain arithmetic on any such DAG, and every value stays a probability <= 1.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    bld = _Builder(K)
    inputs = [bld.add(INPUT, var=int(rng.integers(0, n_vars)), table=i) for i in range(width)]
    sums_or_inputs = list(inputs)
    products: list[int] = []
    sum_children: dict[int, list[int]] = {}
    for level in range(n_levels):
        new_p = []
        for _ in range(int(rng.integers(1, width + 1))):
            p = bld.add(PRODUCT)
            k = int(rng.integers(1, min(3, len(sums_or_inputs)) + 1))
            for ch in rng.choice(len(sums_or_inputs), size=k, replace=False):
                bld.link(p, sums_or_inputs[int(ch)])
            new_p.append(p)
        products.extend(new_p)
        new_s = []
        for _ in range(int(rng.integers(1, width + 1))):
            n_real = K if rng.random() < 0.7 else int(rng.integers(1, K + 1))
            sblk = bld.add(SUM, n_real=n_real)
            k = int(rng.integers(1, min(4, len(products)) + 1))
            sum_children[sblk] = [products[int(c)] for c in rng.choice(len(products), size=k, replace=False)]
            new_s.append(sblk)
        sums_or_inputs.extend(new_s)
    root = bld.add(SUM, n_real=1)
    k = int(rng.integers(1, min(4, len(products)) + 1))
    sum_children[root] = [products[int(c)] for c in rng.choice(len(products), size=k, replace=False)]

    n_param_blocks = 0
    owner_of_list: dict[int, list[int]] = {}                # sum block -> its parameter block ids
    by_count: dict[int, list[int]] = {}
    for sblk, chs in sum_children.items():
        donors = [d for d in by_count.get(len(chs), []) if bld.n_real[d] == bld.n_real[sblk]]
        if sblk != root and donors and rng.random() < tie_prob:
            ids = owner_of_list[donors[int(rng.integers(0, len(donors)))]]
        else:
            ids = list(range(n_param_blocks, n_param_blocks + len(chs)))
            n_param_blocks += len(chs)
            by_count.setdefault(len(chs), []).append(sblk)
        owner_of_list[sblk] = ids
        for ch, pid in zip(chs, ids):
            bld.link(sblk, ch, pid)

    theta = np.zeros((n_param_blocks + 1, K, K), dtype=np.float32)
    done = set()
    for sblk, chs in sum_children.items():
        ids = owner_of_list[sblk]
        if ids[0] in done:
            continue
        done.update(ids)
        rows = bld.n_real[sblk]
        Wt = _f32_floor(_dirichlet_rows(rng, alpha, (rows, len(chs) * K)))
        for j, pid in enumerate(ids):
            theta[pid + 1, :rows, :] = Wt[:, j * K:(j + 1) * K]
    tables = np.empty((width, n_cats, K), dtype=np.float32)
    for t in range(width):
        tables[t] = _f32_floor(_dirichlet_rows(rng, min(1.0, 2 * alpha), (K, n_cats))).T
    x = rng.integers(0, n_cats, size=(B, n_vars))
    return _make(name or f"random_v{n_vars}_L{n_levels}_w{width}_K{K}_B{B}_s{seed}", bld, root, n_param_blocks, n_vars, n_cats,
                 width, theta, tables, x, {"kind": "random"})


def non_alternating(n_vars: int, n_levels: int, width: int, K: int, B: int, seed: int, *, n_cats=4, p_insert=0.5,
                    alpha=0.5) -> Workload:
    """non_alternating_from a random_circuit without tying (not normalised in general: plain arithmetic on a DAG)."""
    base = random_circuit(n_vars, n_levels, width, K, B, seed, n_cats=n_cats, tie_prob=0.0, alpha=alpha)
    return non_alternating_from(base, seed, p_insert=p_insert, alpha=alpha)


def non_alternating_from(base: Workload, seed: int, *, p_insert=0.5, alpha=0.5) -> Workload:
    """A DAG with consecutive sum / sum and product / product blocks (the case the footnote to Def. 2 collapses).

    Rewrites a random share of the edges of `base` (an alternating circuit without tied parameters): a sum edge S -> P becomes
    S -> T -> P with a new sum block T (S keeps its row sums: the old K x K weights are replaced by rows of the same
    mass, T gets Dirichlet rows over P and sometimes a second product child), a product edge P -> c becomes
    P -> Q -> c with a new single-child product block Q; chains of two inserted blocks occur as well.  The result is
    normalised whenever the base circuit is smooth, decomposable and normalised (an inserted sum block only mixes
    product blocks of the scope of the edge it replaces when `base` is a tree-shaped circuit such as an HCLT)."""
    K = base.K
    rng = np.random.Generator(np.random.PCG64(seed + 7919))
    bld = _Builder(K)
    for u in range(base.n_blocks):
        bld.add(int(base.type[u]), n_real=int(base.n_real[u]), var=int(base.in_var[u]), table=int(base.in_table[u]))
    mats: list[np.ndarray] = [base.theta[p + 1].astype(np.float64) for p in range(base.n_param_blocks)]
    products = [u for u in range(base.n_blocks) if base.type[u] == PRODUCT]
    mix = base.meta.get("kind") == "random"            # a second, unrelated child keeps a random DAG valid but not a smooth one

    def new_param(M) -> int:
        mats.append(M)
        return len(mats) - 1

    def inserted_sum(child: int, depth: int) -> int:
        """new sum block over `child` (a product block), with probability 1/3 over another inserted sum block"""
        t = bld.add(SUM)
        second = [q for q in products if q < child] if mix else []
        chs = [child] + ([second[int(rng.integers(0, len(second)))]] if second and rng.random() < 0.5 else [])
        Wt = _dirichlet_rows(rng, alpha, (K, len(chs) * K))
        for j, c in enumerate(chs):
            tgt = inserted_sum(c, depth + 1) if depth < 1 and rng.random() < 0.33 else c
            bld.link(t, tgt, new_param(Wt[:, j * K:(j + 1) * K]))
        return t

    for u in range(base.n_blocks):
        for e in range(base.child_ptr[u], base.child_ptr[u + 1]):
            c, pb = int(base.child[e]), int(base.param_blk[e])
            if base.type[u] == SUM and rng.random() < p_insert:
                M = mats[pb]
                A = _dirichlet_rows(rng, alpha, (K, K)) * M.sum(axis=1, keepdims=True)      # same row mass as before
                bld.link(u, inserted_sum(c, 0), new_param(A))
            elif base.type[u] == PRODUCT and rng.random() < p_insert:
                q = bld.add(PRODUCT, n_real=int(base.n_real[c]))
                if rng.random() < 0.33:                                                     # a chain of two
                    q2 = bld.add(PRODUCT, n_real=int(base.n_real[c]))
                    bld.link(q2, c)
                    bld.link(q, q2)
                else:
                    bld.link(q, c)
                bld.link(u, q)
            else:
                bld.link(u, c, pb)
    theta = np.zeros((len(mats) + 1, K, K), dtype=np.float32)
    for p, M in enumerate(mats):
        theta[p + 1] = np.where(M > 0, np.maximum(M, FLT_MIN), 0.0).astype(np.float32)
    return _make(f"nonalt_{base.name}_s{seed}", bld, base.root_block, len(mats), base.n_vars, base.n_cats, base.n_tables, theta,
                 base.tables, base.x, {"kind": "non_alternating"})


# --------------------------------------------------------------------------------------------
# The five benchmark configurations and their reduced twins
# --------------------------------------------------------------------------------------------
DEFAULT_K = {1: 32, 2: 64, 3: 64, 4: 128, 5: 32}


def config(idx: int, *, K: int | None = None, B: int | None = None, draw: bool = True) -> Workload:
    """Full-size configuration `idx` (1-based).  Seed = SEED_BASE + idx.
    draw=False builds the structure only (parameters and data all zero)."""
    K = K or DEFAULT_K[idx]
    seed = SEED_BASE + idx
    if idx == 1:
        return hmm(16, 32, 64, K, B or 128, seed, draw=draw, name=f"cfg1_hmm_T16_H32_V64_B{B or 128}")
    if idx == 2:
        return hclt(784, 128, K, B or 512, seed, data="gauss", draw=draw, name=f"cfg2_hclt_D784_M128_B{B or 512}")
    if idx == 3:
        return hclt(3072, 256, K, B or 256, seed, data="gauss_corr", draw=draw,
                    name=f"cfg3_hclt_D3072_M256_B{B or 256}")
    if idx == 4:
        return hmm(32, 4096, 50257, K, B or 256, seed, alpha_trans=0.1, alpha_emis=0.1, tokens="zipf",
                   keep_dense=False, draw=draw, name=f"cfg4_hmm_T32_H4096_V50257_B{B or 256}")
    if idx == 5:
        return pd(8, 4, 256, K, B or 256, seed, keep=0.25, draw=draw, name=f"cfg5_pd_32x32_M256_keep25_B{B or 256}")
    raise ValueError(idx)


def rat_config(*, K: int | None = None, B: int | None = None, draw: bool = True) -> Workload:
    """RAT-SPN stand-in at the size of the paper's batch-size table (App. D: 465 K nodes, 33.4 M edges): 784 variables,
    depth 4, 4 replicas, 256 sums per region -> 29.4 M sum edges; the node count is larger (940 K) because every
    replica owns its input distributions.  Seed = SEED_BASE + 6."""
    return rat_spn(784, 4, 4, 256, K or 32, B or 512, SEED_BASE + 6, draw=draw, name=f"rat_D784_d4_R4_S256_B{B or 512}")


def reduced(idx: int, *, K: int | None = None, B: int | None = None) -> Workload:
    """Same structure family and value distributions as `config(idx)`, at a size a plain CPU
    implementation finishes in seconds; still spans several blocks and a ragged batch tail."""
    seed = SEED_BASE + 100 + idx
    if idx == 1:
        return hmm(6, 64, 50, K or 32, B or 77, seed)
    if idx == 2:
        return hclt(24, 64, K or 32, B or 100, seed, n_cats=64, data="gauss")
    if idx == 3:
        return hclt(40, 128, K or 64, B or 70, seed, n_cats=32, data="gauss_corr")
    if idx == 4:
        return hmm(5, 256, 1000, K or 64, B or 96, seed, alpha_trans=0.1, alpha_emis=0.1, tokens="zipf")
    if idx == 5:
        return pd(3, 2, 64, K or 32, B or 45, seed, keep=0.25, n_cats=16)
    if idx == 6:
        return rat_spn(24, 2, 2, 64, K or 32, B or 50, seed, n_cats=16)
    raise ValueError(idx)
