"""Tolerances of the GPU parity tests, derived from the arithmetic of the fp32 path.

Log-likelihoods / node log-probabilities:  |g - o| <= 1e-4 |o| + 1e-5  (the absolute term covers values near 0:
a fully marginalised sample has ll = 0).

Flows (node, parameter, table):  |g - o| <= 1e-3 |o| + floor, where `floor` is only what fp32 cannot hold:

* node flows.  A flow below FLT_MIN = 2^-126 is flushed to zero when it is stored (and the log_nf = log F - l built
  from it becomes -inf).  An absolute error in a node's flow reaches each descendant with a total weight of at most
  one (edge flows of a sum node add up to its flow, Def. 2, and in a decomposable circuit every node's flow is at most
  the root's), so a node's flow is off by at most FLT_MIN per ancestor:  floor = FLT_MIN * (number of nodes).
* table flows are sums of node flows over the samples and the input blocks that share the table:
  floor = (terms per table entry) * node floor.
* parameter flows are theta * sum over samples and tied block pairs of exp(log_nf_s + l_c), computed as a product of
  two fp32 factors that carries the fixed scale e^-24 (see the parameter-flow kernels).  Lost per term:
    - the node-flow error above, passed on with weight theta p_c / p_s <= 1;
    - a product below FLT_MIN, i.e. theta * FLT_MIN * e^24 = theta * 3.2e-28;
    - in a sample whose largest term of the block pair, e^g, exceeds e^23.4 (this takes a weight below e^-23 on an
      edge that carries the pair's largest flow ratio) one factor of a small term can underflow: the term is then
      below e^(g / 2 - 75) <= e^-31.4, times theta.
  floor[entry] = sum over the entry's terms of (node floor + theta[entry] * max(FLT_MIN e^24, [g > 23.4] e^(g/2 - 75))),
  with g taken from the oracle's own node values.  A factor SLACK covers the rounding of g itself.
"""
import numpy as np

LL_RTOL = 1e-4
LL_ATOL = 1e-5
FLOW_RTOL = 1e-3
FLT_MIN = float(np.finfo(np.float32).tiny)
SPLIT_SCALE = 24.0            # the parameter-flow products carry e^-24
SLACK = 4.0

SUM = 2


def node_flow_floor(w):
    return SLACK * FLT_MIN * w.n_blocks * w.K


def table_flow_floor(w, B):
    """One scalar per table: B samples x the input blocks that use the table."""
    users = np.bincount(np.asarray(w.in_table)[np.asarray(w.in_table) >= 0], minlength=w.n_tables)
    return (node_flow_floor(w) * B * np.maximum(users, 1)).reshape(-1, 1, 1)


def theta_flow_floor(w, theta, lp, flow):
    """Array shaped like theta.  lp, flow: the oracle's node log-probabilities and flows [B, n_blocks * K]."""
    K, n = w.K, w.n_blocks
    B = lp.shape[0]
    L = lp.reshape(B, n, K)
    with np.errstate(divide="ignore", invalid="ignore"):
        nf = np.log(flow.reshape(B, n, K)) - L                      # log_nf of Alg. 3; -inf - -inf -> nan
    nf = np.where(np.isnan(nf), -np.inf, nf)
    a = nf.max(axis=2)                                              # [B, n] block maximum of log_nf
    lmax = L.max(axis=2)                                            # [B, n] largest child value of a block
    per_block = np.zeros(w.n_param_blocks + 1)                      # sum over terms of the theta-proportional part
    terms = np.zeros(w.n_param_blocks + 1)
    base = FLT_MIN * np.exp(SPLIT_SCALE)
    for u in np.nonzero(np.asarray(w.type) == SUM)[0]:
        e0, e1 = int(w.child_ptr[u]), int(w.child_ptr[u + 1])
        ch = np.asarray(w.child[e0:e1])
        pb = np.asarray(w.param_blk[e0:e1]) + 1
        with np.errstate(invalid="ignore", over="ignore"):
            g = a[:, u, None] + lmax[:, ch]                         # [B, n_children]
            lost = np.where(g > 23.4, np.exp(0.5 * g - 75.0), 0.0)
        lost = np.maximum(np.where(np.isnan(lost), 0.0, lost), base)
        np.add.at(per_block, pb, lost.sum(axis=0))
        np.add.at(terms, pb, B)
    th = np.asarray(theta, dtype=np.float64)
    return SLACK * (th * per_block[:, None, None] + (terms * node_flow_floor(w) / SLACK)[:, None, None])


def flow_excess(got, ref, floor):
    """Largest |got - ref| - (1e-3 |ref| + floor) and where; <= 0 means within tolerance."""
    err = np.abs(got - ref) - (FLOW_RTOL * np.abs(ref) + floor)
    at = np.unravel_index(np.argmax(err), err.shape)
    return float(err[at]), at


def error_by_decade(got, ref, floor):
    """Rows (decade, count, worst relative error, count below the floor) over the non-zero reference entries: the
    worst relative error is taken over the entries whose reference value exceeds floor / 1e-3 (those the relative
    term alone has to cover)."""
    ref = np.asarray(ref)
    floor = np.broadcast_to(np.asarray(floor, dtype=np.float64), ref.shape).ravel()
    got, ref = np.asarray(got).ravel(), ref.ravel()
    nz = ref > 0
    r, g, f = ref[nz], got[nz], floor[nz]
    rel = np.abs(g - r) / r
    dec = np.floor(np.log10(r)).astype(int)
    rows = []
    for d in range(int(dec.max()), int(dec.min()) - 1, -1):
        sel = dec == d
        if not sel.any():
            continue
        above = sel & (r * FLOW_RTOL > f)
        rows.append((d, int(sel.sum()), float(rel[above].max()) if above.any() else float("nan"), int((sel & ~above).sum())))
    return rows
