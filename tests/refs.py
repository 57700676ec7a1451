"""Textbook reference computations used to pin the oracle (independent of oracle/ and of the GPU path).

Everything here is the classical algorithm for the *model* (HMM, latent tree), not for the circuit:
the circuit oracle must reproduce these numbers because the circuit encodes the same distribution.
Written with torch float64 so that autograd gives d log p / d log(parameter) = expected counts.
"""
import numpy as np
import torch


def hmm_loglik_torch(log_pi, log_A, log_E, x):
    """Forward algorithm in log space.  x: LongTensor [B, T].  Returns [B]."""
    B, T = x.shape
    alpha = log_pi[None, :] + log_E[:, x[:, 0]].T                      # [B, H]
    for t in range(1, T):
        alpha = torch.logsumexp(alpha[:, :, None] + log_A[None, :, :], dim=1) + log_E[:, x[:, t]].T
    return torch.logsumexp(alpha, dim=1)


def hmm_loglik_scaled(pi, A, E, x):
    """Rabiner's scaled forward recursion, float64 numpy, one sequence at a time."""
    out = []
    for seq in x:
        a = pi * E[:, seq[0]]
        c = a.sum(); ll = np.log(c); a = a / c
        for t in range(1, len(seq)):
            a = (a @ A) * E[:, seq[t]]
            c = a.sum(); ll += np.log(c); a = a / c
        out.append(ll)
    return np.array(out)


def hmm_baum_welch_counts(pi, A, E, x):
    """Expected counts by the alpha-beta recursions (float64 numpy, scaled).
    Returns (gamma0 [H], xi [H, H], emis [H, V], ll [B])."""
    H, V = E.shape
    g0 = np.zeros(H); xi = np.zeros((H, H)); em = np.zeros((H, V)); lls = []
    for seq in x:
        T = len(seq)
        al = np.zeros((T, H)); be = np.zeros((T, H)); c = np.zeros(T)
        a = pi * E[:, seq[0]]; c[0] = a.sum(); al[0] = a / c[0]
        for t in range(1, T):
            a = (al[t - 1] @ A) * E[:, seq[t]]; c[t] = a.sum(); al[t] = a / c[t]
        be[T - 1] = 1.0
        for t in range(T - 2, -1, -1):
            be[t] = (A @ (E[:, seq[t + 1]] * be[t + 1])) / c[t + 1]
        gam = al * be
        g0 += gam[0]
        for t in range(T):
            em[:, seq[t]] += gam[t]
        for t in range(T - 1):
            xi += al[t][:, None] * A * (E[:, seq[t + 1]] * be[t + 1])[None, :] / c[t + 1]
        lls.append(np.log(c).sum())
    return g0, xi, em, np.array(lls)


def latent_tree_loglik_torch(parent, order, log_pi, log_W, log_tab, x):
    """Upward sum-product on a rooted latent tree.
    log_W[c]: [M, M] log P(z_c = k' | z_parent = k) (index [k, k']);  log_tab[v]: [M, n_cats];  x: [B, D]."""
    D = len(parent)
    kids = [[] for _ in range(D)]
    for v in order[1:]:
        kids[int(parent[v])].append(v)
    msg = [None] * D
    for v in reversed(order):
        m = log_tab[v][:, x[:, v]].T                                     # [B, M]
        for c in kids[v]:
            m = m + torch.logsumexp(log_W[c][None, :, :] + msg[c][:, None, :], dim=2)
        msg[v] = m
    return torch.logsumexp(log_pi[None, :] + msg[0], dim=1)
