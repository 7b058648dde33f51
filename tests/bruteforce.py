"""Exhaustive enumeration on tiny graphs, written from the energy function (Eq. 1 of the
paper) alone: E(x) = sum_i theta_i(x_i) + sum_(i,j) theta_ij(x_i, x_j).  Independent of
the oracle and of the GPU library; used to pin the oracle."""
import itertools

import numpy as np


def all_labelings(n_nodes, L):
    return np.array(list(itertools.product(range(L), repeat=n_nodes)), dtype=np.int64)


def energies(X, unary, edges):
    """X [M,n] labelings; unary [n,L]; edges = list of (src, dst, weight, V) with the
    pairwise term weight * V[x_src][x_dst]."""
    n = unary.shape[0]
    E = np.zeros(X.shape[0], np.float64)
    for i in range(n):
        E += unary[i][X[:, i]]
    for (s, d, w, V) in edges:
        E += w * V[X[:, s], X[:, d]]
    return E


def min_marginals(unary, edges, L):
    n = unary.shape[0]
    X = all_labelings(n, L)
    E = energies(X, unary, edges)
    mm = np.empty((n, L), np.float64)
    for i in range(n):
        for lam in range(L):
            mm[i, lam] = E[X[:, i] == lam].min()
    return mm, X[np.argmin(E)], E.min()
