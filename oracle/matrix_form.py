"""The paper's matrix form of the tree SSM, written out in numpy (fp64).
TEST INFRASTRUCTURE ONLY; meant for tiny trees (it builds N x N matrices).

Follows Sec. 3 step by step, per batch element and head (scalar decay per
head, so diag(log A_i) is the scalar dt_i * A_h):

  1. tree mask      L_ij = 1 iff t_j is on the path from the root to t_i
                    (the indicator definition of L, path inclusive of t_i)
  2. A_tree = L A_log            (Eq. a_tree)
  3. (M_x)_i  = C_i * exp(A_tree_i)
     (M_u)_ij = L_ij * <C_i, B_j> * exp(A_tree_i - A_tree_j)
  4. y = M_x x0 + M_u u (+ D x), with u_j = dt_j x_j the discretised input and
     x0 the initial state h0.

The path membership of step 1 is found by walking parents from each node, which
is a different procedure from the leaf enumeration the C oracle uses.
"""
from __future__ import annotations

import numpy as np


def tree_mask(parent: np.ndarray) -> np.ndarray:
    """L in {0,1}^{N x N} by the indicator definition."""
    n = len(parent)
    L = np.zeros((n, n), dtype=np.float64)
    for i in range(n):
        v = i
        while v >= 0:
            L[i, v] = 1.0
            v = int(parent[v])
    return L


def ssd_matrix(parent, x, dt, A, Bm, Cm, D=None, h0=None) -> np.ndarray:
    """One tree.  x [N,H,P], dt [N,H], A [H], Bm/Cm [N,G,S], D [H] or None,
    h0 [H,P,S] or None.  Returns y [N,H,P] fp64."""
    x, dt, A, Bm, Cm = (np.asarray(a, dtype=np.float64) for a in (x, dt, A, Bm, Cm))
    N, H, P = x.shape
    G, S = Bm.shape[1], Bm.shape[2]
    L = tree_mask(np.asarray(parent))
    y = np.zeros((N, H, P))
    for h in range(H):
        g = h // (H // G)
        a_log = dt[:, h] * A[h]                     # log of the scalar decay of each node
        a_tree = L @ a_log                          # Eq. a_tree
        CB = Cm[:, g, :] @ Bm[:, g, :].T            # <C_i, B_j>
        diff = a_tree[:, None] - a_tree[None, :]
        M_u = np.where(L > 0, CB * np.exp(np.where(L > 0, diff, 0.0)), 0.0)
        u = dt[:, h, None] * x[:, h, :]
        y[:, h, :] = M_u @ u
        if h0 is not None:
            x0 = np.asarray(h0, dtype=np.float64)[h]            # [P,S]
            M_x = Cm[:, g, :] * np.exp(a_tree)[:, None]        # [N,S]
            y[:, h, :] += M_x @ x0.T
        if D is not None:
            y[:, h, :] += float(np.asarray(D)[h]) * x[:, h, :]
    return y
