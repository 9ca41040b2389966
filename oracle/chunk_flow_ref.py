"""numpy fp64 statement of the chunk flow of ParallelFlow (arXiv 2504.00492), Section 3.1-3.2.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).  It exists so that the sequential recurrence
in pf_oracle.c can be pinned against the paper's own second route to the same numbers, and so
that every identity the GPU kernels rely on is checked on the CPU first.

Conventions.  "Row form" of the Remark after Theorem 3.2: a chunk of L tokens with rank R is
stored as A, Bm in R^{L x R x d_k}, Atil in R^{L x R x d_v}; A[t, i, :] is column i of the paper's
d x R matrix A_t.  Flattening (t, i) -> t*R + i is the isomorphism used in the proof of
Proposition 3.3, under which tensor composition is the ordinary matrix product.

State S is d_v x d_k.  The paper writes d x d; with d_v != d_k the shapes that make every product
well defined are W in R^{n x d_k} and U in R^{n x d_v}, n = L*R.
"""
from __future__ import annotations

import numpy as np


def delta_drivers(K, V, beta):
    """Delta-rule drivers (Remark in Section 3.1, column by column for rank R).

    K [L,R,dk], V [L,R,dv], beta [L,R]  ->  A = beta k, Atil = -beta v, Bm = -k.
    """
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    beta = np.asarray(beta, dtype=np.float64)
    return beta[..., None] * K, -beta[..., None] * V, -K


def strict_time_mask(L, R):
    """M of Theorem 3.2: entry ((t,i),(s,j)) is 1 iff s < t, whatever i and j are."""
    tok = np.repeat(np.arange(L), R)
    return (tok[None, :] < tok[:, None]).astype(np.float64)


def inclusive_time_mask(L, R):
    """Readout mask: entry (t,(s,j)) is 1 iff s <= t (token t's own R columns are included,
    because the readout of Section 1.1 uses the state that already holds token t)."""
    tok = np.repeat(np.arange(L), R)
    return (tok[None, :] <= np.arange(L)[:, None]).astype(np.float64)


def system_matrix(A, Bm):
    """Id - M (.) A B^T as an n x n matrix (Theorem 3.2)."""
    L, R, dk = A.shape
    n = L * R
    AB = A.reshape(n, dk) @ Bm.reshape(n, dk).T
    return np.eye(n) - strict_time_mask(L, R) * AB


def block_tri_inverse(Cmat, R):
    """Proposition 3.3: inverse of a block lower-triangular matrix with invertible R x R
    diagonal blocks, by block forward substitution.  Written for general diagonal blocks
    even though Theorem 3.2 only ever produces identity blocks there."""
    n = Cmat.shape[0]
    T = n // R
    D = np.zeros_like(Cmat)
    blk = lambda X, t, s: X[t * R:(t + 1) * R, s * R:(s + 1) * R]
    for t in range(T):
        Dtt = np.linalg.inv(blk(Cmat, t, t))
        D[t * R:(t + 1) * R, t * R:(t + 1) * R] = Dtt
        for s in range(t):
            acc = np.zeros((R, R))
            for r in range(s, t):
                acc += blk(Cmat, t, r) @ blk(D, r, s)
            D[t * R:(t + 1) * R, s * R:(s + 1) * R] = -Dtt @ acc
    return D


def chunk_flow(A, Atil, Bm):
    """W = (Id - M (.) A B^T)^{-1} A and U = (same)^{-1} Atil   (Theorem 3.2).
    Returns W [n, dk], U [n, dv]."""
    L, R, dk = A.shape
    n = L * R
    D = block_tri_inverse(system_matrix(A, Bm), R)
    return D @ A.reshape(n, dk), D @ Atil.reshape(n, -1)


def chunk_state(S0, W, U, Bm):
    """S_1 = S_0 + (U + W S_0^T)^T B   (Theorem 3.2)."""
    n = W.shape[0]
    return S0 + (U + W @ S0.T).T @ Bm.reshape(n, -1)


def chunk_readout(Q, S0, W, U, Bm):
    """o_t = S_t q_t for every token t of the chunk, from the same W and U.

    The discrete flow of Section 3.1 truncated at token t gives
    S_t = S_0 + sum_{s<=t} sum_j (S_0 w_{s,j} + u_{s,j}) b_{s,j}^T, because w and u of a token
    depend on earlier tokens only.  Stacking rows:
    O = Q S_0^T + (Mbar (.) Q B^T)(U + W S_0^T)."""
    L = Q.shape[0]
    n = W.shape[0]
    R = n // L
    QB = Q @ Bm.reshape(n, -1).T
    return Q @ S0.T + (inclusive_time_mask(L, R) * QB) @ (U + W @ S0.T)


def chunked_forward(A, Atil, Bm, Q, S0, chunk):
    """Whole sequence by chunks of `chunk` tokens: flow per chunk, readout inside the chunk,
    state handed over at the boundary (the three steps listed in Section 3).  L % chunk == 0."""
    L, R, dk = A.shape
    dv = Atil.shape[2]
    assert L % chunk == 0
    S = np.array(S0, dtype=np.float64, copy=True)
    O = np.empty((L, dv))
    for c0 in range(0, L, chunk):
        sl = slice(c0, c0 + chunk)
        W, U = chunk_flow(A[sl], Atil[sl], Bm[sl])
        O[sl] = chunk_readout(Q[sl], S, W, U, Bm[sl])
        S = chunk_state(S, W, U, Bm[sl])
    return O, S


def sig_delta_grid(X, A, Bm):
    """Diagonal of the grid system of Theorem 3.4 with inhomogeneous term X (no inverse anywhere).

    X = A gives W; X = Atil gives U, which solves the same implicit equation with Atil in place of
    the leading A (discrete flow of Section 3.1: U_k = Atil_k + sum_{m<k} U_m B_m^T A_k), so every
    step of the theorem's proof goes through with Y(t_0, t_k) = X_k.
    Column form as in the theorem: grid value Y(t_m, t_k) in R^{dx x R}, m <= k.
    Returns the diagonal in row form [n, dx]."""
    L, R, dk = A.shape
    dx = X.shape[2]
    Xt = [X[k].T for k in range(L)]     # dx x R
    At = [A[k].T for k in range(L)]     # dk x R
    Bt = [Bm[k].T for k in range(L)]    # dk x R
    G = [[None] * L for _ in range(L)]  # G[m][k] = Y(t_m, t_k)
    for k in range(L):
        G[0][k] = Xt[k].copy()
    for k in range(L - 1):
        for m in range(k):
            G[m + 1][k + 1] = (G[m][k + 1] + G[m + 1][k] - G[m][k]
                               + G[m][m] @ (Bt[m].T @ (At[k + 1] - At[k])))
        G[k + 1][k + 1] = G[k][k + 1] + G[k][k] @ (Bt[k].T @ At[k + 1])
    return np.stack([G[k][k].T for k in range(L)]).reshape(L * R, dx)


def sig_delta_W(A, Bm):
    """W of one chunk by the grid recursion of Theorem 3.4.  Returns W in row form [n, dk]."""
    return sig_delta_grid(A, A, Bm)


def propagator_from_flow(W, Bm):
    """P_{0,1} = Id + sum_k W_k B_k^T  (from W_{s,t} = P_{s,t} A_t in the proof of
    Proposition 3.1 and P = Id + int P dw of Proposition 2.1).  Returns dk x dk."""
    n, dk = W.shape
    return np.eye(dk) + W.T @ Bm.reshape(n, dk)


def exp_rank1_beta(K, beta):
    """Step size that makes a rank-1 delta step the exact flow of its increment (Section 3.3).

    For rank-1 increments the exponential of Section 3.3 has the closed form
    exp(a b^T) = Id + phi(<b, a>) a b^T with phi(x) = (e^x - 1) / x.  Under the delta mapping
    (a = beta k, b = -k) <b, a> = -beta |k|^2, so exp(d omega) = Id - beta_eff k k^T with
    beta_eff = (1 - exp(-beta |k|^2)) / |k|^2.  The input increment, carried by the same flow over
    the step (S' = S a b^T + atil b^T on [0, 1]), picks up the same factor phi, so the exact step is
    the delta rule with beta_eff in place of beta.  |k| = 0 gives beta_eff = beta (phi(0) = 1).
    K [..., dk], beta [...] -> beta_eff [...]."""
    K = np.asarray(K, dtype=np.float64)
    beta = np.asarray(beta, dtype=np.float64)
    s = np.sum(K * K, axis=-1)
    safe = np.where(s > 0, s, 1.0)
    return np.where(s > 0, -np.expm1(-beta * safe) / safe, beta)
