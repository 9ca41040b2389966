"""Pins of the fp64 oracle against what the paper and the mathematics fix (CPU only).

Each test names the passage it leans on.  Together they are chosen so that a dropped term, a
wrong sign, a transposed operand, an off-by-one mask or a pre/post-update readout mix-up in
oracle/pf_oracle.c (or in oracle/chunk_flow_ref.py) fails at least one of them.
"""
import json
import os

import numpy as np
import pytest
import scipy.linalg

from oracle import chunk_flow_ref as cf

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand_delta(rng, L, r, dk, dv, beta_hi=1.0, unit=True, s0=True):
    K = rng.standard_normal((L, r, dk))
    if unit:
        K /= np.linalg.norm(K, axis=-1, keepdims=True)
    V = rng.standard_normal((L, r, dv))
    beta = rng.uniform(0.0, beta_hi, (L, r))
    Q = rng.standard_normal((L, dk))
    S0 = rng.standard_normal((dv, dk)) if s0 else np.zeros((dv, dk))
    return Q, K, V, beta, S0


def _oracle_delta64(oracle, Q, K, V, beta, S0):
    """Delta form in full fp64 through the general-driver entry (no fp32 narrowing)."""
    A, At, Bm = cf.delta_drivers(K, V, beta)
    return oracle.flow_head(A, At, Bm, Q, S0)


# ---------------------------------------------------------------- hand-worked values
@pytest.mark.parametrize("case", ["rank1", "rank2_sum_not_product", "rank2_orthonormal_overwrite"])
def test_hand_worked_examples(oracle, case):
    """tests/golden/hand_worked_delta.json: Section 1.3 (DeltaNet) and Section 3.1 dynamics."""
    g = json.load(open(os.path.join(GOLDEN, "hand_worked_delta.json")))[case]
    K, V, beta, Q, S0 = (np.array(g[x], float) for x in ("k", "v", "beta", "q", "S0"))
    O, SL = _oracle_delta64(oracle, Q, K, V, beta, S0)
    np.testing.assert_allclose(O, np.array(g["O"], float), rtol=0, atol=1e-13)
    np.testing.assert_allclose(SL, np.array(g["S_L"], float), rtol=0, atol=1e-13)
    # and through the batched float32 entry point the GPU tests use
    O2, SL2 = oracle.delta_fwd(Q[None], K[None], V[None], beta[None], S0[None])
    np.testing.assert_allclose(O2[0], np.array(g["O"], float), rtol=0, atol=2e-6)
    np.testing.assert_allclose(SL2[0], np.array(g["S_L"], float), rtol=0, atol=2e-6)


# ---------------------------------------------------------------- P1 linear attention
@pytest.mark.parametrize("seed", [0, 1])
def test_identity_transition_is_causal_linear_attention(oracle, seed):
    """A_t = I (Section 1.1, last sentence): O = (Q K^T (.) M) V with the standard causal mask
    (Section 1.2) and S_L = S0 + V^T K.  Drivers A = 0, Atil = v, B = k."""
    rng = np.random.default_rng(seed)
    L, dk, dv = 13, 5, 3
    Q, K, V = rng.standard_normal((L, dk)), rng.standard_normal((L, dk)), rng.standard_normal((L, dv))
    S0 = rng.standard_normal((dv, dk))
    O, SL = oracle.flow_head(np.zeros((L, 1, dk)), V[:, None], K[:, None], Q, S0)
    ref = np.tril(Q @ K.T) @ V + Q @ S0.T
    np.testing.assert_allclose(O, ref, atol=1e-12)
    np.testing.assert_allclose(SL, S0 + V.T @ K, atol=1e-12)
    # with S0 = None the textbook formula holds verbatim
    O0, _ = oracle.flow_head(np.zeros((L, 1, dk)), V[:, None], K[:, None], Q, None)
    np.testing.assert_allclose(O0, np.tril(Q @ K.T) @ V, atol=1e-12)


# ---------------------------------------------------------------- P2 beta = 0
def test_beta_zero_leaves_state_unchanged(oracle):
    """Section 1.3: with beta = 0 the DeltaNet update is S_t = S_{t-1}; o_t = S0 q_t."""
    rng = np.random.default_rng(2)
    Q, K, V, beta, S0 = _rand_delta(rng, 9, 2, 6, 4)
    O, SL = _oracle_delta64(oracle, Q, K, V, np.zeros_like(beta), S0)
    assert np.array_equal(SL, S0)
    np.testing.assert_allclose(O, Q @ S0.T, atol=1e-13)
    Of, SLf = oracle.delta_fwd(Q[None], K[None], V[None], np.zeros_like(beta)[None], S0[None])
    assert np.array_equal(SLf[0], S0.astype(np.float32).astype(np.float64))


# ---------------------------------------------------------------- P3 projection, P4 reflection
def test_unit_key_beta_one_projects_and_writes_value(oracle):
    """Section 1.3: A = I - k k^T with |k| = 1 is idempotent, and the delta rule stores the
    value: after the update S_t k_t = v_t."""
    rng = np.random.default_rng(3)
    dk, dv = 7, 5
    k = rng.standard_normal(dk); k /= np.linalg.norm(k)
    v = rng.standard_normal(dv)
    S0 = rng.standard_normal((dv, dk))
    zero_v = np.zeros(dv)
    # one token with v = 0 applies A once; two identical tokens apply it twice
    _, S1 = _oracle_delta64(oracle, np.zeros((1, dk)), k[None, None], zero_v[None, None], np.ones((1, 1)), S0)
    _, S2 = _oracle_delta64(oracle, np.zeros((2, dk)), np.stack([k, k])[:, None],
                            np.zeros((2, 1, dv)), np.ones((2, 1)), S0)
    np.testing.assert_allclose(S1, S0 @ (np.eye(dk) - np.outer(k, k)), atol=1e-13)
    np.testing.assert_allclose(S2, S1, atol=1e-13)          # idempotent
    O, S = _oracle_delta64(oracle, k[None], k[None, None], v[None, None], np.ones((1, 1)), S0)
    np.testing.assert_allclose(S @ k, v, atol=1e-13)         # value written
    np.testing.assert_allclose(O[0], v, atol=1e-13)          # readout sees the updated state


def test_unit_key_beta_two_is_an_involution(oracle):
    """Section 1.3: A = I - 2 k k^T is a reflection; applying it twice restores S."""
    rng = np.random.default_rng(4)
    dk, dv = 6, 6
    k = rng.standard_normal(dk); k /= np.linalg.norm(k)
    S0 = rng.standard_normal((dv, dk))
    _, S2 = _oracle_delta64(oracle, np.zeros((2, dk)), np.stack([k, k])[:, None],
                            np.zeros((2, 1, dv)), 2 * np.ones((2, 1)), S0)
    np.testing.assert_allclose(S2, S0, atol=1e-13)


# ---------------------------------------------------------------- P12 literal equation
@pytest.mark.parametrize("r", [1, 3])
def test_matches_literal_equation_in_numpy(oracle, r):
    """Section 1.3 (r = 1) / Section 3.1 dynamics (r > 1) typed out with numpy matrices:
    S <- S (I - sum_j beta_j k_j k_j^T) + sum_j beta_j v_j k_j^T ;  o = S q."""
    rng = np.random.default_rng(5 + r)
    L, dk, dv = 11, 6, 4
    Q, K, V, beta, S0 = _rand_delta(rng, L, r, dk, dv, beta_hi=2.0)
    S = S0.copy()
    Oref = np.empty((L, dv))
    for t in range(L):
        T = np.eye(dk) - sum(beta[t, j] * np.outer(K[t, j], K[t, j]) for j in range(r))
        S = S @ T + sum(beta[t, j] * np.outer(V[t, j], K[t, j]) for j in range(r))
        Oref[t] = S @ Q[t]
    O, SL = _oracle_delta64(oracle, Q, K, V, beta, S0)
    np.testing.assert_allclose(O, Oref, atol=1e-12)
    np.testing.assert_allclose(SL, S, atol=1e-12)


def test_rank_r_with_one_active_column_equals_rank_one(oracle):
    """Remark in Section 3.1: R = 1 is the special case; zero betas are identity columns."""
    rng = np.random.default_rng(8)
    L, dk, dv = 10, 5, 5
    Q, K, V, beta, S0 = _rand_delta(rng, L, 3, dk, dv)
    beta[:, 0] = 0.0
    beta[:, 2] = 0.0
    O3, S3 = _oracle_delta64(oracle, Q, K, V, beta, S0)
    O1, S1 = _oracle_delta64(oracle, Q, K[:, 1:2], V[:, 1:2], beta[:, 1:2], S0)
    np.testing.assert_allclose(O3, O1, atol=1e-13)
    np.testing.assert_allclose(S3, S1, atol=1e-13)


# ---------------------------------------------------------------- P5 chunked == sequential
@pytest.mark.parametrize("r", [1, 2, 4])
@pytest.mark.parametrize("L", [12])
def test_chunked_flow_equals_sequential_for_every_chunk_size(oracle, L, r):
    """Theorem 3.2 + discrete flow of Section 3.1 + the three-step recipe of Section 3:
    for every chunk length dividing L (1 = the recurrence itself, L = fully parallel)."""
    rng = np.random.default_rng(10 + r)
    dk, dv = 5, 3
    Q, K, V, beta, S0 = _rand_delta(rng, L, r, dk, dv, beta_hi=2.0)
    A, At, Bm = cf.delta_drivers(K, V, beta)
    O, SL = oracle.flow_head(A, At, Bm, Q, S0)
    for C in [c for c in range(1, L + 1) if L % c == 0]:
        Oc, Sc = cf.chunked_forward(A, At, Bm, Q, S0, C)
        np.testing.assert_allclose(Oc, O, atol=2e-12, err_msg=f"C={C}")
        np.testing.assert_allclose(Sc, SL, atol=2e-12, err_msg=f"C={C}")


def test_chunked_flow_general_drivers(oracle):
    """Same, for arbitrary shared-B low-rank drivers (Section 3.1, driver parameterisation),
    not only the delta mapping."""
    rng = np.random.default_rng(20)
    L, R, dk, dv = 8, 2, 4, 6
    A = 0.4 * rng.standard_normal((L, R, dk))
    At = rng.standard_normal((L, R, dv))
    Bm = rng.standard_normal((L, R, dk))
    Q = rng.standard_normal((L, dk))
    S0 = rng.standard_normal((dv, dk))
    O, SL = oracle.flow_head(A, At, Bm, Q, S0)
    for C in (1, 2, 4, 8):
        Oc, Sc = cf.chunked_forward(A, At, Bm, Q, S0, C)
        np.testing.assert_allclose(Oc, O, atol=1e-11)
        np.testing.assert_allclose(Sc, SL, atol=1e-11)


# ---------------------------------------------------------------- P6 triangular inverse
def test_block_triangular_inverse(oracle):
    """Proposition 3.3: D C = Id, for general invertible diagonal blocks; and the solve agrees
    with scipy's triangular routine on the unit-diagonal system of Theorem 3.2."""
    rng = np.random.default_rng(30)
    T, R = 6, 3
    n = T * R
    Cm = np.tril(rng.standard_normal((n, n)))
    tok = np.repeat(np.arange(T), R)
    Cm = Cm * (tok[None, :] <= tok[:, None])            # block lower triangular
    for t in range(T):                                   # full (non-triangular) diagonal blocks
        Cm[t * R:(t + 1) * R, t * R:(t + 1) * R] = rng.standard_normal((R, R)) + 3 * np.eye(R)
    D = cf.block_tri_inverse(Cm, R)
    np.testing.assert_allclose(D @ Cm, np.eye(n), atol=1e-11)
    assert np.all(D[tok[None, :] > tok[:, None]] == 0)

    L, r, dk, dv = 9, 2, 5, 4
    Q, K, V, beta, S0 = _rand_delta(rng, L, r, dk, dv, beta_hi=2.0)
    A, At, Bm = cf.delta_drivers(K, V, beta)
    W, U = cf.chunk_flow(A, At, Bm)
    Csys = cf.system_matrix(A, Bm)
    # the system matrix in delta variables is Id + M (.) diag(beta) K K^T
    Kf, bf = K.reshape(L * r, dk), beta.reshape(L * r)
    np.testing.assert_allclose(Csys, np.eye(L * r) + cf.strict_time_mask(L, r) * (bf[:, None] * (Kf @ Kf.T)),
                               atol=1e-14)
    Wl = scipy.linalg.solve_triangular(Csys, A.reshape(L * r, dk), lower=True, unit_diagonal=True)
    Ul = scipy.linalg.solve_triangular(Csys, At.reshape(L * r, dv), lower=True, unit_diagonal=True)
    np.testing.assert_allclose(W, Wl, atol=1e-12)
    np.testing.assert_allclose(U, Ul, atol=1e-12)


# ---------------------------------------------------------------- P7 propagator
def test_flow_propagator_is_ordered_product(oracle):
    """Proposition 2.1 / proof of Proposition 3.1 (W = P A): Id + sum_k W_k B_k^T equals the
    time-ordered product of the per-token transitions, left to right."""
    rng = np.random.default_rng(40)
    L, r, dk, dv = 7, 2, 5, 3
    Q, K, V, beta, S0 = _rand_delta(rng, L, r, dk, dv, beta_hi=2.0)
    A, At, Bm = cf.delta_drivers(K, V, beta)
    W, _ = cf.chunk_flow(A, At, Bm)
    P = np.eye(dk)
    for t in range(L):
        P = P @ (np.eye(dk) - sum(beta[t, j] * np.outer(K[t, j], K[t, j]) for j in range(r)))
    np.testing.assert_allclose(cf.propagator_from_flow(W, Bm), P, atol=1e-12)
    # and the oracle's S_L with v = 0 is S0 P
    _, SL = _oracle_delta64(oracle, Q, K, np.zeros_like(V), beta, S0)
    np.testing.assert_allclose(SL, S0 @ P, atol=1e-12)


# ---------------------------------------------------------------- P8 Theorem 3.4
@pytest.mark.parametrize("R", [1, 2])
def test_signature_grid_recursion_gives_same_W(oracle, R):
    """Theorem 3.4: the diagonal of the grid system solves the implicit equation for W."""
    rng = np.random.default_rng(50 + R)
    L, dk = 9, 4
    A = 0.5 * rng.standard_normal((L, R, dk))
    Bm = rng.standard_normal((L, R, dk))
    At = rng.standard_normal((L, R, 3))
    W, U = cf.chunk_flow(A, At, Bm)
    np.testing.assert_allclose(cf.sig_delta_W(A, Bm), W, atol=1e-10)
    # the same grid with Atil as inhomogeneous term gives U (it solves the same implicit equation)
    np.testing.assert_allclose(cf.sig_delta_grid(At, A, Bm), U, atol=1e-10)
    # and both satisfy that implicit equation, written out token by token
    for k in range(L):
        acc_w, acc_u = A[k].T.copy(), At[k].T.copy()
        for m in range(k):
            coef = Bm[m] @ A[k].T                                  # B_m^T A_k, R x R
            acc_w += W[m * R:(m + 1) * R].T @ coef
            acc_u += U[m * R:(m + 1) * R].T @ coef
        np.testing.assert_allclose(W[k * R:(k + 1) * R].T, acc_w, atol=1e-10)
        np.testing.assert_allclose(U[k * R:(k + 1) * R].T, acc_u, atol=1e-10)


# ---------------------------------------------------------------- P9 orthonormal keys
def test_orthonormal_keys_closed_form(oracle):
    """With mutually orthonormal keys M (.) A B^T = 0 (Theorem 3.2), hence W = A, U = Atil and
    S_L = S0 (I - sum beta k k^T) + sum beta v k^T; with beta = 1 every value is recalled."""
    rng = np.random.default_rng(60)
    L, r, dk, dv = 3, 2, 8, 5
    Qo, _ = np.linalg.qr(rng.standard_normal((dk, dk)))
    K = Qo[:L * r].reshape(L, r, dk)
    V = rng.standard_normal((L, r, dv))
    beta = rng.uniform(0.2, 1.8, (L, r))
    S0 = rng.standard_normal((dv, dk))
    Qm = rng.standard_normal((L, dk))
    A, At, Bm = cf.delta_drivers(K, V, beta)
    W, U = cf.chunk_flow(A, At, Bm)
    np.testing.assert_allclose(W, A.reshape(L * r, dk), atol=1e-13)
    np.testing.assert_allclose(U, At.reshape(L * r, dv), atol=1e-13)
    Kf, Vf, bf = K.reshape(-1, dk), V.reshape(-1, dv), beta.reshape(-1)
    closed = S0 @ (np.eye(dk) - (Kf.T * bf) @ Kf) + (Vf.T * bf) @ Kf
    _, SL = _oracle_delta64(oracle, Qm, K, V, beta, S0)
    np.testing.assert_allclose(SL, closed, atol=1e-12)
    _, SL1 = _oracle_delta64(oracle, Qm, K, V, np.ones_like(beta), S0)
    np.testing.assert_allclose(SL1 @ Kf.T, Vf.T, atol=1e-12)


# ---------------------------------------------------------------- P10 linearity, P11 composition
def test_linearity_in_values_and_initial_state(oracle):
    """Section 3.1 dynamics are linear in (V, S0) for fixed K, beta, Q."""
    rng = np.random.default_rng(70)
    L, r, dk, dv = 10, 2, 5, 4
    Q, K, V1, beta, S01 = _rand_delta(rng, L, r, dk, dv, beta_hi=2.0)
    V2, S02 = rng.standard_normal(V1.shape), rng.standard_normal(S01.shape)
    a, b = 0.7, -1.3
    O1, S1 = _oracle_delta64(oracle, Q, K, V1, beta, S01)
    O2, S2 = _oracle_delta64(oracle, Q, K, V2, beta, S02)
    O3, S3 = _oracle_delta64(oracle, Q, K, a * V1 + b * V2, beta, a * S01 + b * S02)
    np.testing.assert_allclose(O3, a * O1 + b * O2, atol=1e-12)
    np.testing.assert_allclose(S3, a * S1 + b * S2, atol=1e-12)


def test_split_sequence_composes_through_the_state(oracle):
    """Proposition 2.1: the flow over [0, L) is the flow over [0, L1) followed by [L1, L)."""
    rng = np.random.default_rng(80)
    L, L1, r, dk, dv = 14, 5, 2, 4, 6
    Q, K, V, beta, S0 = _rand_delta(rng, L, r, dk, dv, beta_hi=2.0)
    O, SL = _oracle_delta64(oracle, Q, K, V, beta, S0)
    Oa, Sa = _oracle_delta64(oracle, Q[:L1], K[:L1], V[:L1], beta[:L1], S0)
    Ob, Sb = _oracle_delta64(oracle, Q[L1:], K[L1:], V[L1:], beta[L1:], Sa)
    assert np.array_equal(np.concatenate([Oa, Ob]), O)
    assert np.array_equal(Sb, SL)


# ---------------------------------------------------------------- P13 one-chunk S1, transposition
def test_state_formula_needs_the_transpose(oracle):
    """Theorem 3.2: S_1 = S_0 + (U + W S_0^T)^T B.  With a non-symmetric S_0 and d_v != d_k the
    variant without the transpose (W S_0) is either ill-shaped or wrong; the oracle sides
    with the theorem."""
    rng = np.random.default_rng(90)
    L, r, d = 6, 2, 5
    Q, K, V, beta, S0 = _rand_delta(rng, L, r, d, d, beta_hi=1.5)
    A, At, Bm = cf.delta_drivers(K, V, beta)
    W, U = cf.chunk_flow(A, At, Bm)
    _, SL = oracle.flow_head(A, At, Bm, Q, S0)
    np.testing.assert_allclose(cf.chunk_state(S0, W, U, Bm), SL, atol=1e-12)
    wrong = S0 + (U + W @ S0).T @ Bm.reshape(L * r, d)
    assert np.abs(wrong - SL).max() > 1e-3


# ---------------------------------------------------------------- batched float entry
def test_batched_float_entry_matches_per_head_double(oracle):
    """pf_oracle_delta_fwd (float inputs, OpenMP over heads) == per-head general routine."""
    rng = np.random.default_rng(100)
    N, L, r, dk, dv = 3, 9, 2, 6, 4
    Q = rng.standard_normal((N, L, dk)).astype(np.float32)
    K = rng.standard_normal((N, L, r, dk)).astype(np.float32)
    V = rng.standard_normal((N, L, r, dv)).astype(np.float32)
    beta = rng.uniform(0, 2, (N, L, r)).astype(np.float32)
    S0 = rng.standard_normal((N, dv, dk)).astype(np.float32)
    O, SL = oracle.delta_fwd(Q, K, V, beta, S0, nthreads=2)
    for h in range(N):
        Oh, Sh = _oracle_delta64(oracle, Q[h], K[h], V[h], beta[h], S0[h])
        assert np.array_equal(O[h], Oh) and np.array_equal(SL[h], Sh)
    O2, SL2 = oracle.delta_fwd(Q, K, V, beta, None, want_O=False)
    assert O2 is None and SL2.shape == (N, dv, dk)


def test_empty_sequence(oracle):
    dk, dv = 4, 3
    S0 = np.arange(12, dtype=np.float64).reshape(dv, dk)
    O, SL = oracle.flow_head(np.zeros((0, 1, dk)), np.zeros((0, 1, dv)), np.zeros((0, 1, dk)),
                             np.zeros((0, dk)), S0)
    assert O.shape == (0, dv) and np.array_equal(SL, S0)


# ---------------------------------------------------------------- product form (contrast case)
def test_product_form_is_the_ordered_product_of_rank_one_factors(oracle):
    """The product-form oracle against the definition written out in numpy: per token r factors
    (I - beta k k^T) applied left to right, each with its own input term; readout after the last."""
    rng = np.random.default_rng(90)
    L, r, dk, dv = 6, 3, 5, 4
    Q, K, V, beta, S0 = _rand_delta(rng, L, r, dk, dv, beta_hi=2.0)
    O, SL = oracle.delta_product_fwd(Q, K, V, beta, S0)
    K32, V32, Q32, b32, S032 = (np.asarray(x, dtype=np.float32).astype(np.float64) for x in (K, V, Q, beta, S0))
    S = S032.copy()
    for t in range(L):
        for j in range(r):
            k, v, b = K32[t, j], V32[t, j], b32[t, j]
            S = S @ (np.eye(dk) - b * np.outer(k, k)) + b * np.outer(v, k)
        np.testing.assert_allclose(O[t], S @ Q32[t], atol=1e-12)
    np.testing.assert_allclose(SL, S, atol=1e-12)


def test_product_form_against_additive_form(oracle):
    """r = 1: the two forms are the same recurrence.  Keys of one token mutually orthogonal: the
    factors commute and their product is I - sum beta k k^T, and each input term passes the later
    factors unchanged, so the forms agree.  Correlated keys: they differ (the contrast is real)."""
    rng = np.random.default_rng(91)
    L, dk, dv = 5, 6, 3
    Q, K, V, beta, S0 = _rand_delta(rng, L, 1, dk, dv)
    Oa, Sa = oracle.delta_fwd(Q, K, V, beta, S0)
    Op, Sp = oracle.delta_product_fwd(Q, K, V, beta, S0)
    np.testing.assert_allclose(Op, Oa, atol=1e-12)
    np.testing.assert_allclose(Sp, Sa, atol=1e-12)
    r = 2
    Q, K, V, beta, S0 = _rand_delta(rng, L, r, dk, dv)
    for t in range(L):                                   # orthonormalise the two keys of each token
        K[t] = np.linalg.qr(K[t].T)[0].T
    K = K.astype(np.float32).astype(np.float64)
    Oa, Sa = oracle.delta_fwd(Q, K, V, beta, S0)
    Op, Sp = oracle.delta_product_fwd(Q, K, V, beta, S0)
    np.testing.assert_allclose(Op, Oa, atol=1e-5)        # keys orthogonal up to the fp32 rounding of K
    np.testing.assert_allclose(Sp, Sa, atol=1e-5)
    Q, K, V, beta, S0 = _rand_delta(rng, L, r, dk, dv)   # generic (correlated) keys
    _, Sa = oracle.delta_fwd(Q, K, V, beta, S0)
    _, Sp = oracle.delta_product_fwd(Q, K, V, beta, S0)
    assert np.abs(Sa - Sp).max() > 1e-3


# ---------------------------------------------------------------- Section 3.3, rank-1 exponential
def test_exponential_step_matches_matrix_exponential(oracle):
    """exp(a b^T) for the delta increment against scipy's expm, and the whole step (transition and
    input) against the exact flow of S' = S a b^T + atil b^T over [0, 1], computed with expm of
    the augmented generator.  Then the small-step limit and |k| = 0."""
    from scipy.linalg import expm
    rng = np.random.default_rng(95)
    dk, dv = 5, 3
    for beta in (0.05, 0.7, 1.9, 4.0):
        k = rng.standard_normal(dk) * rng.uniform(0.3, 1.5)
        v = rng.standard_normal(dv)
        S0 = rng.standard_normal((dv, dk))
        be = float(cf.exp_rank1_beta(k, beta))
        a, b, at = beta * k, -k, -beta * v
        np.testing.assert_allclose(expm(np.outer(a, b)), np.eye(dk) - be * np.outer(k, k), atol=1e-12)
        # augmented system: [S 1] ' = [S 1] [[a b^T, 0], [atil b^T, 0]]  (row vectors, one row of S at a time)
        gen = np.zeros((dk + dv, dk + dv))
        gen[:dk, :dk] = np.outer(a, b)
        gen[dk:, :dk] = np.outer(at, b)
        E = expm(gen)
        S1_exact = S0 @ E[:dk, :dk] + E[dk:, :dk]
        S1_step = S0 @ (np.eye(dk) - be * np.outer(k, k)) + be * np.outer(v, k)
        np.testing.assert_allclose(S1_step, S1_exact, atol=1e-12)
        # the delta-rule oracle run with beta_eff is that exact step
        _, SL = oracle.flow_head((be * k)[None, None], (-be * v)[None, None], (-k)[None, None],
                                 np.zeros((1, dk)), S0)
        np.testing.assert_allclose(SL, S1_exact, atol=1e-12)
    k = rng.standard_normal(dk)
    s = k @ k
    np.testing.assert_allclose(cf.exp_rank1_beta(k, 1e-4), 1e-4 - 0.5e-8 * s, rtol=1e-6)   # Euler is the first order
    assert cf.exp_rank1_beta(np.zeros(dk), 0.8) == 0.8
    # unit keys: beta_eff = 1 - exp(-beta) stays below 1, whatever beta is (no reflection)
    ku = k / np.linalg.norm(k)
    np.testing.assert_allclose(cf.exp_rank1_beta(ku, np.array([0.5, 2.0, 50.0])), 1 - np.exp(-np.array([0.5, 2.0, 50.0])), rtol=1e-12)


def test_streaming_compare_returns_the_sums_of_a_known_perturbation(oracle):
    """delta_compare holds a candidate against the recurrence and returns sums only.  Pin: with a
    candidate built from delta_fwd's own output plus a KNOWN perturbation, the sums are the
    perturbation's (numpy), per head and per token; a candidate equal to the reference gives
    zeros; a perturbation of one element of one token shows up in that token and head alone."""
    rng = np.random.default_rng(5)
    N, L, R, dk, dv = 3, 41, 2, 12, 20
    Q = rng.standard_normal((N, L, dk)).astype(np.float32)
    K = (rng.standard_normal((N, L, R, dk)) / 4).astype(np.float32)
    V = rng.standard_normal((N, L, R, dv)).astype(np.float32)
    b = rng.random((N, L, R)).astype(np.float32)
    S0 = rng.standard_normal((N, dv, dk)).astype(np.float32)
    O, SL = oracle.delta_fwd(Q, K, V, b, S0)
    O32, S32 = O.astype(np.float32), SL.astype(np.float32)

    c = oracle.delta_compare(Q, K, V, b, S0, O32, S32)
    rounding = (O32.astype(np.float64) - O) ** 2
    assert np.allclose(c["err2"], rounding.sum(-1), rtol=1e-9, atol=0)
    assert np.allclose(c["ref2"], (O * O).sum(-1), rtol=1e-12)
    assert c["err2"].max() < 1e-10 * c["ref2"].max()

    pert = rng.standard_normal(O.shape) * 1e-2
    Oc = (O + pert).astype(np.float32)
    Sc = (SL * 1.01).astype(np.float32)
    c = oracle.delta_compare(Q, K, V, b, S0, Oc, Sc)
    d = Oc.astype(np.float64) - O
    assert np.allclose(c["err2"], (d * d).sum(-1), rtol=1e-9)
    assert np.allclose(c["maxabs"], np.abs(d).max(axis=(1, 2)), rtol=1e-12)
    assert np.allclose(c["s_err2"], ((Sc.astype(np.float64) - SL) ** 2).sum(axis=(1, 2)), rtol=1e-9)
    assert np.allclose(c["s_ref2"], (SL * SL).sum(axis=(1, 2)), rtol=1e-12)

    Oc = O32.copy()
    Oc[1, 17, 3] += 0.5
    c = oracle.delta_compare(Q, K, V, b, None if S0 is None else S0, Oc)
    hot = np.zeros((N, L), dtype=bool)
    hot[1, 17] = True
    assert abs(c["err2"][1, 17] - 0.25) < 1e-3 and c["err2"][~hot].max() < 1e-9
    assert abs(c["maxabs"][1] - 0.5) < 1e-3 and c["maxabs"][0] < 1e-4 and c["s_err2"] is None
