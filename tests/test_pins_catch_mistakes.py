"""The pins of tests/test_oracle_pins.py are meant to fail for every plausible mistake in an
implementation of the recurrence.  This file plants such mistakes, one at a time, in a small
numpy stand-in that offers the oracle's two entry points, runs the pins on it, and checks that
each mistake is caught by at least one pin (and that the stand-in without a mistake passes all
of them).  The planted mistakes live here, on the CPU; nothing of this touches oracle/ or the
GPU path.
"""
import numpy as np
import pytest

import test_oracle_pins as pins


class StandIn:
    """Token-by-token recurrence of Section 3.1 (general drivers A, Atil, B; readout of
    Section 1.1) with one optional planted mistake."""

    def __init__(self, mistake=None):
        self.mistake = mistake

    def flow_head(self, A, Atil, Bm, Q, S0=None, want_O=True):
        m = self.mistake
        A, Atil, Bm, Q = (np.asarray(x, dtype=np.float64) for x in (A, Atil, Bm, Q))
        L, R, dk = A.shape
        dv = Atil.shape[2]
        S = np.zeros((dv, dk)) if (S0 is None or m == "ignores_initial_state") else np.array(S0, dtype=np.float64)
        O = np.zeros((L, dv))
        for t in range(L):
            if m == "readout_before_update":
                O[t] = S @ Q[t]
            tb = t - 1 if (m == "b_of_previous_token" and t > 0) else t
            if m == "columns_see_each_other":        # product of r rank-1 factors instead of one rank-r increment
                for j in range(R):
                    S = S + np.outer(S @ A[t, j], Bm[tb, j]) + np.outer(Atil[t, j], Bm[tb, j])
            else:
                SA = S @ A[t].T                       # [dv, R]: every column sees the old state
                if m == "transition_dropped":
                    SA = 0 * SA
                if m == "transition_sign":
                    SA = -SA
                inp = Atil[t].T                       # [dv, R]
                if m == "input_sign":
                    inp = -inp
                if m == "only_first_column":
                    SA, inp = SA[:, :1], inp[:, :1]
                    S = S + (SA + inp) @ Bm[tb, :1]
                elif m == "a_and_b_swapped":
                    S = S + (S @ Bm[tb].T) @ A[t] + inp @ Bm[tb]
                else:
                    S = S + (SA + inp) @ Bm[tb]
            if m != "readout_before_update":
                O[t] = (S.T @ Q[t][:dv] if m == "readout_with_transposed_state" and dv == dk else S @ Q[t])
        return (O if want_O else None), S

    def delta_fwd(self, Q, K, V, beta, S0=None, want_O=True, nthreads=0):
        m = self.mistake
        K = np.asarray(K, dtype=np.float32).astype(np.float64)
        V = np.asarray(V, dtype=np.float32).astype(np.float64)
        Q = np.asarray(Q, dtype=np.float32).astype(np.float64)
        beta = np.asarray(beta, dtype=np.float32).astype(np.float64)
        lead = K.shape[:-3]
        L, R, dk = K.shape[-3:]
        dv = V.shape[-1]
        N = int(np.prod(lead)) if lead else 1
        Kf, Vf, Qf, bf = K.reshape(N, L, R, dk), V.reshape(N, L, R, dv), Q.reshape(N, L, dk), beta.reshape(N, L, R)
        S0f = None if S0 is None else np.asarray(S0, dtype=np.float32).astype(np.float64).reshape(N, dv, dk)
        O = np.zeros((N, L, dv))
        SL = np.zeros((N, dv, dk))
        for h in range(N):
            bk = bf[h][..., None]
            A = bk * Kf[h]
            At = -(Vf[h] if m == "beta_missing_on_values" else bk * Vf[h])
            o, s = self.flow_head(A, At, -Kf[h], Qf[h], None if S0f is None else S0f[h])
            O[h], SL[h] = o, s
        return (O.reshape(lead + (L, dv)) if want_O else None), SL.reshape(lead + (dv, dk))


def _pin_calls():
    """Every pin of test_oracle_pins.py that exercises the recurrence, with its parameters."""
    calls = []
    for case in ("rank1", "rank2_sum_not_product", "rank2_orthonormal_overwrite"):
        calls.append((pins.test_hand_worked_examples, dict(case=case)))
    for seed in (0, 1):
        calls.append((pins.test_identity_transition_is_causal_linear_attention, dict(seed=seed)))
    calls.append((pins.test_beta_zero_leaves_state_unchanged, {}))
    calls.append((pins.test_unit_key_beta_one_projects_and_writes_value, {}))
    calls.append((pins.test_unit_key_beta_two_is_an_involution, {}))
    for r in (1, 3):
        calls.append((pins.test_matches_literal_equation_in_numpy, dict(r=r)))
    calls.append((pins.test_rank_r_with_one_active_column_equals_rank_one, {}))
    for r in (1, 2, 4):
        calls.append((pins.test_chunked_flow_equals_sequential_for_every_chunk_size, dict(L=12, r=r)))
    calls.append((pins.test_chunked_flow_general_drivers, {}))
    calls.append((pins.test_flow_propagator_is_ordered_product, {}))
    calls.append((pins.test_orthonormal_keys_closed_form, {}))
    calls.append((pins.test_linearity_in_values_and_initial_state, {}))
    calls.append((pins.test_split_sequence_composes_through_the_state, {}))
    calls.append((pins.test_state_formula_needs_the_transpose, {}))
    return calls


def _failing_pins(impl):
    failed = []
    for fn, kw in _pin_calls():
        try:
            fn(impl, **kw)
        except AssertionError:
            failed.append(fn.__name__ + (str(kw) if kw else ""))
    return failed


def test_stand_in_without_a_mistake_passes_every_pin():
    assert _failing_pins(StandIn(None)) == []


MISTAKES = [
    "readout_before_update",          # o_t = S_{t-1} q_t
    "columns_see_each_other",         # product form instead of the additive rank-r increment
    "transition_dropped",             # S_t = S_{t-1} + Atil B^T (plain linear attention)
    "transition_sign",                # S_{t-1}(I + beta k k^T)
    "input_sign",                     # - beta v k^T
    "only_first_column",              # r > 1 silently truncated to rank 1
    "a_and_b_swapped",                # S B A^T instead of S A B^T
    "b_of_previous_token",            # off-by-one in time on B
    "ignores_initial_state",          # S_0 dropped
    "readout_with_transposed_state",  # o = S^T q (only expressible for d_v = d_k)
    "beta_missing_on_values",         # delta mapping: Atil = -v instead of -beta v
]


@pytest.mark.parametrize("mistake", MISTAKES)
def test_every_planted_mistake_is_caught(mistake):
    failed = _failing_pins(StandIn(mistake))
    print(f"[mutant] {mistake}: caught by {len(failed)} pin(s): {failed[:4]}")
    assert failed, f"no pin notices the mistake '{mistake}'"
