"""Pins for the oracle's attention rollout (Eq. 6 - Eq. 9)."""
import numpy as np
import pytest

from oracle import d2cache_oracle as O
from paper_2509_23094_amd import workloads as W


def _random_abars(seed, n_layers, m, L):
    out = []
    for l in range(n_layers):
        a = np.exp(W.logits_rows(seed, m, L, std=1.5, extra=l).astype(np.float64))
        out.append(a / a.sum(axis=1, keepdims=True))
    return out


def test_expand_rows():
    L, S = 7, np.array([1, 4, 5])
    ab = _random_abars(0, 1, 3, L)[0]
    E = O.expand_attention(ab, S, L)
    for i in range(L):
        if i in S:
            np.testing.assert_array_equal(E[i], ab[list(S).index(i)])
        else:
            assert E[i, i] == 1.0 and E[i].sum() == 1.0


def test_transition_and_rollout_are_row_stochastic():
    L, S = 24, W.distinct_sorted_rows(1, 24, 9)
    abars = _random_abars(1, 4, len(S), L)
    Wm = O.transition(O.expand_attention(abars[0], S, L))
    np.testing.assert_allclose(Wm.sum(axis=1), 1.0, atol=1e-14)
    C = O.rollout(abars, S, L)
    np.testing.assert_allclose(C.sum(axis=1), 1.0, atol=1e-13)
    assert abs(O.influence(C).sum() - L) < 1e-11
    assert np.all(C >= 0)
    for i in range(L):                                   # rows outside S never move
        if i not in S:
            e = np.zeros(L); e[i] = 1.0
            np.testing.assert_array_equal(C[i], e)


def test_rollout_empty_selection():
    C = O.rollout([np.zeros((0, 11))] * 3, np.zeros(0, np.int64), 11)
    np.testing.assert_array_equal(C, np.eye(11))
    np.testing.assert_array_equal(O.influence(C), np.ones(11))


def test_rollout_all_rows_is_textbook_rollout():
    # with every row selected, Eq. 6-8 reduce to the product of 0.5 (A + I)
    L, N = 13, 5
    S = np.arange(L)
    abars = _random_abars(2, N, L, L)
    ref = np.eye(L)
    for a in abars:
        ref = 0.5 * (a + np.eye(L)) @ ref
    np.testing.assert_allclose(O.rollout(abars, S, L), ref, atol=1e-14)


def test_rollout_uniform_attention_closed_form():
    # A = J/L in every layer  =>  C = J/L + 2^-N (I - J/L), so c_j = 1
    L, N = 10, 6
    J = np.full((L, L), 1.0 / L)
    C = O.rollout([J] * N, np.arange(L), L)
    np.testing.assert_allclose(C, J + 2.0 ** (-N) * (np.eye(L) - J), atol=1e-15)
    np.testing.assert_allclose(O.influence(C), 1.0, atol=1e-14)


def test_rollout_single_layer_values():
    # one layer: C = W, so c_j = [j not in S] + sum_{i in S} (A_ij + [i = j]) / 2
    L, S = 9, np.array([0, 3, 8])
    ab = _random_abars(3, 1, 3, L)[0]
    c = O.influence(O.rollout([ab], S, L))
    for j in range(L):
        ref = (0.0 if j in S else 1.0) + sum(0.5 * (ab[r, j] + (1.0 if S[r] == j else 0.0)) for r in range(3))
        assert abs(c[j] - ref) < 1e-14


@pytest.mark.parametrize("seed", range(3))
def test_rollout_brute_force_loops(seed):
    L, N = 6, 2
    S = W.distinct_sorted_rows(seed, L, 3)
    abars = _random_abars(seed + 20, N, 3, L)
    C = [[1.0 if i == j else 0.0 for j in range(L)] for i in range(L)]
    for a in abars:
        Wm = [[0.0] * L for _ in range(L)]
        for i in range(L):
            row = [0.0] * L
            if i in S:
                r = list(S).index(i)
                for j in range(L):
                    row[j] = a[r][j]
            else:
                row[i] = 1.0
            row[i] += 1.0
            tot = sum(row)
            Wm[i] = [v / tot for v in row]
        C = [[sum(Wm[i][t] * C[t][j] for t in range(L)) for j in range(L)] for i in range(L)]
    np.testing.assert_allclose(O.rollout(abars, S, L), np.array(C), atol=1e-14)


@pytest.mark.parametrize("seed", range(3))
def test_rollout_compact_block_identity(seed):
    # Rows outside S stay one-hot, so only the |S| x L block moves:
    #   C_S <- (A[:, S] C_S + A[:, not S] scattered + C_S) / 2,  c_j = [j not in S] + colsum(C_S)
    L, N, m = 40, 4, 11
    S = W.distinct_sorted_rows(seed, L, m)
    abars = _random_abars(seed + 30, N, m, L)
    CS = np.zeros((m, L)); CS[np.arange(m), S] = 1.0
    notS = np.ones(L, bool); notS[S] = False
    for a in abars:
        CS = 0.5 * (a[:, S] @ CS + a * notS[None, :] + CS)
    C = O.rollout(abars, S, L)
    np.testing.assert_allclose(C[S], CS, atol=1e-14)
    np.testing.assert_allclose(O.influence(C), notS.astype(float) + CS.sum(axis=0), atol=1e-13)
