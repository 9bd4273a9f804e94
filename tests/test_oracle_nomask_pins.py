"""Pins for the oracle's unmasked functions (Algorithm "LASP-2 w/o Masking" and its backward
pass); no GPU needed.  They are checked against a hand-worked integer example, numpy matmuls
(without the mask the whole computation is two library products), the masked oracle through
the identity full = causal + anti-causal - diagonal, finite differences, and the invariance
under a joint permutation of keys and values that only an unmasked product has."""
import json
import os

import numpy as np
import pytest

from tests.util import slot_partition

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rand(G, N, d, seed):
    rng = np.random.default_rng(seed)
    return [rng.standard_normal((G, N, d)) for _ in range(4)]


def _rel(a, b):
    return np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300)


def test_hand_example(oracle):
    g = json.load(open(os.path.join(GOLD, "nomask_hand_example.json")))
    Q, K, V, dO = (np.array(g[k], dtype=np.float64)[None] for k in ("Q", "K", "V", "dO"))
    want = {k: np.array(g[k], dtype=np.float64)[None] for k in ("O", "dQ", "dK", "dV")}
    assert np.array_equal(oracle.nomask_fwd_def(Q, K, V), want["O"])
    for got, key in zip(oracle.nomask_bwd_def(Q, K, V, dO), ("dQ", "dK", "dV")):
        assert np.array_equal(got, want[key]), key
    for bounds in ([0, 3], [0, 1, 3], [0, 2, 3], [0, 1, 2, 3]):
        O, M, S = oracle.nomask_forward_by_algorithm(Q, K, V, bounds)
        assert np.array_equal(O, want["O"])
        for t in range(len(bounds) - 1):     # every chunk holds the same total
            assert np.array_equal(S[0, t], np.array(g["M"], dtype=np.float64))
        dQ, dK, dV, dS = oracle.nomask_backward_by_algorithm(Q, K, V, dO, bounds)
        assert np.array_equal(dS[0, 0], np.array(g["dM"], dtype=np.float64))
        assert np.array_equal(dQ, want["dQ"])
        assert np.array_equal(dK, want["dK"])
        assert np.array_equal(dV, want["dV"])


@pytest.mark.parametrize("N,d", [(1, 4), (37, 8), (130, 16)])
def test_definition_is_two_matmuls(oracle, N, d):
    """Without the mask, O = Q (K^T V) and the gradients are plain products too."""
    Q, K, V, dO = _rand(3, N, d, 11)
    O = oracle.nomask_fwd_def(Q, K, V)
    dQ, dK, dV = oracle.nomask_bwd_def(Q, K, V, dO)
    for g in range(3):
        M = K[g].T @ V[g]
        dM = Q[g].T @ dO[g]
        assert _rel(O[g], Q[g] @ M) < 1e-13
        assert _rel(dQ[g], dO[g] @ M.T) < 1e-13
        assert _rel(dK[g], V[g] @ dM.T) < 1e-13
        assert _rel(dV[g], K[g] @ dM) < 1e-13


def test_full_equals_causal_plus_anticausal_minus_diagonal(oracle):
    """Ties the unmasked definition to the masked one (Eq. (3)), which has its own pins:
    sum over all j = sum_{j<=i} + sum_{j>=i} - (j = i); the anti-causal sum is the causal one
    on the reversed sequence."""
    Q, K, V, _ = _rand(2, 53, 8, 12)
    causal = oracle.fwd_def(Q, K, V)
    anti = oracle.fwd_def(Q[:, ::-1], K[:, ::-1], V[:, ::-1])[:, ::-1]
    diag = np.einsum("gnd,gnd->gn", Q, K)[..., None] * V
    assert _rel(oracle.nomask_fwd_def(Q, K, V), causal + anti - diag) < 1e-13


@pytest.mark.parametrize("bounds", [[0, 64], [0, 16, 32, 48, 64], [0, 5, 6, 40, 64], [0, 0, 64, 64]])
def test_algorithm_matches_definition(oracle, bounds):
    Q, K, V, dO = _rand(2, 64, 8, 13)
    O, _, _ = oracle.nomask_forward_by_algorithm(Q, K, V, bounds)
    assert _rel(O, oracle.nomask_fwd_def(Q, K, V)) < 1e-13
    got = oracle.nomask_backward_by_algorithm(Q, K, V, dO, bounds)[:3]
    for a, b in zip(got, oracle.nomask_bwd_def(Q, K, V, dO)):
        assert _rel(a, b) < 1e-13


def test_documents_do_not_mix(oracle):
    """Packed documents: each document equals the same computation on it alone."""
    cu = [0, 7, 8, 40, 61]
    Q, K, V, dO = _rand(2, 61, 8, 14)
    O = oracle.nomask_fwd_def(Q, K, V, cu)
    grads = oracle.nomask_bwd_def(Q, K, V, dO, cu)
    for a, b in zip(cu[:-1], cu[1:]):
        sl = slice(a, b)
        assert _rel(O[:, sl], oracle.nomask_fwd_def(Q[:, sl], K[:, sl], V[:, sl])) < 1e-13
        alone = oracle.nomask_bwd_def(Q[:, sl], K[:, sl], V[:, sl], dO[:, sl])
        for x, y in zip(grads, alone):
            assert _rel(x[:, sl], y) < 1e-13
    # the algorithm over slots of 16 tokens per document, totals restarted per document
    bounds, first = slot_partition(61, 16, cu)
    Oa, _, S = oracle.nomask_forward_by_algorithm(Q, K, V, bounds, first)
    assert _rel(Oa, O) < 1e-13
    t = int(np.searchsorted(bounds, 8))     # first slot of the third document
    assert _rel(S[0, t], K[0, 8:40].T @ V[0, 8:40]) < 1e-13
    got = oracle.nomask_backward_by_algorithm(Q, K, V, dO, bounds, first)[:3]
    for x, y in zip(got, grads):
        assert _rel(x, y) < 1e-13


def test_state_total_values(oracle):
    rng = np.random.default_rng(15)
    M = rng.standard_normal((2, 5, 3, 3))
    S = oracle.state_total(M)
    for t in range(5):
        assert _rel(S[:, t], M.sum(axis=1)) < 1e-14
    first = np.array([1, 0, 1, 1, 0], dtype=np.int32)
    S = oracle.state_total(M, first)
    assert _rel(S[:, 0], M[:, 0] + M[:, 1]) < 1e-14 and np.array_equal(S[:, 0], S[:, 1])
    assert np.array_equal(S[:, 2], M[:, 2])
    assert _rel(S[:, 3], M[:, 3] + M[:, 4]) < 1e-14 and np.array_equal(S[:, 3], S[:, 4])


def test_rows_times_state_transpose(oracle):
    rng = np.random.default_rng(16)
    A = rng.standard_normal((1, 6, 3))
    S = rng.standard_normal((1, 2, 3, 3))
    bounds = [0, 2, 6]
    out = oracle.rows_times_state(A, S, bounds)
    outT = oracle.rows_times_state(A, S, bounds, transpose=True)
    assert _rel(out[0, :2], A[0, :2] @ S[0, 0]) < 1e-14 and _rel(out[0, 2:], A[0, 2:] @ S[0, 1]) < 1e-14
    assert _rel(outT[0, :2], A[0, :2] @ S[0, 0].T) < 1e-14 and _rel(outT[0, 2:], A[0, 2:] @ S[0, 1].T) < 1e-14


def test_gradient_by_finite_differences(oracle):
    Q, K, V, dO = _rand(1, 9, 3, 17)
    dQ, dK, dV = oracle.nomask_bwd_def(Q, K, V, dO)
    loss = lambda q, k, v: float(np.sum(dO * oracle.nomask_fwd_def(q, k, v)))
    eps = 1e-6
    rng = np.random.default_rng(18)
    for name, X, dX in (("Q", Q, dQ), ("K", K, dK), ("V", V, dV)):
        for _ in range(6):
            i, a = int(rng.integers(9)), int(rng.integers(3))
            Xp, Xm = X.copy(), X.copy()
            Xp[0, i, a] += eps
            Xm[0, i, a] -= eps
            args_p = {"Q": (Xp, K, V), "K": (Q, Xp, V), "V": (Q, K, Xp)}[name]
            args_m = {"Q": (Xm, K, V), "K": (Q, Xm, V), "V": (Q, K, Xm)}[name]
            fd = (loss(*args_p) - loss(*args_m)) / (2 * eps)
            assert abs(fd - dX[0, i, a]) <= 1e-6 * max(1.0, abs(fd)), (name, i, a)


def test_invariant_under_joint_permutation_of_keys_and_values(oracle):
    """Only an unmasked product ignores the order of the (k_j, v_j) pairs; the masked one must not."""
    Q, K, V, _ = _rand(1, 31, 4, 19)
    perm = np.random.default_rng(20).permutation(31)
    full = oracle.nomask_fwd_def(Q, K, V)
    assert _rel(oracle.nomask_fwd_def(Q, K[:, perm], V[:, perm]), full) < 1e-13
    assert _rel(oracle.fwd_def(Q, K[:, perm], V[:, perm]), oracle.fwd_def(Q, K, V)) > 1e-3


def test_row_sampler_matches_full_definition(oracle):
    cu = [0, 7, 8, 40, 61]
    Q, K, V, dO = _rand(1, 61, 8, 21)
    full = (oracle.nomask_fwd_def(Q, K, V, cu),) + oracle.nomask_bwd_def(Q, K, V, dO, cu)
    rows = np.array([60, 0, 7, 8, 39, 40, 6])
    for which in range(4):
        got = oracle.nomask_def_rows(Q[0], K[0], V[0], dO[0], rows, which, cu)
        assert _rel(got, full[which][0][rows]) < 1e-13
    g = json.load(open(os.path.join(GOLD, "nomask_hand_example.json")))
    A = {k: np.array(g[k], dtype=np.float64) for k in g if not k.startswith("_")}
    for which, key in enumerate(("O", "dQ", "dK", "dV")):
        got = oracle.nomask_def_rows(A["Q"], A["K"], A["V"], A["dO"], np.array([2, 0, 1]), which)
        assert np.array_equal(got, A[key][[2, 0, 1]])
