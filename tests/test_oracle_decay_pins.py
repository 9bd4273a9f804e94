"""Pins for the oracle's scalar-decay functions (mask entries lam^(i-j)); no GPU needed.  The
paper gives no formulas for the decayed variants it evaluates, so the decayed definition is the
reference; it is tied to a hand-worked example, to geometric-series closed forms, to the plain
(already pinned) oracle at lam = 1 and through the rescaling identity, to finite differences,
and the recurrence and the chunked steps derived from it must reproduce it for any partition."""
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
    g = json.load(open(os.path.join(GOLD, "decay_hand_example.json")))
    Q, K, V, dO = (np.array(g[k], dtype=np.float64)[None] for k in ("Q", "K", "V", "dO"))
    want = {k: np.array(g[k], dtype=np.float64)[None] for k in ("O", "dQ", "dK", "dV")}
    lam = g["lam"]
    assert np.array_equal(oracle.fwd_def_decay(Q, K, V, lam), want["O"])
    assert np.array_equal(oracle.fwd_rec_decay(Q, K, V, lam), want["O"])
    for fam in (oracle.bwd_def_decay, oracle.bwd_rec_decay):
        for got, key in zip(fam(Q, K, V, dO, lam), ("dQ", "dK", "dV")):
            assert np.array_equal(got, want[key]), (fam.__name__, key)
    for bounds in ([0, 3], [0, 1, 3], [0, 2, 3], [0, 1, 2, 3]):
        assert np.array_equal(oracle.forward_by_algorithm_decay(Q, K, V, bounds, lam)[0], want["O"])
        got = oracle.backward_by_algorithm_decay(Q, K, V, dO, bounds, lam)[:3]
        for x, key in zip(got, ("dQ", "dK", "dV")):
            assert np.array_equal(x, want[key]), (bounds, key)


def test_geometric_series_closed_form(oracle):
    """All-ones inputs: every score is d, so o_i = d (1 - lam^(i+1)) / (1 - lam) in every column."""
    N, d = 40, 4
    ones = np.ones((2, N, d))
    lam = np.array([0.5, 0.9])
    O = oracle.fwd_def_decay(ones, ones, ones, lam)
    i = np.arange(N)
    for g in range(2):
        want = d * (1 - lam[g] ** (i + 1)) / (1 - lam[g])
        assert np.allclose(O[g], want[:, None], rtol=1e-13)


def test_lam_one_is_the_plain_oracle(oracle):
    Q, K, V, dO = _rand(2, 45, 8, 31)
    cu = [0, 9, 30, 45]
    assert _rel(oracle.fwd_def_decay(Q, K, V, 1.0, cu), oracle.fwd_def(Q, K, V, cu)) < 1e-14
    for a, b in zip(oracle.bwd_def_decay(Q, K, V, dO, 1.0, cu), oracle.bwd_def(Q, K, V, dO, cu)):
        assert _rel(a, b) < 1e-14
    bounds, first = slot_partition(45, 8, cu)
    M = oracle.chunk_states_decay(K, V, bounds, 1.0)
    assert _rel(M, oracle.chunk_states(K, V, bounds)) < 1e-14
    assert _rel(oracle.state_prefix_decay(M, bounds, 1.0, first), oracle.state_prefix(M, first)) < 1e-14
    assert _rel(oracle.state_prefix_decay(M, bounds, 1.0, first, reverse=True),
                oracle.state_prefix(M, first, reverse=True)) < 1e-14


def test_rescaling_identity_ties_decay_to_the_plain_definition(oracle):
    """lam^(i-j) (q_i.k_j) = (lam^i q_i).(lam^-j k_j): the decayed output is the plain (pinned)
    definition on rescaled queries and keys.  Short sequence so that lam^-j stays tame."""
    Q, K, V, _ = _rand(2, 24, 4, 32)
    lam = np.array([0.8, 0.95])
    pos = np.arange(24)
    Qs = Q * (lam[:, None] ** pos)[..., None]
    Ks = K * (lam[:, None] ** -pos)[..., None]
    assert _rel(oracle.fwd_def_decay(Q, K, V, lam), oracle.fwd_def(Qs, Ks, V)) < 1e-12


@pytest.mark.parametrize("bounds", [[0, 70], [0, 16, 32, 48, 64, 70], [0, 5, 6, 40, 70], [0, 0, 70, 70]])
def test_three_families_agree(oracle, bounds):
    Q, K, V, dO = _rand(3, 70, 8, 33)
    lam = np.array([0.5, 0.97, 1.0])
    O = oracle.fwd_def_decay(Q, K, V, lam)
    assert _rel(oracle.fwd_rec_decay(Q, K, V, lam), O) < 1e-13
    assert _rel(oracle.forward_by_algorithm_decay(Q, K, V, bounds, lam)[0], O) < 1e-13
    ref = oracle.bwd_def_decay(Q, K, V, dO, lam)
    for fam in (oracle.bwd_rec_decay(Q, K, V, dO, lam), oracle.backward_by_algorithm_decay(Q, K, V, dO, bounds, lam)[:3]):
        for a, b in zip(fam, ref):
            assert _rel(a, b) < 1e-13


def test_packed_documents(oracle):
    cu = [0, 7, 8, 40, 61]
    Q, K, V, dO = _rand(2, 61, 8, 34)
    lam = np.array([0.9, 0.6])
    O = oracle.fwd_def_decay(Q, K, V, lam, cu)
    grads = oracle.bwd_def_decay(Q, K, V, dO, lam, cu)
    for a, b in zip(cu[:-1], cu[1:]):
        sl = slice(a, b)
        assert _rel(O[:, sl], oracle.fwd_def_decay(Q[:, sl], K[:, sl], V[:, sl], lam)) < 1e-13
    assert _rel(oracle.fwd_rec_decay(Q, K, V, lam, cu), O) < 1e-13
    for x, y in zip(oracle.bwd_rec_decay(Q, K, V, dO, lam, cu), grads):
        assert _rel(x, y) < 1e-13
    bounds, first = slot_partition(61, 16, cu)
    assert _rel(oracle.forward_by_algorithm_decay(Q, K, V, bounds, lam, first)[0], O) < 1e-13
    for x, y in zip(oracle.backward_by_algorithm_decay(Q, K, V, dO, bounds, lam, first)[:3], grads):
        assert _rel(x, y) < 1e-13


def test_state_values(oracle):
    """Anchors and the decayed combine on a tiny case written out term by term."""
    rng = np.random.default_rng(35)
    K = rng.standard_normal((1, 5, 2)); V = rng.standard_normal((1, 5, 2))
    lam, bounds = 0.5, [0, 2, 5]
    outer = lambda j: np.outer(K[0, j], V[0, j])
    M = oracle.chunk_states_decay(K, V, bounds, lam)[0]
    assert np.allclose(M[0], 0.5 * outer(0) + outer(1))
    assert np.allclose(M[1], 0.25 * outer(2) + 0.5 * outer(3) + outer(4))
    Ms = oracle.chunk_states_decay(K, V, bounds, lam, anchor_start=True)[0]
    assert np.allclose(Ms[0], outer(0) + 0.5 * outer(1))
    assert np.allclose(Ms[1], outer(2) + 0.5 * outer(3) + 0.25 * outer(4))
    P = oracle.state_prefix_decay(M[None], bounds, lam)[0]
    assert np.allclose(P[0], 0) and np.allclose(P[1], M[0])
    R = oracle.state_prefix_decay(Ms[None], bounds, lam, reverse=True)[0]
    assert np.allclose(R[1], 0) and np.allclose(R[0], Ms[1])
    # three chunks: the middle chunk's length weights the carried state
    b3 = [0, 1, 3, 5]
    M3 = oracle.chunk_states_decay(K, V, b3, lam)[0]
    P3 = oracle.state_prefix_decay(M3[None], b3, lam)[0]
    assert np.allclose(P3[2], 0.25 * M3[0] + M3[1])


def test_gradient_by_finite_differences(oracle):
    Q, K, V, dO = _rand(1, 9, 3, 36)
    lam = 0.7
    dQ, dK, dV = oracle.bwd_def_decay(Q, K, V, dO, lam)
    loss = lambda q, k, v: float(np.sum(dO * oracle.fwd_def_decay(q, k, v, lam)))
    eps = 1e-6
    rng = np.random.default_rng(37)
    for name, X, dX in (("Q", Q, dQ), ("K", K, dK), ("V", V, dV)):
        for _ in range(6):
            i, a = int(rng.integers(9)), int(rng.integers(3))
            Xp, Xm = X.copy(), X.copy()
            Xp[0, i, a] += eps
            Xm[0, i, a] -= eps
            ap = {"Q": (Xp, K, V), "K": (Q, Xp, V), "V": (Q, K, Xp)}[name]
            am = {"Q": (Xm, K, V), "K": (Q, Xm, V), "V": (Q, K, Xm)}[name]
            fd = (loss(*ap) - loss(*am)) / (2 * eps)
            assert abs(fd - dX[0, i, a]) <= 1e-6 * max(1.0, abs(fd)), (name, i, a)


def test_row_sampler_matches_full_definition(oracle):
    cu = [0, 7, 8, 40, 61]
    Q, K, V, dO = _rand(1, 61, 8, 38)
    lam = 0.8
    full = (oracle.fwd_def_decay(Q, K, V, lam, cu),) + oracle.bwd_def_decay(Q, K, V, dO, lam, cu)
    rows = np.array([60, 0, 7, 8, 39, 40, 6])
    for which in range(4):
        got = oracle.def_rows_decay(Q[0], K[0], V[0], dO[0], rows, which, lam, cu)
        assert _rel(got, full[which][0][rows]) < 1e-13
    g = json.load(open(os.path.join(GOLD, "decay_hand_example.json")))
    A = {k: np.array(g[k], dtype=np.float64) for k in ("Q", "K", "V", "dO", "O", "dQ", "dK", "dV")}
    for which, key in enumerate(("O", "dQ", "dK", "dV")):
        got = oracle.def_rows_decay(A["Q"], A["K"], A["V"], A["dO"], np.array([2, 0, 1]), which, g["lam"])
        assert np.array_equal(got, A[key][[2, 0, 1]])
