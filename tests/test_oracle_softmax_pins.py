"""Pins for the oracle's softmax attention (compute line of Algorithm "AllGather-based Context
Parallelism"); no GPU needed: scipy's softmax as the library special case, closed forms (uniform
scores give means, a dominant key is copied), invariances of the softmax, finite differences for
the gradient, documents that do not mix, and an example whose exponentials are powers of two."""
import numpy as np
import pytest
from scipy.special import logsumexp, softmax


def _rand(G, N, d, seed):
    rng = np.random.default_rng(seed)
    return [rng.standard_normal((G, N, d)) for _ in range(4)]


def _rel(a, b):
    return np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300)


@pytest.mark.parametrize("causal", [False, True])
def test_matches_scipy_softmax(oracle, causal):
    Q, K, V, _ = _rand(3, 41, 8, 51)
    O, lse = oracle.softmax_fwd(Q, K, V, causal)
    for g in range(3):
        S = Q[g] @ K[g].T / np.sqrt(8)
        if causal:
            S = np.where(np.tril(np.ones((41, 41), bool)), S, -np.inf)
        assert _rel(O[g], softmax(S, axis=1) @ V[g]) < 1e-13
        assert np.allclose(lse[g], logsumexp(S, axis=1), rtol=1e-13, atol=1e-13)


def test_powers_of_two_example(oracle):
    """d = 1, q = 1, keys k_j = j ln 2, values v_j = j: scores j ln 2, so P_ij = 2^j / sum 2^j
    and, causally, o_i = sum_{j<=i} j 2^j / (2^(i+1) - 1) = ((i - 1) 2^(i+1) + 2) / (2^(i+1) - 1)."""
    N = 6
    Q = np.ones((1, N, 1)); K = (np.arange(N) * np.log(2.0)).reshape(1, N, 1); V = np.arange(N, dtype=float).reshape(1, N, 1)
    O, lse = oracle.softmax_fwd(Q, K, V, causal=True)
    i = np.arange(N)
    want = ((i - 1) * 2.0 ** (i + 1) + 2) / (2.0 ** (i + 1) - 1)
    assert np.allclose(O[0, :, 0], want, rtol=1e-14)
    assert np.allclose(lse[0], np.log(2.0 ** (i + 1) - 1), rtol=1e-14)
    full, _ = oracle.softmax_fwd(Q, K, V, causal=False)
    assert np.allclose(full[0, :, 0], ((N - 2) * 2.0 ** N + 2) / (2.0 ** N - 1), rtol=1e-14)


def test_uniform_scores_give_means(oracle):
    Q, _, V, _ = _rand(2, 30, 4, 52)
    K = np.zeros_like(Q)
    O, lse = oracle.softmax_fwd(Q, K, V, causal=True)
    want = np.cumsum(V, axis=1) / np.arange(1, 31)[None, :, None]
    assert _rel(O, want) < 1e-14 and np.allclose(lse, np.log(np.arange(1, 31))[None])
    O, _ = oracle.softmax_fwd(Q, K, V, causal=False)
    assert _rel(O, np.broadcast_to(V.mean(axis=1, keepdims=True), V.shape)) < 1e-14


def test_dominant_key_is_copied_and_rows_are_convex_combinations(oracle):
    Q, K, V, _ = _rand(1, 12, 4, 53)
    K2 = K.copy(); K2[0, 5] = 400.0 * Q[0, 9] / np.linalg.norm(Q[0, 9]) ** 2 * 2.0   # score (9,5) = 400
    O, _ = oracle.softmax_fwd(Q, K2, V, causal=False)
    assert np.allclose(O[0, 9], V[0, 5], atol=1e-12)
    ones = np.ones_like(V)
    O, _ = oracle.softmax_fwd(Q, K, ones, causal=True)
    assert np.allclose(O, 1.0, rtol=1e-14)


def test_invariances(oracle):
    Q, K, V, _ = _rand(2, 25, 6, 54)
    O, lse = oracle.softmax_fwd(Q, K, V, causal=False)
    perm = np.random.default_rng(55).permutation(25)
    assert _rel(oracle.softmax_fwd(Q, K[:, perm], V[:, perm])[0], O) < 1e-13           # order of the keys
    u = np.random.default_rng(56).standard_normal(6)
    Qorth = Q - (Q @ u)[..., None] * u / (u @ u)                                         # q . u = 0
    assert _rel(oracle.softmax_fwd(Qorth, K + 3.0 * u, V)[0], oracle.softmax_fwd(Qorth, K, V)[0]) < 1e-12
    assert _rel(oracle.softmax_fwd(Q, K, V, causal=True)[0][:, -1], O[:, -1]) < 1e-13   # last row sees everything


def test_documents_do_not_mix(oracle):
    cu = [0, 7, 8, 40, 61]
    Q, K, V, dO = _rand(2, 61, 8, 57)
    for causal in (False, True):
        O, lse = oracle.softmax_fwd(Q, K, V, causal, cu)
        grads = oracle.softmax_bwd(Q, K, V, dO, causal, cu)
        for a, b in zip(cu[:-1], cu[1:]):
            sl = slice(a, b)
            Oa, la = oracle.softmax_fwd(Q[:, sl], K[:, sl], V[:, sl], causal)
            assert _rel(O[:, sl], Oa) < 1e-13 and np.allclose(lse[:, sl], la)
            alone = oracle.softmax_bwd(Q[:, sl], K[:, sl], V[:, sl], dO[:, sl], causal)
            for x, y in zip(grads, alone):
                assert _rel(x[:, sl], y) < 1e-13
        rows = np.array([60, 0, 7, 8, 39, 40, 6])
        got, gl = oracle.softmax_rows(Q[1], K[1], V[1], rows, causal, cu)
        assert _rel(got, O[1][rows]) < 1e-14 and np.allclose(gl, lse[1][rows])


@pytest.mark.parametrize("causal", [False, True])
def test_gradient_by_finite_differences(oracle, causal):
    Q, K, V, dO = _rand(1, 9, 3, 58)
    dQ, dK, dV = oracle.softmax_bwd(Q, K, V, dO, causal)
    loss = lambda q, k, v: float(np.sum(dO * oracle.softmax_fwd(q, k, v, causal)[0]))
    eps = 1e-6
    rng = np.random.default_rng(59)
    for name, X, dX in (("Q", Q, dQ), ("K", K, dK), ("V", V, dV)):
        for _ in range(6):
            i, a = int(rng.integers(9)), int(rng.integers(3))
            Xp, Xm = X.copy(), X.copy()
            Xp[0, i, a] += eps
            Xm[0, i, a] -= eps
            ap = {"Q": (Xp, K, V), "K": (Q, Xp, V), "V": (Q, K, Xp)}[name]
            am = {"Q": (Xm, K, V), "K": (Q, Xm, V), "V": (Q, K, Xm)}[name]
            fd = (loss(*ap) - loss(*am)) / (2 * eps)
            assert abs(fd - dX[0, i, a]) <= 2e-6 * max(1.0, abs(fd)), (name, i, a)


def test_gradient_identities(oracle):
    """Rows of P sum to one, so shifting a query's scores changes nothing: sum_j dS_ij = 0, which
    makes dQ orthogonal to nothing in general but gives sum_j dK_j = scale * sum_i (sum_j dS_ij) q_i = 0
    when all queries are equal; and dV sums to the sum of dO."""
    Q, K, V, dO = _rand(1, 14, 4, 60)
    Qc = np.broadcast_to(Q[:, :1], Q.shape).copy()
    dQ, dK, dV = oracle.softmax_bwd(Qc, K, V, dO, causal=False)
    assert np.allclose(dK.sum(axis=1), 0.0, atol=1e-13)
    assert np.allclose(dV.sum(axis=1), dO.sum(axis=1), rtol=1e-13)


@pytest.mark.parametrize("causal", [False, True])
def test_gradient_rows_equal_the_full_gradient(oracle, causal):
    """The row-sampled form used at sizes where the full gradient is out of reach is the same
    definition: every row it returns equals that row of softmax_bwd (itself pinned above by
    finite differences), with and without documents."""
    for cu in (None, [0, 5, 6, 30, 47]):
        Q, K, V, dO = _rand(2, 47, 8, 61)
        O, lse = oracle.softmax_fwd(Q, K, V, causal, cu)
        full = oracle.softmax_bwd(Q, K, V, dO, causal, cu)
        rows = np.array([46, 0, 5, 6, 29, 30, 17, 4])
        for g in range(2):
            delta = np.sum(dO[g] * O[g], axis=1)
            for which in range(3):
                got = oracle.softmax_bwd_rows(Q[g], K[g], V[g], dO[g], lse[g], delta, rows, which, causal, cu)
                assert _rel(got, full[which][g][rows]) < 1e-12, (which, g)
