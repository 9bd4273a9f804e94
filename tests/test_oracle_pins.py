"""Pins for the CPU oracle: everything here runs without a GPU.

The oracle is checked against things other than itself: a hand-worked integer
example (tests/golden/hand_example.json), closed forms, identities that follow
from the mathematics (trilinearity, Euler), special cases that collapse to a
numpy matmul, and three separately written programs (definition, recurrence,
chunked algorithm) that must agree.
"""
import json
import os

import numpy as np
import pytest

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rand(G, N, d, seed):
    rng = np.random.default_rng(seed)
    return [rng.standard_normal((G, N, d)) for _ in range(4)]


def _rel(a, b):
    return np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300)


# ---------------------------------------------------------------- hand example
def test_hand_example_all_families(oracle):
    g = json.load(open(os.path.join(GOLD, "hand_example.json")))
    Q, K, V, dO = (np.array(g[k], dtype=np.float64)[None] for k in ("Q", "K", "V", "dO"))
    want = {k: np.array(g[k], dtype=np.float64)[None] for k in ("O", "dQ", "dK", "dV")}
    assert np.array_equal(oracle.fwd_def(Q, K, V), want["O"])
    assert np.array_equal(oracle.fwd_rec(Q, K, V), want["O"])
    for fam in (oracle.bwd_def, oracle.bwd_rec):
        dQ, dK, dV = fam(Q, K, V, dO)
        assert np.array_equal(dQ, want["dQ"])
        assert np.array_equal(dK, want["dK"])
        assert np.array_equal(dV, want["dV"])
    for bounds in ([0, 3], [0, 1, 3], [0, 2, 3], [0, 1, 2, 3]):
        O, M, P = oracle.forward_by_algorithm(Q, K, V, bounds)
        assert np.array_equal(O, want["O"])
        assert np.array_equal(M.sum(axis=1)[0], np.array(g["M_total"], dtype=np.float64))
        dQ, dK, dV, dM, dP = oracle.backward_by_algorithm(Q, K, V, dO, bounds)
        assert np.array_equal(dQ, want["dQ"])
        assert np.array_equal(dK, want["dK"])
        assert np.array_equal(dV, want["dV"])
    rows = np.array([2, 0, 1])
    for which, key in enumerate(("O", "dQ", "dK", "dV")):
        got = oracle.def_rows(Q[0], K[0], V[0], dO[0], rows, which)
        assert np.array_equal(got, want[key][0][rows])


def test_hand_example_chunk_state_values(oracle):
    """Per-chunk states and exclusive prefixes of the hand example, chunk = one token."""
    g = json.load(open(os.path.join(GOLD, "hand_example.json")))
    K = np.array(g["K"], dtype=np.float64)[None]
    V = np.array(g["V"], dtype=np.float64)[None]
    M = oracle.chunk_states(K, V, [0, 1, 2, 3])[0]
    assert np.array_equal(M[0], [[1, 0], [2, 0]])      # k1^T v1
    assert np.array_equal(M[1], [[0, 3], [0, 4]])      # k2^T v2
    assert np.array_equal(M[2], [[10, 15], [12, 18]])  # k3^T v3
    P = oracle.state_prefix(M[None])[0]
    assert np.array_equal(P[0], np.zeros((2, 2)))       # empty prefix is zero
    assert np.array_equal(P[1], [[1, 0], [2, 0]])
    assert np.array_equal(P[2], [[1, 3], [2, 4]])
    R = oracle.state_prefix(M[None], reverse=True)[0]
    assert np.array_equal(R[2], np.zeros((2, 2)))       # empty suffix is zero
    assert np.array_equal(R[1], [[10, 15], [12, 18]])
    assert np.array_equal(R[0], [[10, 18], [12, 22]])


# ---------------------------------------------------------------- closed forms
@pytest.mark.parametrize("N,d", [(1, 1), (5, 4), (17, 3)])
def test_closed_form_all_ones(oracle, N, d):
    """Q=K=V=1/sqrt(d): q.k = 1, so o_i = (i+1)/sqrt(d); with dO = 1: G_ij = sqrt(d),
    dQ_i = (i+1), dK_j = dV_j... = (N-j) entries (1-based counts), all columns equal."""
    c = 1.0 / np.sqrt(d)
    X = np.full((1, N, d), c)
    dO = np.ones((1, N, d))
    i = np.arange(N, dtype=np.float64)
    for fwd in (oracle.fwd_def, oracle.fwd_rec):
        O = fwd(X, X, X)
        assert np.allclose(O, ((i + 1) * c)[None, :, None], rtol=1e-13)
    for bwd in (oracle.bwd_def, oracle.bwd_rec):
        dQ, dK, dV = bwd(X, X, X, dO)
        # G_ij = sum_c 1*c = d*c = sqrt(d); dQ_i = sum_{j<=i} sqrt(d)*c = (i+1)
        assert np.allclose(dQ, (i + 1)[None, :, None], rtol=1e-13)
        assert np.allclose(dK, (N - i)[None, :, None], rtol=1e-13)
        # S_ij = 1; dV_j = sum_{i>=j} 1 * dO_i = (N-j)
        assert np.allclose(dV, (N - i)[None, :, None], rtol=1e-13)


def test_closed_form_one_hot_counts(oracle):
    """K = V = one-hot rows cycling with period d: the state is a diagonal count matrix and
    o_i[c] = q_i[c] * #{j <= i : j mod d == c}."""
    N, d = 11, 4
    E = np.eye(d)[np.arange(N) % d][None]
    rng = np.random.default_rng(5)
    Q = rng.standard_normal((1, N, d))
    counts = np.array([[np.sum(np.arange(i + 1) % d == c) for c in range(d)] for i in range(N)])
    want = Q * counts[None]
    assert np.allclose(oracle.fwd_def(Q, E, E), want, rtol=1e-13, atol=1e-13)
    assert np.allclose(oracle.fwd_rec(Q, E, E), want, rtol=1e-13, atol=1e-13)
    M = oracle.chunk_states(E, E, [0, N])[0, 0]
    assert np.array_equal(M, np.diag(counts[-1]).astype(np.float64))


def test_docs_of_length_one(oracle):
    """Every document one token long: o_i = (q_i.k_i) v_i and nothing else."""
    Q, K, V, dO = _rand(2, 6, 3, 11)
    cu = list(range(7))
    s = np.sum(Q * K, axis=-1, keepdims=True)
    g = np.sum(dO * V, axis=-1, keepdims=True)
    for fwd in (oracle.fwd_def, oracle.fwd_rec):
        assert np.allclose(fwd(Q, K, V, cu), s * V, rtol=1e-13, atol=1e-14)
    for bwd in (oracle.bwd_def, oracle.bwd_rec):
        dQ, dK, dV = bwd(Q, K, V, dO, cu)
        assert np.allclose(dQ, g * K, rtol=1e-13, atol=1e-14)
        assert np.allclose(dK, g * Q, rtol=1e-13, atol=1e-14)
        assert np.allclose(dV, s * dO, rtol=1e-13, atol=1e-14)


# ------------------------------------------------- reductions to numpy matmul
@pytest.mark.parametrize("N,d", [(1, 1), (7, 4), (33, 5)])
def test_single_chunk_is_tril_matmul(oracle, N, d):
    """One chunk covering the sequence: O = tril(Q K^T) V, a library matmul (LASP-2 intra-chunk formula)."""
    Q, K, V, dO = _rand(2, N, d, 3)
    for g in range(2):
        S = np.tril(Q[g] @ K[g].T)
        Gm = np.tril(dO[g] @ V[g].T)
        assert _rel(oracle.fwd_def(Q, K, V)[g], S @ V[g]) < 1e-13
        dQ, dK, dV = oracle.bwd_def(Q, K, V, dO)
        assert _rel(dQ[g], Gm @ K[g]) < 1e-13
        assert _rel(dK[g], Gm.T @ Q[g]) < 1e-13
        assert _rel(dV[g], S.T @ dO[g]) < 1e-13


def test_last_row_is_unmasked_attention(oracle):
    """The last token sees everything: o_N = q_N (K^T V)  (LASP-2 w/o Masking, O_t = Q_t M_{1:T})."""
    Q, K, V, _ = _rand(3, 29, 6, 4)
    O = oracle.fwd_def(Q, K, V)
    for g in range(3):
        assert _rel(O[g, -1], Q[g, -1] @ (K[g].T @ V[g])) < 1e-13


def test_total_state_is_KtV(oracle):
    """Sum of all chunk states = K^T V over the sequence; last exclusive prefix + last state too."""
    Q, K, V, dO = _rand(2, 37, 5, 6)
    bounds = [0, 4, 4, 13, 20, 37]          # includes an empty chunk
    M = oracle.chunk_states(K, V, bounds)
    P = oracle.state_prefix(M)
    dM = oracle.chunk_states(Q, dO, bounds)
    dP = oracle.state_prefix(dM, reverse=True)
    for g in range(2):
        assert _rel(M[g].sum(0), K[g].T @ V[g]) < 1e-13
        assert _rel(P[g, -1] + M[g, -1], K[g].T @ V[g]) < 1e-13
        assert _rel(dP[g, 0] + dM[g, 0], Q[g].T @ dO[g]) < 1e-13
        assert np.all(P[g, 0] == 0) and np.all(dP[g, -1] == 0)


# ------------------------------------------------ the three families agree
@pytest.mark.parametrize("N,d", [(1, 1), (2, 1), (7, 4), (16, 4), (33, 3)])
def test_definition_equals_recurrence(oracle, N, d):
    Q, K, V, dO = _rand(2, N, d, 100 + N)
    assert _rel(oracle.fwd_rec(Q, K, V), oracle.fwd_def(Q, K, V)) < 1e-12
    for a, b in zip(oracle.bwd_rec(Q, K, V, dO), oracle.bwd_def(Q, K, V, dO)):
        assert _rel(a, b) < 1e-12


@pytest.mark.parametrize("C", [1, 2, 4, 5, 33, 40])
def test_chunk_size_invariance(oracle, C):
    """The chunked algorithm reproduces the definition for any chunk length, ragged tail included."""
    N, d = 33, 4
    Q, K, V, dO = _rand(2, N, d, 7)
    bounds = list(range(0, N, C)) + [N]
    O, _, _ = oracle.forward_by_algorithm(Q, K, V, bounds)
    assert _rel(O, oracle.fwd_def(Q, K, V)) < 1e-12
    got = oracle.backward_by_algorithm(Q, K, V, dO, bounds)[:3]
    for a, b in zip(got, oracle.bwd_def(Q, K, V, dO)):
        assert _rel(a, b) < 1e-12


def test_packed_equals_concatenation(oracle):
    """Packed batch with state reset at boundaries = each document run alone, concatenated."""
    cu = [0, 3, 4, 15, 22, 40]
    Q, K, V, dO = _rand(2, 40, 4, 8)
    for fwd, bwd in ((oracle.fwd_def, oracle.bwd_def), (oracle.fwd_rec, oracle.bwd_rec)):
        O = fwd(Q, K, V, cu)
        grads = bwd(Q, K, V, dO, cu)
        for a, b in zip(cu[:-1], cu[1:]):
            sl = slice(a, b)
            assert _rel(O[:, sl], fwd(Q[:, sl], K[:, sl], V[:, sl])) < 1e-12
            alone = bwd(Q[:, sl], K[:, sl], V[:, sl], dO[:, sl])
            for x, y in zip(grads, alone):
                assert _rel(x[:, sl], y) < 1e-12
    # chunked algorithm with chunks that never span a document, prefix restarted per document
    bounds, first = [0], []
    for a, b in zip(cu[:-1], cu[1:]):
        pos = a
        while pos < b:
            first.append(1 if pos == a else 0)
            pos = min(pos + 4, b)
            bounds.append(pos)
    O, _, _ = oracle.forward_by_algorithm(Q, K, V, bounds, first)
    assert _rel(O, oracle.fwd_def(Q, K, V, cu)) < 1e-12
    got = oracle.backward_by_algorithm(Q, K, V, dO, bounds, first)[:3]
    for x, y in zip(got, oracle.bwd_def(Q, K, V, dO, cu)):
        assert _rel(x, y) < 1e-12


def test_sampled_rows_match_full(oracle):
    cu = [0, 9, 10, 31]
    Q, K, V, dO = _rand(1, 31, 5, 9)
    rows = np.array([0, 8, 9, 10, 17, 30])
    full = (oracle.fwd_def(Q, K, V, cu),) + oracle.bwd_def(Q, K, V, dO, cu)
    for which in range(4):
        got = oracle.def_rows(Q[0], K[0], V[0], dO[0], rows, which, cu)
        assert _rel(got, full[which][0][rows]) < 1e-13


# ------------------------------------------------ gradients vs the forward itself
@pytest.mark.parametrize("cu", [None, [0, 5, 6, 19]])
def test_finite_differences_are_exact(oracle, cu):
    """<dO, O> is linear in each of Q, K, V separately, so a finite difference with ANY step
    equals the directional derivative <grad, E> up to fp64 rounding."""
    Q, K, V, dO = _rand(2, 19, 4, 12)
    rng = np.random.default_rng(13)
    loss = lambda q, k, v: np.sum(dO * oracle.fwd_def(q, k, v, cu))
    base = loss(Q, K, V)
    for bwd in (oracle.bwd_def, oracle.bwd_rec):
        dQ, dK, dV = bwd(Q, K, V, dO, cu)
        for step in (1.0, 1e-3):
            E = rng.standard_normal(Q.shape) * step
            assert abs((loss(Q + E, K, V) - base) - np.sum(dQ * E)) < 1e-10 * (1 + abs(base))
            assert abs((loss(Q, K + E, V) - base) - np.sum(dK * E)) < 1e-10 * (1 + abs(base))
            assert abs((loss(Q, K, V + E) - base) - np.sum(dV * E)) < 1e-10 * (1 + abs(base))


def test_euler_identities(oracle):
    """Linearity in each argument gives <dQ,Q> = <dK,K> = <dV,V> = <dO,O>."""
    cu = [0, 11, 23]
    Q, K, V, dO = _rand(2, 23, 5, 14)
    O = oracle.fwd_def(Q, K, V, cu)
    dQ, dK, dV = oracle.bwd_def(Q, K, V, dO, cu)
    ref = np.sum(dO * O)
    for a, b in ((dQ, Q), (dK, K), (dV, V)):
        assert abs(np.sum(a * b) - ref) < 1e-11 * abs(ref)


# ------------------------------------------------ planted mistakes are caught
def test_pins_catch_planted_mistakes(oracle):
    """A wrong oracle (strict mask, transposed state, swapped K/V) must fail the hand example."""
    g = json.load(open(os.path.join(GOLD, "hand_example.json")))
    Q, K, V = (np.array(g[k], dtype=np.float64) for k in ("Q", "K", "V"))
    want = np.array(g["O"], dtype=np.float64)
    strict = np.tril(Q @ K.T, -1) @ V                      # diagonal dropped
    swapped = np.tril(Q @ V.T) @ K                         # K and V exchanged
    transposed = np.stack([Q[i] @ (K[: i + 1].T @ V[: i + 1]).T for i in range(3)])  # M^T
    for wrong in (strict, swapped, transposed):
        assert not np.array_equal(wrong, want)


# ------------------------------------------------ cost-model arithmetic
def test_cost_model_arithmetic():
    g = json.load(open(os.path.join(GOLD, "cost_model.json")))
    for c in g["cases"]:
        elems = c["B"] * c["H"] * c["d"] ** 2
        assert round(elems / 1e9, 2) == c["elements_billion"]
        assert round(elems * 2 / 1e9, 2) == pytest.approx(c["fp16_GB"], abs=0.011)
    assert g["steps_lasp2"] == 2 and g["steps_lasp1_W64"] == 2 * (64 - 1)
