"""CPU oracle for causal linear attention (LASP-2, Eq. (3), Eq. (4), and the
steps of the masked forward/backward algorithms).

TEST INFRASTRUCTURE ONLY: imported by tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py.  The GPU library never imports or links this.

All functions take and return float64 numpy arrays shaped [G, N, d] (G = B*H
independent groups).  `cu` is the list of document offsets (None = one
document covering all N tokens).
"""
import ctypes
import os

import numpy as np

from . import build as _build

_LIB = None
_c_dp = ctypes.POINTER(ctypes.c_double)
_c_lp = ctypes.POINTER(ctypes.c_long)
_c_ip = ctypes.POINTER(ctypes.c_int)


def _lib():
    global _LIB
    if _LIB is None:
        path = _build.build(force=False)
        _LIB = ctypes.CDLL(path)
        _LIB.lasp2_oracle_threads.restype = ctypes.c_int
    return _LIB


def threads() -> int:
    return int(_lib().lasp2_oracle_threads())


def _d(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(_c_dp)


def _l(a):
    a = np.ascontiguousarray(a, dtype=np.int64)
    return a, a.ctypes.data_as(_c_lp)


def _cu(cu, N):
    if cu is None:
        cu = [0, N]
    cu = np.asarray(cu, dtype=np.int64)
    assert cu[0] == 0 and cu[-1] == N and np.all(np.diff(cu) > 0), "bad document offsets"
    return cu


def _gnd(x):
    assert x.ndim == 3, "expected [G, N, d]"
    return x.shape


def fwd_def(Q, K, V, cu=None):
    """Eq. (3), brute force."""
    G, N, d = _gnd(Q)
    Q, q = _d(Q); K, k = _d(K); V, v = _d(V)
    O = np.empty((G, N, d)); o = O.ctypes.data_as(_c_dp)
    cu, c = _l(_cu(cu, N))
    _lib().lasp2_oracle_fwd_def(q, k, v, o, ctypes.c_long(G), ctypes.c_long(N), ctypes.c_long(d),
                                c, ctypes.c_long(len(cu) - 1))
    return O


def bwd_def(Q, K, V, dO, cu=None):
    """Analytic gradient of <dO, O> under Eq. (3), brute force."""
    G, N, d = _gnd(Q)
    Q, q = _d(Q); K, k = _d(K); V, v = _d(V); dO, g = _d(dO)
    dQ = np.empty((G, N, d)); dK = np.empty((G, N, d)); dV = np.empty((G, N, d))
    cu, c = _l(_cu(cu, N))
    _lib().lasp2_oracle_bwd_def(q, k, v, g, dQ.ctypes.data_as(_c_dp), dK.ctypes.data_as(_c_dp),
                                dV.ctypes.data_as(_c_dp), ctypes.c_long(G), ctypes.c_long(N),
                                ctypes.c_long(d), c, ctypes.c_long(len(cu) - 1))
    return dQ, dK, dV


def def_rows(Q, K, V, dO, rows, which, cu=None):
    """Rows `rows` of O (which=0), dQ (1), dK (2) or dV (3) for ONE group; Q,K,V,dO are [N, d]."""
    N, d = Q.shape
    Q, q = _d(Q); K, k = _d(K); V, v = _d(V)
    if dO is None:
        assert which == 0
        g = None
    else:
        dO, g = _d(dO)
    rows, r = _l(rows)
    out = np.empty((len(rows), d))
    cu, c = _l(_cu(cu, N))
    _lib().lasp2_oracle_def_rows(q, k, v, g, ctypes.c_long(N), ctypes.c_long(d), c,
                                 ctypes.c_long(len(cu) - 1), r, ctypes.c_long(len(rows)),
                                 ctypes.c_int(which), out.ctypes.data_as(_c_dp))
    return out


def fwd_rec(Q, K, V, cu=None):
    """Eq. (4), token recurrence."""
    G, N, d = _gnd(Q)
    Q, q = _d(Q); K, k = _d(K); V, v = _d(V)
    O = np.empty((G, N, d))
    cu, c = _l(_cu(cu, N))
    _lib().lasp2_oracle_fwd_rec(q, k, v, O.ctypes.data_as(_c_dp), ctypes.c_long(G), ctypes.c_long(N),
                                ctypes.c_long(d), c, ctypes.c_long(len(cu) - 1))
    return O


def bwd_rec(Q, K, V, dO, cu=None):
    """Backward of Eq. (4): forward scan for dQ, reverse adjoint scan for dK, dV."""
    G, N, d = _gnd(Q)
    Q, q = _d(Q); K, k = _d(K); V, v = _d(V); dO, g = _d(dO)
    dQ = np.empty((G, N, d)); dK = np.empty((G, N, d)); dV = np.empty((G, N, d))
    cu, c = _l(_cu(cu, N))
    _lib().lasp2_oracle_bwd_rec(q, k, v, g, dQ.ctypes.data_as(_c_dp), dK.ctypes.data_as(_c_dp),
                                dV.ctypes.data_as(_c_dp), ctypes.c_long(G), ctypes.c_long(N),
                                ctypes.c_long(d), c, ctypes.c_long(len(cu) - 1))
    return dQ, dK, dV


def _bounds(bounds, N):
    b = np.asarray(bounds, dtype=np.int64)
    assert b[0] == 0 and b[-1] == N and np.all(np.diff(b) >= 0), "bad chunk bounds"
    return b


def chunk_states(K, V, bounds):
    """M_t = K_t^T V_t for every chunk t of the partition `bounds`; returns [G, T, d, d]."""
    G, N, d = _gnd(K)
    K, k = _d(K); V, v = _d(V)
    b, bp = _l(_bounds(bounds, N))
    T = len(b) - 1
    M = np.empty((G, T, d, d))
    _lib().lasp2_oracle_chunk_states(k, v, M.ctypes.data_as(_c_dp), ctypes.c_long(G), ctypes.c_long(N),
                                     ctypes.c_long(d), bp, ctypes.c_long(T))
    return M


def state_prefix(M, first=None, reverse=False):
    """Exclusive PrefixSum (or SuffixSum) of [G, T, d, d] states, restarted at document edges."""
    G, T, d, d2 = M.shape
    assert d == d2
    M, m = _d(M)
    P = np.empty_like(M)
    if first is None:
        fp = None
    else:
        first = np.ascontiguousarray(first, dtype=np.int32)
        assert first.shape == (T,)
        fp = first.ctypes.data_as(_c_ip)
    _lib().lasp2_oracle_state_prefix(m, P.ctypes.data_as(_c_dp), ctypes.c_long(G), ctypes.c_long(T),
                                     ctypes.c_long(d), fp, ctypes.c_int(1 if reverse else 0))
    return P


def attn_fwd_chunked(Q, K, V, P, bounds):
    """O_t = [(Q_t K_t^T) (.) Psi] V_t + Q_t P_t per chunk."""
    G, N, d = _gnd(Q)
    Q, q = _d(Q); K, k = _d(K); V, v = _d(V); P, p = _d(P)
    b, bp = _l(_bounds(bounds, N))
    O = np.zeros((G, N, d))
    _lib().lasp2_oracle_attn_fwd_chunked(q, k, v, p, O.ctypes.data_as(_c_dp), ctypes.c_long(G),
                                         ctypes.c_long(N), ctypes.c_long(d), bp, ctypes.c_long(len(b) - 1))
    return O


def attn_bwd_chunked(Q, K, V, dO, P, dP, bounds):
    """dQ_t, dK_t, dV_t per chunk from the cached prefix P_t and the suffix dP_t."""
    G, N, d = _gnd(Q)
    Q, q = _d(Q); K, k = _d(K); V, v = _d(V); dO, g = _d(dO); P, p = _d(P); dP, dp = _d(dP)
    b, bp = _l(_bounds(bounds, N))
    dQ = np.zeros((G, N, d)); dK = np.zeros((G, N, d)); dV = np.zeros((G, N, d))
    _lib().lasp2_oracle_attn_bwd_chunked(q, k, v, g, p, dp, dQ.ctypes.data_as(_c_dp),
                                         dK.ctypes.data_as(_c_dp), dV.ctypes.data_as(_c_dp),
                                         ctypes.c_long(G), ctypes.c_long(N), ctypes.c_long(d), bp,
                                         ctypes.c_long(len(b) - 1))
    return dQ, dK, dV


def forward_by_algorithm(Q, K, V, bounds, first=None):
    """All forward steps in the paper's order: states -> prefix -> intra + inter."""
    M = chunk_states(K, V, bounds)
    P = state_prefix(M, first, reverse=False)
    return attn_fwd_chunked(Q, K, V, P, bounds), M, P


def backward_by_algorithm(Q, K, V, dO, bounds, first=None):
    """All backward steps in the paper's order: dM_t -> suffix -> intra + inter."""
    P = state_prefix(chunk_states(K, V, bounds), first, reverse=False)
    dM = chunk_states(Q, dO, bounds)
    dP = state_prefix(dM, first, reverse=True)
    return attn_bwd_chunked(Q, K, V, dO, P, dP, bounds) + (dM, dP)


# ---------------------------------------------------------------------------
# Without masking (Algorithm "LASP-2 w/o Masking" and its backward pass)
# ---------------------------------------------------------------------------

def nomask_fwd_def(Q, K, V, cu=None):
    """O_i = sum over ALL j of the document of (q_i . k_j) v_j, brute force."""
    G, N, d = _gnd(Q)
    Q, q = _d(Q); K, k = _d(K); V, v = _d(V)
    O = np.empty((G, N, d))
    cu, c = _l(_cu(cu, N))
    _lib().lasp2_oracle_nomask_fwd_def(q, k, v, O.ctypes.data_as(_c_dp), ctypes.c_long(G), ctypes.c_long(N),
                                       ctypes.c_long(d), c, ctypes.c_long(len(cu) - 1))
    return O


def nomask_bwd_def(Q, K, V, dO, cu=None):
    """Analytic gradient of <dO, O> for the unmasked definition, brute force."""
    G, N, d = _gnd(Q)
    Q, q = _d(Q); K, k = _d(K); V, v = _d(V); dO, g = _d(dO)
    dQ = np.empty((G, N, d)); dK = np.empty((G, N, d)); dV = np.empty((G, N, d))
    cu, c = _l(_cu(cu, N))
    _lib().lasp2_oracle_nomask_bwd_def(q, k, v, g, dQ.ctypes.data_as(_c_dp), dK.ctypes.data_as(_c_dp),
                                       dV.ctypes.data_as(_c_dp), ctypes.c_long(G), ctypes.c_long(N),
                                       ctypes.c_long(d), c, ctypes.c_long(len(cu) - 1))
    return dQ, dK, dV


def nomask_def_rows(Q, K, V, dO, rows, which, cu=None):
    """Rows `rows` of O (which=0), dQ (1), dK (2) or dV (3) of the unmasked definition, ONE group."""
    N, d = Q.shape
    Q, q = _d(Q); K, k = _d(K); V, v = _d(V)
    if dO is None:
        assert which == 0
        g = None
    else:
        dO, g = _d(dO)
    rows, r = _l(rows)
    out = np.empty((len(rows), d))
    cu, c = _l(_cu(cu, N))
    _lib().lasp2_oracle_nomask_def_rows(q, k, v, g, ctypes.c_long(N), ctypes.c_long(d), c,
                                        ctypes.c_long(len(cu) - 1), r, ctypes.c_long(len(rows)),
                                        ctypes.c_int(which), out.ctypes.data_as(_c_dp))
    return out


def state_total(M, first=None):
    """Sum of the [G, T, d, d] states of each document, handed to every chunk of that document."""
    G, T, d, d2 = M.shape
    assert d == d2
    M, m = _d(M)
    S = np.empty_like(M)
    if first is None:
        fp = None
    else:
        first = np.ascontiguousarray(first, dtype=np.int32)
        assert first.shape == (T,)
        fp = first.ctypes.data_as(_c_ip)
    _lib().lasp2_oracle_state_total(m, S.ctypes.data_as(_c_dp), ctypes.c_long(G), ctypes.c_long(T),
                                    ctypes.c_long(d), fp)
    return S


def rows_times_state(A, S, bounds, transpose=False):
    """out_t = A_t S_t (or A_t S_t^T) per chunk."""
    G, N, d = _gnd(A)
    A, a = _d(A); S, s = _d(S)
    b, bp = _l(_bounds(bounds, N))
    assert S.shape == (G, len(b) - 1, d, d)
    out = np.zeros((G, N, d))
    _lib().lasp2_oracle_rows_times_state(a, s, out.ctypes.data_as(_c_dp), ctypes.c_long(G), ctypes.c_long(N),
                                         ctypes.c_long(d), bp, ctypes.c_long(len(b) - 1),
                                         ctypes.c_int(1 if transpose else 0))
    return out


def nomask_forward_by_algorithm(Q, K, V, bounds, first=None):
    """Forward steps without masking: M_t -> M_{1:T} -> O_t = Q_t M_{1:T}."""
    M = chunk_states(K, V, bounds)
    S = state_total(M, first)
    return rows_times_state(Q, S, bounds), M, S


def nomask_backward_by_algorithm(Q, K, V, dO, bounds, first=None):
    """Backward steps without masking: dM_t -> dM_{1:T}; dQ = dO M^T, dK = V dM^T, dV = K dM."""
    S = state_total(chunk_states(K, V, bounds), first)
    dS = state_total(chunk_states(Q, dO, bounds), first)
    dQ = rows_times_state(dO, S, bounds, transpose=True)
    dK = rows_times_state(V, dS, bounds, transpose=True)
    dV = rows_times_state(K, dS, bounds)
    return dQ, dK, dV, dS


# ---------------------------------------------------------------------------
# Scalar decay: lam is one factor in (0, 1] per group (shape [G]); lam = 1 is the plain case.
# ---------------------------------------------------------------------------

def _lam(lam, G):
    lam = np.ascontiguousarray(np.broadcast_to(np.asarray(lam, dtype=np.float64), (G,)))
    assert np.all(lam > 0) and np.all(lam <= 1), "decay factors must lie in (0, 1]"
    return lam, lam.ctypes.data_as(_c_dp)


def fwd_def_decay(Q, K, V, lam, cu=None):
    """O_i = sum_{j<=i} lam^(i-j) (q_i . k_j) v_j, brute force."""
    G, N, d = _gnd(Q)
    Q, q = _d(Q); K, k = _d(K); V, v = _d(V)
    O = np.empty((G, N, d))
    cu, c = _l(_cu(cu, N)); lam, lp = _lam(lam, G)
    _lib().lasp2_oracle_fwd_def_decay(q, k, v, O.ctypes.data_as(_c_dp), ctypes.c_long(G), ctypes.c_long(N),
                                      ctypes.c_long(d), c, ctypes.c_long(len(cu) - 1), lp)
    return O


def bwd_def_decay(Q, K, V, dO, lam, cu=None):
    G, N, d = _gnd(Q)
    Q, q = _d(Q); K, k = _d(K); V, v = _d(V); dO, g = _d(dO)
    dQ = np.empty((G, N, d)); dK = np.empty((G, N, d)); dV = np.empty((G, N, d))
    cu, c = _l(_cu(cu, N)); lam, lp = _lam(lam, G)
    _lib().lasp2_oracle_bwd_def_decay(q, k, v, g, dQ.ctypes.data_as(_c_dp), dK.ctypes.data_as(_c_dp),
                                      dV.ctypes.data_as(_c_dp), ctypes.c_long(G), ctypes.c_long(N),
                                      ctypes.c_long(d), c, ctypes.c_long(len(cu) - 1), lp)
    return dQ, dK, dV


def fwd_rec_decay(Q, K, V, lam, cu=None):
    """M_s = lam M_{s-1} + k_s^T v_s, o_s = q_s M_s."""
    G, N, d = _gnd(Q)
    Q, q = _d(Q); K, k = _d(K); V, v = _d(V)
    O = np.empty((G, N, d))
    cu, c = _l(_cu(cu, N)); lam, lp = _lam(lam, G)
    _lib().lasp2_oracle_fwd_rec_decay(q, k, v, O.ctypes.data_as(_c_dp), ctypes.c_long(G), ctypes.c_long(N),
                                      ctypes.c_long(d), c, ctypes.c_long(len(cu) - 1), lp)
    return O


def bwd_rec_decay(Q, K, V, dO, lam, cu=None):
    G, N, d = _gnd(Q)
    Q, q = _d(Q); K, k = _d(K); V, v = _d(V); dO, g = _d(dO)
    dQ = np.empty((G, N, d)); dK = np.empty((G, N, d)); dV = np.empty((G, N, d))
    cu, c = _l(_cu(cu, N)); lam, lp = _lam(lam, G)
    _lib().lasp2_oracle_bwd_rec_decay(q, k, v, g, dQ.ctypes.data_as(_c_dp), dK.ctypes.data_as(_c_dp),
                                      dV.ctypes.data_as(_c_dp), ctypes.c_long(G), ctypes.c_long(N),
                                      ctypes.c_long(d), c, ctypes.c_long(len(cu) - 1), lp)
    return dQ, dK, dV


def chunk_states_decay(X, Y, bounds, lam, anchor_start=False):
    """Decayed chunk states, anchored at each chunk's last token (or its first)."""
    G, N, d = _gnd(X)
    X, x = _d(X); Y, y = _d(Y)
    b, bp = _l(_bounds(bounds, N)); lam, lp = _lam(lam, G)
    T = len(b) - 1
    M = np.empty((G, T, d, d))
    _lib().lasp2_oracle_chunk_states_decay(x, y, M.ctypes.data_as(_c_dp), ctypes.c_long(G), ctypes.c_long(N),
                                           ctypes.c_long(d), bp, ctypes.c_long(T), lp,
                                           ctypes.c_int(1 if anchor_start else 0))
    return M


def state_prefix_decay(M, bounds, lam, first=None, reverse=False):
    """Decayed exclusive combine of [G, T, d, d] states over the chunk partition `bounds`."""
    G, T, d, d2 = M.shape
    assert d == d2
    M, m = _d(M)
    b, bp = _l(np.asarray(bounds, dtype=np.int64)); lam, lp = _lam(lam, G)
    assert len(b) == T + 1
    P = np.empty_like(M)
    if first is None:
        fp = None
    else:
        first = np.ascontiguousarray(first, dtype=np.int32)
        assert first.shape == (T,)
        fp = first.ctypes.data_as(_c_ip)
    _lib().lasp2_oracle_state_prefix_decay(m, P.ctypes.data_as(_c_dp), ctypes.c_long(G), ctypes.c_long(T),
                                           ctypes.c_long(d), fp, ctypes.c_int(1 if reverse else 0), bp, lp)
    return P


def attn_fwd_chunked_decay(Q, K, V, P, bounds, lam):
    G, N, d = _gnd(Q)
    Q, q = _d(Q); K, k = _d(K); V, v = _d(V); P, p = _d(P)
    b, bp = _l(_bounds(bounds, N)); lam, lp = _lam(lam, G)
    O = np.zeros((G, N, d))
    _lib().lasp2_oracle_attn_fwd_chunked_decay(q, k, v, p, O.ctypes.data_as(_c_dp), ctypes.c_long(G),
                                               ctypes.c_long(N), ctypes.c_long(d), bp,
                                               ctypes.c_long(len(b) - 1), lp)
    return O


def attn_bwd_chunked_decay(Q, K, V, dO, P, dP, bounds, lam):
    G, N, d = _gnd(Q)
    Q, q = _d(Q); K, k = _d(K); V, v = _d(V); dO, g = _d(dO); P, p = _d(P); dP, dp = _d(dP)
    b, bp = _l(_bounds(bounds, N)); lam, lp = _lam(lam, G)
    dQ = np.zeros((G, N, d)); dK = np.zeros((G, N, d)); dV = np.zeros((G, N, d))
    _lib().lasp2_oracle_attn_bwd_chunked_decay(q, k, v, g, p, dp, dQ.ctypes.data_as(_c_dp),
                                               dK.ctypes.data_as(_c_dp), dV.ctypes.data_as(_c_dp),
                                               ctypes.c_long(G), ctypes.c_long(N), ctypes.c_long(d), bp,
                                               ctypes.c_long(len(b) - 1), lp)
    return dQ, dK, dV


def forward_by_algorithm_decay(Q, K, V, bounds, lam, first=None):
    """Decayed forward steps: states (end-anchored) -> decayed prefix -> intra + inter."""
    M = chunk_states_decay(K, V, bounds, lam)
    P = state_prefix_decay(M, bounds, lam, first, reverse=False)
    return attn_fwd_chunked_decay(Q, K, V, P, bounds, lam), M, P


def backward_by_algorithm_decay(Q, K, V, dO, bounds, lam, first=None):
    """Decayed backward steps: dM (start-anchored) -> decayed suffix -> intra + inter."""
    P = state_prefix_decay(chunk_states_decay(K, V, bounds, lam), bounds, lam, first, reverse=False)
    dM = chunk_states_decay(Q, dO, bounds, lam, anchor_start=True)
    dP = state_prefix_decay(dM, bounds, lam, first, reverse=True)
    return attn_bwd_chunked_decay(Q, K, V, dO, P, dP, bounds, lam) + (dM, dP)


def def_rows_decay(Q, K, V, dO, rows, which, lam, cu=None):
    """Rows `rows` of O (which=0), dQ (1), dK (2) or dV (3) of the decayed definition, ONE group."""
    N, d = Q.shape
    Q, q = _d(Q); K, k = _d(K); V, v = _d(V)
    if dO is None:
        assert which == 0
        g = None
    else:
        dO, g = _d(dO)
    rows, r = _l(rows)
    out = np.empty((len(rows), d))
    cu, c = _l(_cu(cu, N))
    _lib().lasp2_oracle_def_rows_decay(q, k, v, g, ctypes.c_long(N), ctypes.c_long(d), c,
                                       ctypes.c_long(len(cu) - 1), r, ctypes.c_long(len(rows)),
                                       ctypes.c_int(which), ctypes.c_double(float(lam)),
                                       out.ctypes.data_as(_c_dp))
    return out


# ---------------------------------------------------------------------------
# Softmax attention (Algorithm "AllGather-based Context Parallelism", compute line)
# ---------------------------------------------------------------------------

def softmax_fwd(Q, K, V, causal=False, cu=None):
    """O = Softmax(Q K^T / sqrt(d)) V per group and document; returns (O, lse)."""
    G, N, d = _gnd(Q)
    Q, q = _d(Q); K, k = _d(K); V, v = _d(V)
    O = np.empty((G, N, d)); lse = np.empty((G, N))
    cu, c = _l(_cu(cu, N))
    _lib().lasp2_oracle_softmax_fwd(q, k, v, O.ctypes.data_as(_c_dp), lse.ctypes.data_as(_c_dp),
                                    ctypes.c_long(G), ctypes.c_long(N), ctypes.c_long(d), c,
                                    ctypes.c_long(len(cu) - 1), ctypes.c_int(1 if causal else 0))
    return O, lse


def softmax_bwd(Q, K, V, dO, causal=False, cu=None):
    G, N, d = _gnd(Q)
    Q, q = _d(Q); K, k = _d(K); V, v = _d(V); dO, g = _d(dO)
    dQ = np.empty((G, N, d)); dK = np.empty((G, N, d)); dV = np.empty((G, N, d))
    cu, c = _l(_cu(cu, N))
    _lib().lasp2_oracle_softmax_bwd(q, k, v, g, dQ.ctypes.data_as(_c_dp), dK.ctypes.data_as(_c_dp),
                                    dV.ctypes.data_as(_c_dp), ctypes.c_long(G), ctypes.c_long(N),
                                    ctypes.c_long(d), c, ctypes.c_long(len(cu) - 1),
                                    ctypes.c_int(1 if causal else 0))
    return dQ, dK, dV


def softmax_rows(Q, K, V, rows, causal=False, cu=None):
    """Rows `rows` of the softmax output and their log-sum-exp for ONE group; Q,K,V are [N, d]."""
    N, d = Q.shape
    Q, q = _d(Q); K, k = _d(K); V, v = _d(V)
    rows, r = _l(rows)
    out = np.empty((len(rows), d)); lse = np.empty(len(rows))
    cu, c = _l(_cu(cu, N))
    _lib().lasp2_oracle_softmax_rows(q, k, v, ctypes.c_long(N), ctypes.c_long(d), c,
                                     ctypes.c_long(len(cu) - 1), r, ctypes.c_long(len(rows)),
                                     ctypes.c_int(1 if causal else 0), out.ctypes.data_as(_c_dp),
                                     lse.ctypes.data_as(_c_dp))
    return out, lse

def softmax_bwd_rows(Q, K, V, dO, lse, delta, rows, which, causal=False, cu=None):
    """Rows `rows` of dQ (which=0), dK (1) or dV (2) for ONE group; Q,K,V,dO are [N, d]; lse and
    delta = rowsum(dO * O) are this oracle's own forward results for all N rows of the group."""
    N, d = Q.shape
    Q, q = _d(Q); K, k = _d(K); V, v = _d(V); dO, g = _d(dO)
    lse, l = _d(lse); delta, dl = _d(delta)
    rows, r = _l(rows)
    out = np.empty((len(rows), d))
    cu, c = _l(_cu(cu, N))
    _lib().lasp2_oracle_softmax_bwd_rows(q, k, v, g, l, dl, ctypes.c_long(N), ctypes.c_long(d), c,
                                         ctypes.c_long(len(cu) - 1), r, ctypes.c_long(len(rows)),
                                         ctypes.c_int(which), ctypes.c_int(1 if causal else 0),
                                         out.ctypes.data_as(_c_dp))
    return out
