"""ctypes binding of liblasp2.so: same names as the C ABI in include/lasp2.h.

Argument marshalling only.  Tensors are torch CUDA tensors (torch is used for
device memory and streams); every step of the computation runs in the HIP
library.  There is no fallback: if the library is missing, importing the
entry points raises.
"""
import ctypes
import os

import numpy as np
import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
# LASP2_LIB_PATH names another build of the same library (e.g. the -DLASP2_FULL_WAITS checking
# variant, see build.py); there is still no fallback: the named file must exist.
LIB_PATH = os.environ.get("LASP2_LIB_PATH") or os.path.join(_PKG, "liblasp2.so")

LASP2_F32, LASP2_BF16 = 0, 1
STATUS = {0: "LASP2_OK", -1: "LASP2_ERR_NULL", -2: "LASP2_ERR_SHAPE", -3: "LASP2_ERR_DTYPE",
          -4: "LASP2_ERR_SEQLENS", -5: "LASP2_ERR_WORKSPACE", -6: "LASP2_ERR_ALIGN",
          -7: "LASP2_ERR_LAUNCH", -8: "LASP2_ERR_DECAY"}


class Desc(ctypes.Structure):
    """Mirror of lasp2_desc_t."""
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("N", ctypes.c_int32),
                ("d", ctypes.c_int32), ("C", ctypes.c_int32), ("L", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("n_seqs", ctypes.c_int32),
                ("cu_seqlens_host", ctypes.c_void_p), ("cu_seqlens_dev", ctypes.c_void_p),
                ("decay_host", ctypes.c_void_p), ("decay_dev", ctypes.c_void_p)]


class Lasp2Error(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__(f"{where}: {STATUS.get(code, code)} ({status_string(code)})")


_lib = None


def lib():
    """The loaded C-ABI library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2502_07563_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        vp, i64p, szp = ctypes.c_void_p, ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_size_t)
        dp = ctypes.POINTER(Desc)
        L.lasp2_num_slots.argtypes = [dp, i64p]
        L.lasp2_workspace_size.argtypes = [dp, szp]
        L.lasp2_walk_slots.argtypes = [dp, ctypes.c_int, i64p]
        L.lasp2_chunk_states.argtypes = [dp, vp, vp, vp, vp]
        L.lasp2_state_prefix.argtypes = [dp, vp, vp, ctypes.c_int, vp]
        L.lasp2_attn_fwd.argtypes = [dp, vp, vp, vp, vp, vp, vp]
        L.lasp2_attn_bwd.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        L.lasp2_attn_bwd_noalloc.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.lasp2_state_total.argtypes = [dp, vp, vp, vp]
        L.lasp2_nomask_fwd.argtypes = [dp, vp, vp, vp, vp]
        L.lasp2_nomask_bwd.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        L.lasp2_softmax_fwd.argtypes = [dp, vp, vp, vp, vp, vp, ctypes.c_int, vp]
        L.lasp2_softmax_workspace_size.argtypes = [dp, szp]
        L.lasp2_softmax_bwd.argtypes = [dp] + [vp] * 10 + [ctypes.c_size_t, ctypes.c_int, vp]
        i64 = ctypes.c_int64
        L.lasp2_softmax_fwd_share.argtypes = [dp, i64, i64, vp, vp, vp, vp, vp, ctypes.c_int, vp]
        L.lasp2_softmax_share_workspace_size.argtypes = [dp, i64, szp]
        L.lasp2_softmax_bwd_share.argtypes = [dp, i64, i64] + [vp] * 10 + [ctypes.c_size_t, ctypes.c_int, vp]
        L.lasp2_status_string.argtypes = [ctypes.c_int]
        L.lasp2_status_string.restype = ctypes.c_char_p
        for name in ("lasp2_num_slots", "lasp2_workspace_size", "lasp2_walk_slots", "lasp2_chunk_states",
                     "lasp2_state_prefix", "lasp2_attn_fwd", "lasp2_attn_bwd", "lasp2_attn_bwd_noalloc",
                     "lasp2_state_total",
                     "lasp2_nomask_fwd", "lasp2_nomask_bwd", "lasp2_softmax_fwd",
                     "lasp2_softmax_workspace_size", "lasp2_softmax_bwd", "lasp2_softmax_fwd_share",
                     "lasp2_softmax_share_workspace_size", "lasp2_softmax_bwd_share"):
            getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def status_string(code: int) -> str:
    return lib().lasp2_status_string(int(code)).decode()


class Problem:
    """A descriptor plus the host/device copies of the packed-sequence offsets it points to."""

    def __init__(self, B, H, N, d, C, L=0, dtype="bf16", cu_seqlens=None, device="cuda", decay=None):
        self.B, self.H, self.N, self.d, self.C, self.L = B, H, N, d, C, L
        self.dtype = dtype
        self.torch_dtype = {"f32": torch.float32, "bf16": torch.bfloat16}[dtype]
        self.desc = Desc(B=B, H=H, N=N, d=d, C=C, L=L,
                         dtype={"f32": LASP2_F32, "bf16": LASP2_BF16}[dtype], n_seqs=0,
                         cu_seqlens_host=None, cu_seqlens_dev=None, decay_host=None, decay_dev=None)
        self._cu_host = self._cu_dev = None
        if cu_seqlens is not None:
            self._cu_host = np.ascontiguousarray(cu_seqlens, dtype=np.int32)
            self._cu_dev = torch.from_numpy(self._cu_host).to(device)
            self.desc.n_seqs = len(self._cu_host) - 1
            self.desc.cu_seqlens_host = self._cu_host.ctypes.data
            self.desc.cu_seqlens_dev = self._cu_dev.data_ptr()

        self._decay_host = self._decay_dev = None
        if decay is not None:      # one factor per head
            self._decay_host = np.ascontiguousarray(np.broadcast_to(np.asarray(decay, dtype=np.float32), (H,)))
            self._decay_dev = torch.from_numpy(self._decay_host.copy()).to(device)
            self.desc.decay_host = self._decay_host.ctypes.data
            self.desc.decay_dev = self._decay_dev.data_ptr()

    @property
    def ref(self):
        return ctypes.byref(self.desc)


def _check(code, where):
    if code != 0:
        raise Lasp2Error(code, where)


def _ptr(t):
    """Device address of a tensor for the C ABI.  The kernels trust their pointers, so what torch
    can tell about them is checked here: device memory, dense layout."""
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("lasp2: tensors must live in device memory (got a host tensor)")
    if not t.is_contiguous():
        raise ValueError("lasp2: tensors must be contiguous")
    return ctypes.c_void_p(t.data_ptr())


def _rows(p, t, n_tokens, name):
    """A [B,H,n_tokens,d] tensor of the problem's dtype (None passes: the library reports it)."""
    if t is None:
        return
    if t.dtype != p.torch_dtype:
        raise ValueError(f"lasp2: {name} has dtype {t.dtype}, the problem is {p.torch_dtype}")
    if t.numel() != p.B * p.H * n_tokens * p.d:
        raise ValueError(f"lasp2: {name} has {t.numel()} elements, expected B*H*{n_tokens}*d = "
                         f"{p.B * p.H * n_tokens * p.d}")


def _f32(t, numel, name):
    """An fp32 array of at least `numel` elements (states, log-sum-exp, scratch)."""
    if t is None:
        return
    if t.dtype != torch.float32:
        raise ValueError(f"lasp2: {name} must be float32, got {t.dtype}")
    if t.numel() < numel:
        raise ValueError(f"lasp2: {name} has {t.numel()} elements, needs at least {numel}")


def _states(p, t, name):
    """An fp32 [B,H,T_s,d,d] state array."""
    _f32(t, p.B * p.H * lasp2_num_slots(p) * p.d * p.d, name)


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def lasp2_num_slots(p: Problem) -> int:
    out = ctypes.c_int64(0)
    _check(lib().lasp2_num_slots(p.ref, ctypes.byref(out)), "lasp2_num_slots")
    return out.value


def lasp2_walk_slots(p: Problem, backward=False) -> int:
    out = ctypes.c_int64(0)
    _check(lib().lasp2_walk_slots(p.ref, 1 if backward else 0, ctypes.byref(out)), "lasp2_walk_slots")
    return out.value


def lasp2_workspace_size(p: Problem) -> int:
    out = ctypes.c_size_t(0)
    _check(lib().lasp2_workspace_size(p.ref, ctypes.byref(out)), "lasp2_workspace_size")
    return out.value


def lasp2_chunk_states(p: Problem, K, V, M, stream=None):
    _rows(p, K, p.N, 'K'); _rows(p, V, p.N, 'V'); _states(p, M, 'M')
    _check(lib().lasp2_chunk_states(p.ref, _ptr(K), _ptr(V), _ptr(M), _stream(stream)),
           "lasp2_chunk_states")


def lasp2_state_prefix(p: Problem, M, P, reverse=False, stream=None):
    _states(p, M, 'M'); _states(p, P, 'P')
    _check(lib().lasp2_state_prefix(p.ref, _ptr(M), _ptr(P), 1 if reverse else 0, _stream(stream)),
           "lasp2_state_prefix")


def lasp2_attn_fwd(p: Problem, Q, K, V, P, O, stream=None):
    for n, t in (('Q', Q), ('K', K), ('V', V), ('O', O)):
        _rows(p, t, p.N, n)
    _states(p, P, 'P')
    _check(lib().lasp2_attn_fwd(p.ref, _ptr(Q), _ptr(K), _ptr(V), _ptr(P), _ptr(O), _stream(stream)),
           "lasp2_attn_fwd")


def lasp2_attn_bwd(p: Problem, Q, K, V, dO, P, dQ, dK, dV, workspace, stream=None):
    for n, t in (('Q', Q), ('K', K), ('V', V), ('dO', dO), ('dQ', dQ), ('dK', dK), ('dV', dV)):
        _rows(p, t, p.N, n)
    _states(p, P, 'P')
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().lasp2_attn_bwd(p.ref, _ptr(Q), _ptr(K), _ptr(V), _ptr(dO), _ptr(P), _ptr(dQ),
                                _ptr(dK), _ptr(dV), _ptr(workspace), ctypes.c_size_t(nbytes),
                                _stream(stream)), "lasp2_attn_bwd")


NOALLOC_SCRATCH_BYTES = (64 << 20) + (64 << 10)     # LASP2_NOALLOC_SCRATCH_BYTES


def lasp2_attn_bwd_noalloc(p: Problem, Q, K, V, dO, P, dQ, dK, dV, stream=None):
    for n, t in (('Q', Q), ('K', K), ('V', V), ('dO', dO), ('dQ', dQ), ('dK', dK), ('dV', dV)):
        _rows(p, t, p.N, n)
    _states(p, P, 'P')
    _check(lib().lasp2_attn_bwd_noalloc(p.ref, _ptr(Q), _ptr(K), _ptr(V), _ptr(dO), _ptr(P), _ptr(dQ),
                                        _ptr(dK), _ptr(dV), _stream(stream)), "lasp2_attn_bwd_noalloc")


def lasp2_state_total(p: Problem, M, S, stream=None):
    _states(p, M, 'M'); _states(p, S, 'S')
    _check(lib().lasp2_state_total(p.ref, _ptr(M), _ptr(S), _stream(stream)), "lasp2_state_total")


def lasp2_nomask_fwd(p: Problem, Q, S, O, stream=None):
    _rows(p, Q, p.N, 'Q'); _rows(p, O, p.N, 'O'); _states(p, S, 'S')
    _check(lib().lasp2_nomask_fwd(p.ref, _ptr(Q), _ptr(S), _ptr(O), _stream(stream)), "lasp2_nomask_fwd")


def lasp2_nomask_bwd(p: Problem, Q, K, V, dO, S, dQ, dK, dV, workspace, stream=None):
    for n, t in (('Q', Q), ('K', K), ('V', V), ('dO', dO), ('dQ', dQ), ('dK', dK), ('dV', dV)):
        _rows(p, t, p.N, n)
    _states(p, S, 'S')
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().lasp2_nomask_bwd(p.ref, _ptr(Q), _ptr(K), _ptr(V), _ptr(dO), _ptr(S), _ptr(dQ),
                                  _ptr(dK), _ptr(dV), _ptr(workspace), ctypes.c_size_t(nbytes),
                                  _stream(stream)), "lasp2_nomask_bwd")


def lasp2_softmax_fwd(p: Problem, Q, K, V, O, LSE, causal=False, stream=None):
    for n, t in (('Q', Q), ('K', K), ('V', V), ('O', O)):
        _rows(p, t, p.N, n)
    _f32(LSE, p.B * p.H * p.N, 'LSE')
    _check(lib().lasp2_softmax_fwd(p.ref, _ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(LSE),
                                   1 if causal else 0, _stream(stream)), "lasp2_softmax_fwd")


def lasp2_softmax_workspace_size(p: Problem) -> int:
    out = ctypes.c_size_t(0)
    _check(lib().lasp2_softmax_workspace_size(p.ref, ctypes.byref(out)), "lasp2_softmax_workspace_size")
    return out.value


def lasp2_softmax_bwd(p: Problem, Q, K, V, O, dO, LSE, dQ, dK, dV, workspace, causal=False, stream=None):
    for n, t in (('Q', Q), ('K', K), ('V', V), ('O', O), ('dO', dO), ('dQ', dQ), ('dK', dK), ('dV', dV)):
        _rows(p, t, p.N, n)
    _f32(LSE, p.B * p.H * p.N, 'LSE')
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().lasp2_softmax_bwd(p.ref, _ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(dO), _ptr(LSE),
                                   _ptr(dQ), _ptr(dK), _ptr(dV), _ptr(workspace), ctypes.c_size_t(nbytes),
                                   1 if causal else 0, _stream(stream)), "lasp2_softmax_bwd")


def lasp2_softmax_fwd_share(p: Problem, q_begin, q_len, Q_t, K, V, O_t, LSE_t, causal=False, stream=None):
    _rows(p, Q_t, q_len, 'Q_t'); _rows(p, O_t, q_len, 'O_t'); _rows(p, K, p.N, 'K'); _rows(p, V, p.N, 'V')
    _f32(LSE_t, p.B * p.H * q_len, 'LSE_t')
    _check(lib().lasp2_softmax_fwd_share(p.ref, ctypes.c_int64(q_begin), ctypes.c_int64(q_len), _ptr(Q_t),
                                         _ptr(K), _ptr(V), _ptr(O_t), _ptr(LSE_t), 1 if causal else 0,
                                         _stream(stream)), "lasp2_softmax_fwd_share")


def lasp2_softmax_share_workspace_size(p: Problem, q_len) -> int:
    out = ctypes.c_size_t(0)
    _check(lib().lasp2_softmax_share_workspace_size(p.ref, ctypes.c_int64(q_len), ctypes.byref(out)),
           "lasp2_softmax_share_workspace_size")
    return out.value


def lasp2_softmax_bwd_share(p: Problem, q_begin, q_len, Q_t, K, V, O_t, dO_t, LSE_t, dQ_t, dK, dV, workspace,
                            causal=False, stream=None):
    for n, t in (('Q_t', Q_t), ('O_t', O_t), ('dO_t', dO_t), ('dQ_t', dQ_t)):
        _rows(p, t, q_len, n)
    for n, t in (('K', K), ('V', V), ('dK', dK), ('dV', dV)):
        _rows(p, t, p.N, n)
    _f32(LSE_t, p.B * p.H * q_len, 'LSE_t')
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().lasp2_softmax_bwd_share(p.ref, ctypes.c_int64(q_begin), ctypes.c_int64(q_len), _ptr(Q_t),
                                         _ptr(K), _ptr(V), _ptr(O_t), _ptr(dO_t), _ptr(LSE_t), _ptr(dQ_t),
                                         _ptr(dK), _ptr(dV), _ptr(workspace), ctypes.c_size_t(nbytes),
                                         1 if causal else 0, _stream(stream)), "lasp2_softmax_bwd_share")


def alloc_states(p: Problem, device="cuda"):
    """fp32 [B,H,T_s,d,d] state array (device memory from torch)."""
    return torch.empty((p.B, p.H, lasp2_num_slots(p), p.d, p.d), dtype=torch.float32, device=device)


def alloc_workspace(p: Problem, device="cuda"):
    """Scratch for lasp2_attn_bwd / lasp2_nomask_bwd: lasp2_workspace_size(p) bytes as a flat fp32 array
    (the state array first, then the backward's pacing counters)."""
    return torch.empty(lasp2_workspace_size(p) // 4, dtype=torch.float32, device=device)


def workspace_states(p: Problem, ws):
    """The fp32 [B,H,T_s,d,d] state array at the head of a workspace."""
    T_s = lasp2_num_slots(p)
    return ws[:p.B * p.H * T_s * p.d * p.d].view(p.B, p.H, T_s, p.d, p.d)


def forward(p: Problem, Q, K, V, stream=None):
    """chunk_states -> state_prefix (in place) -> attn_fwd.  Returns (O, P)."""
    P = alloc_states(p, Q.device)
    O = torch.empty_like(Q)
    lasp2_chunk_states(p, K, V, P, stream)
    lasp2_state_prefix(p, P, P, False, stream)
    lasp2_attn_fwd(p, Q, K, V, P, O, stream)
    return O, P


def backward(p: Problem, Q, K, V, dO, P, stream=None):
    """attn_bwd with a freshly allocated workspace.  Returns (dQ, dK, dV, the workspace's state array)."""
    ws = alloc_workspace(p, Q.device)
    dQ, dK, dV = torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V)
    lasp2_attn_bwd(p, Q, K, V, dO, P, dQ, dK, dV, ws, stream)
    return dQ, dK, dV, workspace_states(p, ws)


def nomask_forward(p: Problem, Q, K, V, stream=None):
    """chunk_states -> state_total (in place) -> nomask_fwd.  Returns (O, S)."""
    S = alloc_states(p, Q.device)
    O = torch.empty_like(Q)
    lasp2_chunk_states(p, K, V, S, stream)
    lasp2_state_total(p, S, S, stream)
    lasp2_nomask_fwd(p, Q, S, O, stream)
    return O, S


def nomask_backward(p: Problem, Q, K, V, dO, S, stream=None):
    """nomask_bwd with a freshly allocated workspace.  Returns (dQ, dK, dV, the workspace's state array)."""
    ws = alloc_workspace(p, Q.device)
    dQ, dK, dV = torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V)
    lasp2_nomask_bwd(p, Q, K, V, dO, S, dQ, dK, dV, ws, stream)
    return dQ, dK, dV, workspace_states(p, ws)
