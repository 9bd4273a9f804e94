"""Helpers for the GPU parity tests: the slot rule restated independently of the library,
input staging, and the error metric."""
import numpy as np

from paper_2502_07563_amd import synth

TOL = {"f32": 1e-4, "bf16": 2e-2}   # rel. L2 bound on O, dQ, dK, dV (inputs fp32 / bf16, fp32 accumulate)
TOL_STATE = 1e-4                    # fp32 states from exactly representable products, fp32 accumulation


def slot_partition(N, L, cu=None):
    """Token bounds of the state slots and the flag 'slot opens a document'."""
    cu = [0, N] if cu is None else list(cu)
    bounds, first = [0], []
    for a, b in zip(cu[:-1], cu[1:]):
        pos = a
        while pos < b:
            first.append(1 if pos == a else 0)
            pos = min(pos + L, b)
            bounds.append(pos)
    return np.array(bounds, dtype=np.int64), np.array(first, dtype=np.int32)


def rel_l2(got, want):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    return float(np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-300))


def host_inputs(seed, G, N, d, dtype, names=("Q", "K", "V", "dO")):
    """fp32 host tensors [G,N,d] whose values are exactly representable in `dtype`."""
    return {n: synth.gen_tensor(seed, n, G, N, d, dtype) for n in names}


def to_device(x, B, H, dtype):
    import torch
    t = torch.from_numpy(x).reshape(B, H, x.shape[1], x.shape[2])
    t = t.to("cuda")
    return t.to(torch.bfloat16) if dtype == "bf16" else t


def to_host(t):
    G = t.shape[0] * t.shape[1]
    return t.float().cpu().numpy().reshape((G,) + tuple(t.shape[2:])).astype(np.float64)
