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


def max_block_rel_l2(got, want, block=256):
    """Largest relative L2 error over blocks of `block` consecutive rows: for every group and every
    block, |got - want| over |want| restricted to the block's rows.  got, want: [G, N, d] (or [N, d]).
    A fault confined to a few rows cannot hide in this number the way it can in a whole-tensor
    norm, where rows far along the sequence outweigh the early ones.  Returns (error, group, first
    row of the worst block)."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    if got.ndim == 2:
        got, want = got[None], want[None]
    assert got.shape == want.shape, (got.shape, want.shape)
    if got.shape[1] == 0:
        return 0.0, 0, 0
    diff = got - want
    e2 = np.einsum("gnd,gnd->gn", diff, diff)
    r2 = np.einsum("gnd,gnd->gn", want, want)
    starts = np.arange(0, got.shape[1], block)
    be = np.add.reduceat(e2, starts, axis=1)
    br = np.add.reduceat(r2, starts, axis=1)
    ratio = np.sqrt(be / np.maximum(br, 1e-300))
    ratio = np.where(np.isfinite(ratio), ratio, np.inf)     # NaN left in an output counts as infinite
    g, b = np.unravel_index(int(np.argmax(ratio)), ratio.shape)
    return float(ratio[g, b]), int(g), int(starts[b])


def assert_close_blocks(name, got, want, tol, block=256):
    """The parity bar for O, dQ, dK, dV: the whole-tensor relative L2 error and its maximum over
    blocks of 256 rows both within `tol`.  Returns the two numbers."""
    whole = rel_l2(got, want)
    worst, g, row = max_block_rel_l2(got, want, block)
    assert np.isfinite(np.asarray(got, dtype=np.float64)).all(), f"{name}: non-finite values in the output"
    assert whole <= tol, f"{name}: rel L2 {whole:.3e} > {tol}"
    assert worst <= tol, f"{name}: rows {row}..{row + block - 1} of group {g} off by {worst:.3e} > {tol}"
    return whole, worst


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
