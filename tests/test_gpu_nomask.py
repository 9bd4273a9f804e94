"""GPU parity of the entry points without masking (state total, O = Q M, and the backward)
against the CPU oracle on seeded inputs (every element enters; the bar is the relative L2 error
of the whole tensor and its maximum over 256-row blocks): fp32 and bf16, several slots, ragged
tails, packed documents, in-place totals."""
import numpy as np
import pytest

from paper_2502_07563_amd import synth
from tests.util import (TOL, TOL_STATE, assert_close_blocks, host_inputs, rel_l2, slot_partition, to_device,
                        to_host)

pytestmark = pytest.mark.gpu


def _run(oracle, B, H, N, d, C, L, dtype, seed, cu=None):
    import torch
    from paper_2502_07563_amd import binding as bd

    G = B * H
    x = host_inputs(seed, G, N, d, dtype)
    p = bd.Problem(B, H, N, d, C, L, dtype, cu)
    bounds, first = slot_partition(N, L if L else C, cu)
    Q, K, V, dO = (to_device(x[n], B, H, dtype) for n in ("Q", "K", "V", "dO"))
    M = bd.alloc_states(p)
    S = torch.full_like(M, float("nan"))
    O = torch.full_like(Q, float("nan"))
    bd.lasp2_chunk_states(p, K, V, M)
    bd.lasp2_state_total(p, M, S)            # out of place
    bd.lasp2_nomask_fwd(p, Q, S, O)
    M2 = M.clone()
    bd.lasp2_state_total(p, M2, M2)          # in place
    dQ, dK, dV = (torch.full_like(Q, float("nan")) for _ in range(3))
    ws_all = bd.alloc_workspace(p)
    ws = bd.workspace_states(p, ws_all)
    bd.lasp2_nomask_bwd(p, Q, K, V, dO, S, dQ, dK, dV, ws_all)
    torch.cuda.synchronize()
    assert torch.equal(M2, S)

    x64 = {k: v.astype(np.float64) for k, v in x.items()}
    errs = {}
    S_ref = oracle.state_total(oracle.chunk_states(x64["K"], x64["V"], bounds), first)
    dS_ref = oracle.state_total(oracle.chunk_states(x64["Q"], x64["dO"], bounds), first)
    errs["S"] = rel_l2(to_host(S), S_ref)
    errs["dS"] = rel_l2(to_host(ws), dS_ref)
    refs = (oracle.nomask_fwd_def(x64["Q"], x64["K"], x64["V"], cu),
            *oracle.nomask_bwd_def(x64["Q"], x64["K"], x64["V"], x64["dO"], cu))
    for name, got, ref in zip(("O", "dQ", "dK", "dV"), (O, dQ, dK, dV), refs):
        errs[name] = rel_l2(to_host(got), ref)
    print({k: f"{v:.2e}" for k, v in errs.items()}, flush=True)
    assert errs["S"] <= TOL_STATE and errs["dS"] <= TOL_STATE, errs
    for name, got, ref in zip(("O", "dQ", "dK", "dV"), (O, dQ, dK, dV), refs):
        assert_close_blocks(name, to_host(got), ref, TOL[dtype])
    return errs


@pytest.mark.parametrize("N,d,C,L", [(1024, 64, 128, 0), (1000, 32, 128, 256), (777, 16, 50, 150),
                                     (5, 16, 1, 2), (1, 16, 8, 0), (130, 128, 64, 128)])
def test_fp32_shapes(oracle, N, d, C, L):
    _run(oracle, 2, 2, N, d, C, L, "f32", seed=40 + N)


@pytest.mark.parametrize("N,C,L", [(2048, 256, 0), (2304, 256, 1024), (1900, 256, 512), (200, 256, 0),
                                   (1536, 128, 512), (1000, 64, 256), (777, 50, 150), (640, 512, 0),
                                   (67, 1, 3), (1024, 32, 128)])
def test_bf16_d128(oracle, N, C, L):
    """bf16, d = 128: the MFMA kernels, whatever the chunk length."""
    _run(oracle, 1, 3, N, 128, C, L, "bf16", seed=60 + N)


def test_bf16_other_d(oracle):
    _run(oracle, 2, 2, 900, 64, 128, 256, "bf16", seed=70)


@pytest.mark.parametrize("dtype,d,C,L", [("f32", 32, 64, 128), ("bf16", 128, 256, 512), ("bf16", 128, 128, 128)])
def test_packed_documents(oracle, dtype, d, C, L):
    cu = synth.doc_offsets(5, 2048, 9, mean_len=2048 / 9, min_len=1)
    _run(oracle, 1, 2, 2048, d, C, L, dtype, seed=80, cu=cu)
