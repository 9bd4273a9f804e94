"""GPU parity of the masked entry points with scalar decay (mask entries lam^(i-j), one factor
per head) against the CPU oracle's decayed definition on seeded inputs (every element enters;
the bar is the relative L2 error of the whole tensor and its maximum over 256-row blocks):
fp32 and bf16 storage, several chunks and slots, ragged tails, packed documents, and the
lam = 1 case, which must reproduce the undecayed path bit for bit."""
import numpy as np
import pytest

from paper_2502_07563_amd import synth
from tests.util import (TOL, TOL_STATE, assert_close_blocks, host_inputs, rel_l2, slot_partition, to_device,
                        to_host)

pytestmark = pytest.mark.gpu


def _lams(H, seed):
    """Per-head factors in the range of the Retention / Lightning Attention schedules, plus a
    strongly decaying head and an undecayed one."""
    base = 1.0 - 2.0 ** (-5.0 - np.arange(H))
    extra = np.array([0.5, 1.0, 0.9])
    lam = np.where(np.arange(H) % 3 == 0, base, extra[np.arange(H) % 3])
    return lam.astype(np.float32)


def _run(oracle, B, H, N, d, C, L, dtype, seed, cu=None, lam=None, check_suffix_states=True):
    import torch
    from paper_2502_07563_amd import binding as bd

    G = B * H
    lam = _lams(H, seed) if lam is None else np.asarray(lam, dtype=np.float32)
    lam_g = np.tile(lam.astype(np.float64), B)          # group g = b*H + h
    x = host_inputs(seed, G, N, d, dtype)
    p = bd.Problem(B, H, N, d, C, L, dtype, cu, decay=lam)
    bounds, first = slot_partition(N, L if L else C, cu)
    Q, K, V, dO = (to_device(x[n], B, H, dtype) for n in ("Q", "K", "V", "dO"))
    M = bd.alloc_states(p)
    P = torch.empty_like(M)
    O = torch.full_like(Q, float("nan"))
    bd.lasp2_chunk_states(p, K, V, M)
    bd.lasp2_state_prefix(p, M, P, False)
    bd.lasp2_attn_fwd(p, Q, K, V, P, O)
    dQ, dK, dV = (torch.full_like(Q, float("nan")) for _ in range(3))
    ws_all = bd.alloc_workspace(p)
    ws = bd.workspace_states(p, ws_all)
    bd.lasp2_attn_bwd(p, Q, K, V, dO, P, dQ, dK, dV, ws_all)
    torch.cuda.synchronize()

    x64 = {k: v.astype(np.float64) for k, v in x.items()}
    errs = {}
    M_ref = oracle.chunk_states_decay(x64["K"], x64["V"], bounds, lam_g)
    P_ref = oracle.state_prefix_decay(M_ref, bounds, lam_g, first)
    dP_ref = oracle.state_prefix_decay(oracle.chunk_states_decay(x64["Q"], x64["dO"], bounds, lam_g, anchor_start=True),
                                       bounds, lam_g, first, reverse=True)
    errs["M"] = rel_l2(to_host(M), M_ref)
    errs["P"] = rel_l2(to_host(P), P_ref)
    # the workspace holds the exclusive suffix afterwards, unless every document is a single slot:
    # all suffixes are then zero and the library does not touch the workspace
    # (and with several slots per walk the suffix states are per walk, not per slot)
    lone = len(first) == (1 if cu is None else len(cu) - 1)
    per_slot = check_suffix_states and bd.lasp2_walk_slots(p, backward=True) == 1
    errs["dP"] = 0.0 if lone or not per_slot else rel_l2(to_host(ws), dP_ref)
    refs = (oracle.fwd_def_decay(x64["Q"], x64["K"], x64["V"], lam_g, cu),
            *oracle.bwd_def_decay(x64["Q"], x64["K"], x64["V"], x64["dO"], lam_g, cu))
    for name, got, ref in zip(("O", "dQ", "dK", "dV"), (O, dQ, dK, dV), refs):
        errs[name] = rel_l2(to_host(got), ref)
    print({k: f"{v:.2e}" for k, v in errs.items()}, flush=True)
    # The MFMA kernels (bf16, d = 128, every factor >= 0.35) round the weighted rows lam^e k to
    # bf16 before the product, so their states carry bf16 rounding; the plain kernels weight in fp32.
    mfma = dtype == "bf16" and d == 128 and float(lam.min()) >= 0.35
    assert max(errs["M"], errs["P"], errs["dP"]) <= (TOL["bf16"] if mfma else TOL_STATE), errs
    for name, got, ref in zip(("O", "dQ", "dK", "dV"), (O, dQ, dK, dV), refs):
        assert_close_blocks(name, to_host(got), ref, TOL[dtype])
    return dict(O=O, dQ=dQ, dK=dK, dV=dV, P=P)


@pytest.mark.parametrize("N,d,C,L", [(1024, 64, 128, 0), (1000, 32, 128, 256), (777, 16, 50, 150),
                                     (5, 16, 1, 2), (1, 16, 8, 0), (130, 128, 64, 128)])
def test_fp32_shapes(oracle, N, d, C, L):
    _run(oracle, 2, 3, N, d, C, L, "f32", seed=90 + N)


@pytest.mark.parametrize("N,d,C,L", [(1024, 128, 256, 512), (900, 64, 128, 256), (300, 128, 64, 0),
                                     (2304, 128, 256, 1024), (1900, 128, 256, 512), (200, 128, 256, 0),
                                     (777, 128, 50, 150), (67, 128, 1, 3),
                                     # last slot = one full 256-row chunk + 150 tokens (three blocks, ends
                                     # inside the second half) / + 40 tokens (a single ragged block): the
                                     # backward walk starts with that chunk
                                     (2454, 128, 256, 1024), (2344, 128, 256, 1024)])
def test_bf16_shapes(oracle, N, d, C, L):
    _run(oracle, 1, 3, N, d, C, L, "bf16", seed=110 + N)


def test_bf16_d128_strong_decay_takes_the_plain_kernels(oracle):
    """A factor below 0.35 is outside the range the MFMA decay kernels are built for."""
    _run(oracle, 1, 3, 700, 128, 128, 256, "bf16", seed=115, lam=[0.2, 0.99, 0.05])


@pytest.mark.parametrize("dtype,d,C,L", [("f32", 32, 64, 128), ("bf16", 128, 128, 256), ("bf16", 128, 256, 1024)])
def test_packed_documents(oracle, dtype, d, C, L):
    cu = synth.doc_offsets(6, 1536, 7, mean_len=1536 / 7, min_len=1)
    _run(oracle, 1, 3, 1536, d, C, L, dtype, seed=120, cu=cu)


@pytest.mark.parametrize("seed", range(8))
def test_random_shapes_bf16_d128(oracle, seed):
    """Seeded random sizes (the draws of tests/test_gpu_parity.py) with decay; one batch row, since the
    decayed oracle is the slow one."""
    from tests.test_gpu_parity import _random_case
    _, H, N, C, L, cu = _random_case(50 + seed)
    print((H, N, C, L, None if cu is None else cu.tolist()), flush=True)
    _run(oracle, 1, H, N, 128, C, L, "bf16", seed=300 + seed, cu=cu)


@pytest.mark.parametrize("ws", [2, 3, 16])
def test_walks_of_several_slots(oracle, monkeypatch, ws):
    """The attention kernels walk `ws` of the caller's slots per workgroup (forced here; by itself the
    library does so only for launches of more walks than the device runs at once): the prefix array is
    then read at every ws-th slot of a document only and the backward's suffix states are per walk."""
    monkeypatch.setenv("LASP2_WALK_SLOTS", str(ws))
    _run(oracle, 1, 3, 2454, 128, 256, 256, "bf16", seed=140 + ws, check_suffix_states=False)
    _run(oracle, 1, 3, 700, 128, 64, 64, "bf16", seed=150 + ws, check_suffix_states=False)     # 128-row kernel by itself
    cu = synth.doc_offsets(6, 1536, 7, mean_len=1536 / 7, min_len=1)
    _run(oracle, 1, 3, 1536, 128, 128, 128, "bf16", seed=160 + ws, cu=cu, check_suffix_states=False)


def test_all_ones_decay_is_bit_identical_to_no_decay(oracle):
    import torch
    from paper_2502_07563_amd import binding as bd
    B, H, N, d, C, L = 1, 2, 600, 32, 64, 128
    with_decay = _run(oracle, B, H, N, d, C, L, "f32", seed=130, lam=np.ones(H))
    x = host_inputs(130, B * H, N, d, "f32")
    p = bd.Problem(B, H, N, d, C, L, "f32")
    Q, K, V, dO = (to_device(x[n], B, H, "f32") for n in ("Q", "K", "V", "dO"))
    O, P = bd.forward(p, Q, K, V)
    dQ, dK, dV, _ = bd.backward(p, Q, K, V, dO, P)
    torch.cuda.synchronize()
    for name, t in (("O", O), ("dQ", dQ), ("dK", dK), ("dV", dV), ("P", P)):
        assert torch.equal(t, with_decay[name]), name
