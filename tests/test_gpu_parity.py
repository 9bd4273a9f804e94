"""GPU parity: every entry point of the C ABI against the CPU oracle on the same seeded inputs,
every element of every output entering the comparison.  The bar for O, dQ, dK, dV is the
tolerance on the relative L2 error of the whole tensor AND on its maximum over blocks of 256
consecutive rows of each (batch, head) (tests/util.py: assert_close_blocks), so that a fault
confined to a few rows of an early chunk fails.  Sizes here are ones the brute-force oracle
finishes in seconds; they span several chunks, several slots and ragged tails."""
import numpy as np
import pytest

from tests.util import (TOL, TOL_STATE, assert_close_blocks, host_inputs, rel_l2, slot_partition, to_device,
                        to_host)

pytestmark = pytest.mark.gpu


def _run_all(oracle, B, H, N, d, C, L, dtype, seed, cu=None, check_bwd=True):
    import torch
    from paper_2502_07563_amd import binding as bd

    G = B * H
    x = host_inputs(seed, G, N, d, dtype)
    p = bd.Problem(B, H, N, d, C, L, dtype, cu)
    Leff = L if L else C
    bounds, first = slot_partition(N, Leff, cu)
    assert bd.lasp2_num_slots(p) == len(first)

    Q, K, V, dO = (to_device(x[n], B, H, dtype) for n in ("Q", "K", "V", "dO"))
    M = bd.alloc_states(p)
    P = torch.empty_like(M)
    O = torch.full_like(Q, float("nan"))
    bd.lasp2_chunk_states(p, K, V, M)
    bd.lasp2_state_prefix(p, M, P, False)
    bd.lasp2_attn_fwd(p, Q, K, V, P, O)
    torch.cuda.synchronize()

    x64 = {k: v.astype(np.float64) for k, v in x.items()}
    errs = {}
    M_ref = oracle.chunk_states(x64["K"], x64["V"], bounds)
    P_ref = oracle.state_prefix(M_ref, first, reverse=False)
    errs["M"] = rel_l2(to_host(M), M_ref)
    errs["P"] = rel_l2(to_host(P), P_ref)
    O_ref = oracle.fwd_def(x64["Q"], x64["K"], x64["V"], cu)
    assert errs["M"] <= TOL_STATE and errs["P"] <= TOL_STATE, errs
    errs["O"], errs["O_blk"] = assert_close_blocks("O", to_host(O), O_ref, TOL[dtype])

    if check_bwd:
        dQ, dK, dV = (torch.full_like(Q, float("nan")) for _ in range(3))
        ws = bd.alloc_workspace(p)
        bd.lasp2_attn_bwd(p, Q, K, V, dO, P, dQ, dK, dV, ws)
        torch.cuda.synchronize()
        dQ_ref, dK_ref, dV_ref = oracle.bwd_def(x64["Q"], x64["K"], x64["V"], x64["dO"], cu)
        # dM_t = Q_t^T dO_t and its suffix combine through the public entry points
        dP = torch.empty_like(M)
        bd.lasp2_chunk_states(p, Q, dO, dP)
        bd.lasp2_state_prefix(p, dP, dP, True)
        torch.cuda.synchronize()
        dP_ref = oracle.state_prefix(oracle.chunk_states(x64["Q"], x64["dO"], bounds), first, reverse=True)
        errs["dP"] = rel_l2(to_host(dP), dP_ref)
        assert errs["dP"] <= TOL_STATE, errs
        for k, got, ref in (("dQ", dQ, dQ_ref), ("dK", dK, dK_ref), ("dV", dV, dV_ref)):
            errs[k], errs[k + "_blk"] = assert_close_blocks(k, to_host(got), ref, TOL[dtype])
    print({k: f"{v:.2e}" for k, v in errs.items()}, flush=True)
    return errs


def test_cfg1_fp32_forward(oracle):
    """Config 1 exactly: fp32, B=1, H=2, N=1024, d=64, C=128 (8 chunks), seed 0."""
    _run_all(oracle, 1, 2, 1024, 64, 128, 0, "f32", seed=0, check_bwd=True)


@pytest.mark.parametrize("N,d,C,L", [(1000, 32, 128, 256), (777, 16, 50, 150), (300, 64, 512, 0),
                                     (5, 16, 1, 2), (1, 16, 8, 0), (130, 128, 64, 128)])
def test_fp32_shapes(oracle, N, d, C, L):
    _run_all(oracle, 2, 2, N, d, C, L, "f32", seed=10 + N)


@pytest.mark.parametrize("N,C,L", [(2048, 256, 0), (2304, 256, 1024), (1900, 256, 512), (200, 256, 0),
                                   (1536, 128, 512), (1000, 64, 256), (777, 50, 150), (640, 512, 0),
                                   (67, 1, 3), (1024, 32, 128)])
def test_bf16_d128(oracle, N, C, L):
    """The MFMA path's shapes (bf16, d=128): several chunks per slot, ragged tails."""
    _run_all(oracle, 1, 3, N, 128, C, L, "bf16", seed=20 + N)


def test_bf16_generic_shapes(oracle):
    _run_all(oracle, 1, 2, 600, 64, 128, 256, "bf16", seed=31)
    _run_all(oracle, 1, 2, 333, 128, 96, 192, "bf16", seed=32)


@pytest.mark.parametrize("dtype,d,C,L", [("bf16", 128, 256, 0), ("bf16", 128, 256, 512),
                                         ("f32", 32, 64, 128)])
def test_packed_documents(oracle, dtype, d, C, L):
    """Packed batch: boundaries not aligned to C, documents shorter than C and of length 1."""
    lens = [64, 700, 1, 255, 256, 257, 1467, 3]
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    _run_all(oracle, 1, 2, int(cu[-1]), d, C, L, dtype, seed=40, cu=cu)


@pytest.mark.parametrize("dtype,d,C,L,ndocs", [("bf16", 128, 64, 64, 33), ("bf16", 128, 128, 256, 150),
                                               ("f32", 32, 32, 64, 97)])
def test_many_documents(oracle, dtype, d, C, L, ndocs):
    """More documents than the kernels keep marks for (32): the slot -> document search starts from
    a mark and walks on; lengths from 1 token to a few slots, so documents of one and of several
    slots alternate."""
    rng = np.random.default_rng(1000 + ndocs)
    lens = rng.integers(1, 3 * L + 2, size=ndocs)
    lens[::7] = 1
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    _run_all(oracle, 1, 2, int(cu[-1]), d, C, L, dtype, seed=45, cu=cu)


@pytest.mark.parametrize("ws", [2, 3, 5, 64])
def test_walks_of_several_slots(oracle, monkeypatch, ws):
    """The bf16 d = 128 attention kernels walk `ws` of the caller's slots per workgroup (forced here; by
    itself the library does so only for launches of more walks than the device runs at once).  The
    prefix array is then read at every ws-th slot of a document only, the backward builds its suffix
    states per walk, and nothing else changes: ragged tails, more than one head and batch row, slots
    shorter than the 128-row kernel's limit, packed documents of one and of many slots."""
    import torch
    from paper_2502_07563_amd import binding as bd
    monkeypatch.setenv("LASP2_WALK_SLOTS", str(ws))
    p = bd.Problem(2, 2, 2304 + 77, 128, 256, 256, "bf16")
    assert bd.lasp2_walk_slots(p) == ws and bd.lasp2_walk_slots(p, backward=True) == ws
    _run_all(oracle, 2, 2, 2304 + 77, 128, 256, 256, "bf16", seed=70 + ws)
    _run_all(oracle, 1, 3, 1000, 128, 64, 64, "bf16", seed=80 + ws)
    _run_all(oracle, 1, 2, 1500, 128, 50, 100, "bf16", seed=90 + ws)
    lens = [64, 700, 1, 255, 256, 257, 1467, 3, 2048]
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    _run_all(oracle, 1, 2, int(cu[-1]), 128, 128, 128, "bf16", seed=100 + ws, cu=cu)
    rng = np.random.default_rng(ws)
    lens = rng.integers(1, 400, size=70)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    _run_all(oracle, 1, 2, int(cu[-1]), 128, 64, 64, "bf16", seed=110 + ws, cu=cu)
    # the fp32 path keeps one walk per slot whatever the variable says
    p32 = bd.Problem(1, 2, 1024, 64, 128, 128, "f32")
    assert bd.lasp2_walk_slots(p32) == 1
    _run_all(oracle, 1, 2, 1024, 64, 128, 128, "f32", seed=120 + ws)


@pytest.mark.parametrize("decay", [False, True])
def test_slot_lengths_around_block_and_half_boundaries(oracle, decay):
    """One slot per document, lengths on both sides of every 64-token block boundary of the 256-row
    tiling (and of its 128-row halves) up to three chunks; each document's outputs and gradients are
    compared on their own, so that a short document cannot hide behind a long one.  The kernel walks
    every chunk as four blocks: the ones past a slot's end are zeroed, not loaded, and with decay the
    backward walk meets them first."""
    import torch
    from paper_2502_07563_amd import binding as bd
    from paper_2502_07563_amd import synth

    lens = [129, 130, 191, 192, 193, 255, 256, 257, 319, 320, 321, 383, 384, 385, 447, 448, 449,
            511, 512, 513, 575, 577, 640, 641, 705, 767, 768]
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    B, H, N, d, C, L, dtype = 1, 2, int(cu[-1]), 128, 256, 1024, "bf16"
    lam = np.array([1.0 - 2.0 ** -6, 0.9], dtype=np.float32) if decay else None
    x = host_inputs(47, B * H, N, d, dtype)
    p = bd.Problem(B, H, N, d, C, L, dtype, cu, decay=lam) if decay else bd.Problem(B, H, N, d, C, L, dtype, cu)
    assert bd.lasp2_num_slots(p) == len(lens)
    Q, K, V, dO = (to_device(x[n], B, H, dtype) for n in ("Q", "K", "V", "dO"))
    M = bd.alloc_states(p)
    P = torch.empty_like(M)
    O, dQ, dK, dV = (torch.full_like(Q, float("nan")) for _ in range(4))
    bd.lasp2_chunk_states(p, K, V, M)
    bd.lasp2_state_prefix(p, M, P, False)
    bd.lasp2_attn_fwd(p, Q, K, V, P, O)
    bd.lasp2_attn_bwd(p, Q, K, V, dO, P, dQ, dK, dV, bd.alloc_workspace(p))
    torch.cuda.synchronize()
    x64 = {k: v.astype(np.float64) for k, v in x.items()}
    if decay:
        lam_g = np.tile(lam.astype(np.float64), B)
        refs = (oracle.fwd_def_decay(x64["Q"], x64["K"], x64["V"], lam_g, cu),
                *oracle.bwd_def_decay(x64["Q"], x64["K"], x64["V"], x64["dO"], lam_g, cu))
    else:
        refs = (oracle.fwd_def(x64["Q"], x64["K"], x64["V"], cu),
                *oracle.bwd_def(x64["Q"], x64["K"], x64["V"], x64["dO"], cu))
    worst = {}
    for name, got, ref in zip(("O", "dQ", "dK", "dV"), (O, dQ, dK, dV), refs):
        got = to_host(got)
        assert np.isfinite(got).all(), name
        for i, n in enumerate(lens):
            a, b = int(cu[i]), int(cu[i + 1])
            e = rel_l2(got[:, a:b], ref[:, a:b])
            worst[name] = max(worst.get(name, 0.0), e)
            assert e <= TOL[dtype], (name, n, e)
    print({k: f"{v:.2e}" for k, v in worst.items()}, flush=True)


def _random_case(seed):
    """A seeded draw of sizes for the bf16, d = 128 path: sequence length, chunk length, slot length,
    heads, and optionally a packing into documents."""
    rng = np.random.default_rng(1000 + seed)
    B, H = int(rng.integers(1, 3)), int(rng.integers(1, 4))
    N = int(rng.choice([rng.integers(1, 300), rng.integers(300, 1200), rng.integers(1200, 2500)]))
    C = int(rng.choice([32, 64, 128, 256, 512]))
    L = int(rng.choice([0, C, 2 * C, 4 * C, 8 * C]))
    cu = None
    if B == 1 and N > 8 and rng.integers(0, 2):
        cuts = np.sort(rng.choice(np.arange(1, N), size=int(rng.integers(1, 7)), replace=False))
        cu = np.concatenate([[0], cuts, [N]]).astype(np.int32)
    return B, H, N, C, L, cu


@pytest.mark.parametrize("seed", range(10))
def test_random_shapes_bf16_d128(oracle, seed):
    B, H, N, C, L, cu = _random_case(seed)
    print((B, H, N, C, L, None if cu is None else cu.tolist()), flush=True)
    _run_all(oracle, B, H, N, 128, C, L, "bf16", seed=200 + seed, cu=cu)


@pytest.mark.parametrize("seed", range(10, 20))
def test_random_shapes_and_walk_lengths_bf16_d128(oracle, monkeypatch, seed):
    """The same draws of sizes with a drawn number of slots per walk forced on the attention kernels."""
    B, H, N, C, L, cu = _random_case(seed)
    ws = int(np.random.default_rng(seed).choice([2, 3, 4, 7, 32]))
    print((B, H, N, C, L, None if cu is None else cu.tolist(), ws), flush=True)
    monkeypatch.setenv("LASP2_WALK_SLOTS", str(ws))
    _run_all(oracle, B, H, N, 128, C, L, "bf16", seed=220 + seed, cu=cu)


def test_prefix_in_place_and_deterministic(oracle):
    import torch
    from paper_2502_07563_amd import binding as bd
    p = bd.Problem(1, 2, 4096, 128, 256, 0, "bf16")
    x = host_inputs(50, 2, 4096, 128, "bf16")
    Q, K, V, dO = (to_device(x[n], 1, 2, "bf16") for n in ("Q", "K", "V", "dO"))
    runs = []
    for _ in range(2):
        M = bd.alloc_states(p)
        bd.lasp2_chunk_states(p, K, V, M)
        P = torch.empty_like(M)
        bd.lasp2_state_prefix(p, M, P, False)
        bd.lasp2_state_prefix(p, M, M, False)          # in place
        torch.cuda.synchronize()
        assert torch.equal(M, P)
        O = torch.empty_like(Q)
        bd.lasp2_attn_fwd(p, Q, K, V, P, O)
        dQ, dK, dV, dP = bd.backward(p, Q, K, V, dO, P)
        torch.cuda.synchronize()
        runs.append((P, O, dQ, dK, dV, dP))
    for a, b in zip(*runs):
        assert torch.equal(a, b), "not run-to-run bit-identical"


def test_result_does_not_depend_on_C_or_L(oracle):
    """Chunk length and slot length change the schedule, not the result (within tolerance)."""
    import torch
    from paper_2502_07563_amd import binding as bd
    N = 3072
    x = host_inputs(60, 2, N, 128, "bf16")
    Q, K, V, dO = (to_device(x[n], 1, 2, "bf16") for n in ("Q", "K", "V", "dO"))
    ref = None
    for C, L in ((256, 0), (256, 1024), (256, 3072), (128, 512), (64, 64)):
        p = bd.Problem(1, 2, N, 128, C, L, "bf16")
        O, P = bd.forward(p, Q, K, V)
        dQ, dK, dV, _ = bd.backward(p, Q, K, V, dO, P)
        torch.cuda.synchronize()
        got = [to_host(t) for t in (O, dQ, dK, dV)]
        if ref is None:
            ref = got
        else:
            for a, b in zip(got, ref):
                assert rel_l2(a, b) <= TOL["bf16"]


def test_runs_on_the_callers_stream(oracle):
    """Work is enqueued on the stream handed in: results on a side stream match the default stream."""
    import torch
    from paper_2502_07563_amd import binding as bd
    p = bd.Problem(1, 2, 2048, 128, 256, 512, "bf16")
    x = host_inputs(70, 2, 2048, 128, "bf16")
    Q, K, V, dO = (to_device(x[n], 1, 2, "bf16") for n in ("Q", "K", "V", "dO"))
    O0, P0 = bd.forward(p, Q, K, V)
    g0 = bd.backward(p, Q, K, V, dO, P0)[:3]
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        O1, P1 = bd.forward(p, Q, K, V, stream=side)
        g1 = bd.backward(p, Q, K, V, dO, P1, stream=side)[:3]
    side.synchronize()
    assert torch.equal(O0, O1) and torch.equal(P0, P1)
    for a, b in zip(g0, g1):
        assert torch.equal(a, b)


def test_maximum_number_of_groups(oracle):
    """B * H = 65 535 (the limit the descriptor check allows) short sequences: one workgroup per group in
    every launch, the last groups at the far end of the one-dimensional grids."""
    _run_all(oracle, 257, 255, 40, 128, 32, 32, "bf16", seed=77)


def test_many_slots_not_multiple_of_eight(oracle):
    """Slot counts that do not fill the last group of eight workgroups of a launch."""
    _run_all(oracle, 1, 1, 256 * 11 + 70, 128, 256, 256, "bf16", seed=71)
    _run_all(oracle, 2, 1, 256 * 3, 128, 256, 256, "bf16", seed=72)


@pytest.mark.parametrize("dtype,d,C,N,decay", [("bf16", 128, 256, 1900, False), ("bf16", 128, 256, 1900, True),
                                               ("bf16", 128, 64, 100, False), ("f32", 32, 64, 700, False),
                                               ("f32", 32, 64, 700, True)])
@pytest.mark.parametrize("packed", [False, True])
def test_serial_carry_schedule_without_state_arrays(oracle, dtype, d, C, N, decay, packed):
    """One slot per sequence (document): lasp2_attn_fwd and lasp2_attn_bwd with P = NULL and no
    chunk_states / state_prefix calls at all, one pass that carries the state from chunk to chunk,
    against the definition.  The backward gets a workspace only where the kernels still want one
    (matrix cores without decay)."""
    import torch
    from paper_2502_07563_amd import binding as bd
    B, H = (1, 3) if packed else (2, 2)
    cu = None
    if packed:
        lens = [N // 5, 1, N // 3, 37] if N > 200 else [N // 4, 1, N // 2, 7]
        lens.append(N - sum(lens))
        cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    longest = N if cu is None else int(np.diff(cu).max())
    L = -(-longest // C) * C
    lam = np.array([0.97, 0.5, 1.0][:H], dtype=np.float32) if decay else None
    p = bd.Problem(B, H, N, d, C, L, dtype, cu, decay=lam)
    assert bd.lasp2_num_slots(p) == (1 if cu is None else len(cu) - 1)
    x = host_inputs(75, B * H, N, d, dtype)
    Q, K, V, dO = (to_device(x[n], B, H, dtype) for n in ("Q", "K", "V", "dO"))
    O, dQ, dK, dV = (torch.full_like(Q, float("nan")) for _ in range(4))
    bd.lasp2_attn_fwd(p, Q, K, V, None, O)
    needs_ws = dtype == "bf16" and d == 128 and not decay
    ws = torch.full((bd.lasp2_workspace_size(p) // 4,), float("nan"), dtype=torch.float32, device="cuda") if needs_ws else None
    bd.lasp2_attn_bwd(p, Q, K, V, dO, None, dQ, dK, dV, ws)
    torch.cuda.synchronize()
    x64 = {k: v.astype(np.float64) for k, v in x.items()}
    if decay:
        lam_g = np.tile(lam.astype(np.float64), B)
        refs = (oracle.fwd_def_decay(x64["Q"], x64["K"], x64["V"], lam_g, cu),
                *oracle.bwd_def_decay(x64["Q"], x64["K"], x64["V"], x64["dO"], lam_g, cu))
    else:
        refs = (oracle.fwd_def(x64["Q"], x64["K"], x64["V"], cu),
                *oracle.bwd_def(x64["Q"], x64["K"], x64["V"], x64["dO"], cu))
    errs = {}
    for name, got, ref in zip(("O", "dQ", "dK", "dV"), (O, dQ, dK, dV), refs):
        errs[name] = assert_close_blocks(name, to_host(got), ref, TOL[dtype])
    print({k: f"{a:.2e}/{b:.2e}" for k, (a, b) in errs.items()}, flush=True)
