"""lasp2_attn_bwd_noalloc (the backward for callers that cannot allocate or hand over a workspace:
its dM states live in a fixed device array inside the library) against lasp2_attn_bwd on the same
inputs, through the C ABI: two calls in a row on the one GPU, the second with a smaller input, so
that whatever the first call left in the shared array must not leak into the second."""
import ctypes

import numpy as np
import pytest

from tests.util import TOL, assert_close_blocks, host_inputs, to_device, to_host

pytestmark = pytest.mark.gpu


def _both(oracle, B, H, N, C, L, seed, cu=None):
    import torch
    from paper_2502_07563_amd import binding as bd
    d, dtype = 128, "bf16"
    p = bd.Problem(B, H, N, d, C, L, dtype, cu)
    x = host_inputs(seed, B * H, N, d, dtype)
    Q, K, V, dO = (to_device(x[n], B, H, dtype) for n in ("Q", "K", "V", "dO"))
    _, P = bd.forward(p, Q, K, V)
    want = [torch.full_like(Q, float("nan")) for _ in range(3)]
    ws = torch.full((bd.lasp2_workspace_size(p) // 4,), float("nan"), dtype=torch.float32, device="cuda")
    bd.lasp2_attn_bwd(p, Q, K, V, dO, P, *want, ws)
    got = [torch.full_like(Q, float("nan")) for _ in range(3)]
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    bd.lasp2_attn_bwd_noalloc(p, Q, K, V, dO, P, *got)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    x64 = {k: v.astype(np.float64) for k, v in x.items()}
    refs = oracle.bwd_def(x64["Q"], x64["K"], x64["V"], x64["dO"], cu)
    for name, g, w, r in zip(("dQ", "dK", "dV"), got, want, refs):
        # against the existing entry point: same kernels, same order of operations
        assert_close_blocks(name + " vs lasp2_attn_bwd", to_host(g), to_host(w), TOL[dtype])
        assert torch.equal(g, w), name
        # and against the oracle itself
        assert_close_blocks(name + " vs oracle", to_host(g), r, TOL[dtype])


def test_two_calls_in_a_row_second_one_smaller(oracle):
    _both(oracle, 1, 3, 2304, 256, 512, seed=91)            # 3 heads x 5 slots (the last one ragged)
    _both(oracle, 1, 2, 700, 256, 256, seed=92)             # fewer heads, fewer and shorter slots
    cu = np.array([0, 300, 301, 1000, 1536], dtype=np.int32)
    _both(oracle, 1, 2, 1536, 128, 256, seed=93, cu=cu)     # packed documents


def test_size_limit_is_an_error_before_any_launch():
    import torch
    from paper_2502_07563_amd import binding as bd
    # 1025 slot states of 64 KiB: one more than the array holds
    p = bd.Problem(1, 1, 1025 * 256, 128, 256, 256, "bf16")
    assert bd.lasp2_workspace_size(p) > bd.NOALLOC_SCRATCH_BYTES
    fake = ctypes.c_void_p(0x1000)
    rc = bd.lib().lasp2_attn_bwd_noalloc(p.ref, fake, fake, fake, fake, fake, fake, fake, fake, None)
    assert rc == -5
