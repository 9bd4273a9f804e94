"""The whole layer step (chunk states, prefix, fused forward, backward) recorded once into a HIP graph
and replayed: the library only enqueues kernels on the caller's stream (its pacing counters are cleared
by a fill kernel, not by a memset), so a capture must give, on every replay, exactly what the eager
calls give.  Between the replays the test does eager work of its own (new inputs, poisoned outputs, an
eager run of the same step) and synchronises."""
import numpy as np
import pytest

from tests.util import TOL, assert_close_blocks, host_inputs, to_device, to_host

pytestmark = pytest.mark.gpu


def _step(bd, p, Q, K, V, dO, M, P, O, dQ, dK, dV, ws):
    bd.lasp2_chunk_states(p, K, V, M)
    bd.lasp2_state_prefix(p, M, P)
    bd.lasp2_attn_fwd(p, Q, K, V, P, O)
    bd.lasp2_attn_bwd(p, Q, K, V, dO, P, dQ, dK, dV, ws)


@pytest.mark.parametrize("B,H,N,C,L,cu", [
    (1, 3, 2304, 256, 512, None),                                            # the fused dV/dK walk with pacing
    (2, 2, 640, 128, 128, None),                                             # 128-row kernel, three problems
    (1, 2, 1536, 128, 256, np.array([0, 300, 301, 1000, 1536], np.int32)),   # packed documents
])
def test_graph_replays_equal_the_eager_step(oracle, B, H, N, C, L, cu):
    import torch
    from paper_2502_07563_amd import binding as bd
    d, dtype = 128, "bf16"
    p = bd.Problem(B, H, N, d, C, L, dtype, cu)

    def inputs(seed):
        x = host_inputs(seed, B * H, N, d, dtype)
        return x, [to_device(x[n], B, H, dtype) for n in ("Q", "K", "V", "dO")]

    _, static_in = inputs(400)
    M, P = bd.alloc_states(p), bd.alloc_states(p)
    ws = bd.alloc_workspace(p)
    outs = [torch.empty_like(static_in[0]) for _ in range(4)]            # O, dQ, dK, dV
    eager = [torch.empty_like(static_in[0]) for _ in range(4)]
    M2, P2, ws2 = bd.alloc_states(p), bd.alloc_states(p), bd.alloc_workspace(p)

    # one eager pass first: whatever a kernel's first launch sets up happens outside the capture
    _step(bd, p, *static_in, M, P, *outs, ws)
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):
        _step(bd, p, *static_in, M, P, *outs, ws)
    torch.cuda.synchronize()

    for r, seed in enumerate((401, 402, 403, 404)):
        x, fresh = inputs(seed)
        for s, f in zip(static_in, fresh):
            s.copy_(f)
        for t in outs + eager + [M, P, M2, P2]:
            t.fill_(float("nan"))
        ws.fill_(float("nan")); ws2.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        _step(bd, p, *fresh, M2, P2, *eager, ws2)
        torch.cuda.synchronize()
        for name, g, e in zip(("O", "dQ", "dK", "dV"), outs, eager):
            assert torch.equal(g, e), f"replay {r}: {name} differs from the eager step"
        assert torch.equal(P, P2), f"replay {r}: prefix states differ"
        if r == 0:
            x64 = {k: v.astype(np.float64) for k, v in x.items()}
            want = (oracle.fwd_def(x64["Q"], x64["K"], x64["V"], cu),) + \
                tuple(oracle.bwd_def(x64["Q"], x64["K"], x64["V"], x64["dO"], cu))
            for name, g, w in zip(("O", "dQ", "dK", "dV"), outs, want):
                assert_close_blocks(name + " (replay) vs oracle", to_host(g), w, TOL[dtype])
