#!/usr/bin/env python3
"""Throughput of the LASP-2 hot path on one MI355X: one "step" is a full forward
(chunk_states -> state_prefix -> attn_fwd) plus a full backward (attn_bwd: dM states,
suffix combine, dQ/dK/dV) of one attention layer over one batch of synthetic input
that is already resident in HBM.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg3]

Prints ONE JSON line.  `value` is tokens/s for the layer; `roofline` prices the
dominant kernel (the fused attention pass, launched once by the forward and once by
the backward) against HBM peak using its algorithmic bytes and its HIP-event duration
measured inside the timed loop; `cpu_baseline` is the CPU oracle timed on a bounded
sample of the same workload.
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 MFMA, published

# Figures that only a counter run can give, copied from the rocprofv3 summaries under profiles/
# (counters cannot be read from inside this script).  tests/test_bench_cli.py parses those
# summaries and fails when a literal here differs from them.
#   traffic_*_bytes: HBM bytes per launch of the attention kernel, FETCH_SIZE + WRITE_SIZE
#                    (profiles/lasp2_kernels_cfg3_hbm_traffic.txt)
#   mfma_insts_*:    v_mfma_f32_32x32x16_bf16 instructions per launch, SQ_INSTS_MFMA
#                    (profiles/attn_kernels_cfg3_sq_counters.txt)
PROFILE_CONSTANTS = {
    "cfg3": {"traffic_fwd_bytes": 4.3626e9, "traffic_bwd_bytes": 7.6922e9,
             "mfma_insts_fwd": 13500416, "mfma_insts_bwd": 32538624},
}
MFMA_FLOP = 2 * 32 * 32 * 16    # one v_mfma_f32_32x32x16_bf16


def nominal_flops_per_token_head(d, C):
    """Algorithmic flop count of the method: 7 masked/unmasked C x C products counted on the
    causal triangle plus 6 state products (forward 2, backward 4) of 2 d^2 each."""
    return 7 * d * (C + 1) + 12 * d * d


def cpu_baseline(cfg, sample_tokens):
    """The oracle (recurrent form, fp64) on all H heads of a `sample_tokens`-long prefix."""
    import numpy as np
    import oracle
    from paper_2502_07563_amd import synth
    G = cfg["B"] * cfg["H"]
    G = min(G, cfg["H"])          # one batch row is enough for a per-layer rate
    x = {n: synth.gen_tensor(cfg["seed"], n, G, sample_tokens, cfg["d"], cfg["dtype"]).astype(np.float64)
         for n in ("Q", "K", "V", "dO")}
    t0 = time.perf_counter()
    oracle.fwd_rec(x["Q"], x["K"], x["V"])
    oracle.bwd_rec(x["Q"], x["K"], x["V"], x["dO"])
    dt = time.perf_counter() - t0
    return {"value": sample_tokens / dt, "unit": "tokens/s", "cores": oracle.threads(), "kind": "oracle",
            "sample": f"recurrent fp64 oracle, fwd+bwd, {G} heads x first {sample_tokens} tokens "
                      f"of the workload, {dt:.1f} s"}


def softmax_main(args):
    """The standard-attention layer of the hybrid model (forward + backward of
    lasp2_softmax_fwd_share / lasp2_softmax_bwd_share), causal, B=1, H=16, d=128: by default a
    whole sequence of 32768 tokens on the one GPU; with --softmax-total T the last rank's share of
    a T-token sequence (its 32768 queries against all T gathered keys).  Priced against the bf16 MFMA peak with
    the algorithmic flop count on the causal triangle: 2 products forward, 5 backward."""
    import numpy as np
    import torch
    from paper_2502_07563_amd import binding as bd
    B, H, d = 1, 16, 128
    n_q = args.softmax_len                       # queries of the call
    N = args.softmax_total or n_q                # gathered keys; the share is the sequence's last n_q tokens
    q_begin = N - n_q
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    p = bd.Problem(B, H, N, d, 64, 0, "bf16")
    gen = torch.Generator(device=dev)
    gen.manual_seed(41)
    mk = lambda n: torch.randn((B, H, n, d), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    Q, dO, K, V = mk(n_q), mk(n_q), mk(N), mk(N)
    O, dQ = torch.empty_like(Q), torch.empty_like(Q)
    dK, dV = torch.empty_like(K), torch.empty_like(K)
    LSE = torch.empty((B, H, n_q), dtype=torch.float32, device=dev)
    ws = torch.empty(bd.lasp2_softmax_share_workspace_size(p, n_q), dtype=torch.uint8, device=dev)
    ev = lambda: torch.cuda.Event(enable_timing=True)
    marks = []

    def step(record):
        e = [ev() for _ in range(3)] if record else None
        if record:
            e[0].record()
        bd.lasp2_softmax_fwd_share(p, q_begin, n_q, Q, K, V, O, LSE, True)
        if record:
            e[1].record()
        bd.lasp2_softmax_bwd_share(p, q_begin, n_q, Q, K, V, O, dO, LSE, dQ, dK, dV, ws, True)
        if record:
            e[2].record()
            marks.append(e)

    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(True)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    t_fwd = sum(m[0].elapsed_time(m[1]) for m in marks) / len(marks)
    t_bwd = sum(m[1].elapsed_time(m[2]) for m in marks) / len(marks)
    pairs = B * H * (n_q * q_begin + n_q * (n_q + 1) / 2.0)     # (query, key) pairs inside the causal mask
    fl_fwd, fl_bwd = 4.0 * pairs * d, 10.0 * pairs * d
    out = {
        "metric": "fwd+bwd tokens/s per layer", "value": B * n_q / (dt / args.steps), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt * 1e3 / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"softmax attention layer of the hybrid model: B={B} H={H} N={N} d={d} causal"
                               + (f", one rank's share: the last {n_q} queries against all {N} gathered keys"
                                  if q_begin else "")},
        "ms": {"softmax_fwd": t_fwd, "softmax_bwd": t_bwd},
        "roofline": {"bound": "mfma", "kernel": "lasp2_softmax_bwd (delta, dQ and dK/dV kernels; the dK/dV "
                     "kernel dominates)", "achieved": fl_bwd / (t_bwd * 1e-3) / 1e12,
                     "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": fl_bwd / (t_bwd * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, "traffic": None,
                     "fwd_TFLOPs": fl_fwd / (t_fwd * 1e-3) / 1e12,
                     "fwd_frac": fl_fwd / (t_fwd * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS},
    }
    if not args.no_cpu_baseline:
        import oracle
        n = min(n_q, 4096)
        rng = np.random.default_rng(41)
        x = [rng.standard_normal((H, n, d)) for _ in range(4)]
        t0 = time.perf_counter()
        oracle.softmax_fwd(x[0], x[1], x[2], True)
        oracle.softmax_bwd(x[0], x[1], x[2], x[3], True)
        dtc = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": n / dtc, "unit": "tokens/s", "cores": oracle.threads(), "kind": "oracle",
                               "sample": f"fp64 oracle, softmax fwd+bwd, {H} heads x {n} tokens, whole sequence "
                                         f"causal (the rate falls as 1/keys; for this workload's "
                                         f"{pairs / (B * H * n_q):.0f} keys per query it would be about "
                                         f"{n / dtc * (n / 2.0) / (pairs / (B * H * n_q)):.1f}), {dtc:.1f} s"}
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg3")
    ap.add_argument("--slot-len", type=int, default=None,
                    help="tokens per state slot L (a multiple of C) instead of the workload's own; "
                         "L = N is the serial-carry schedule with one slot per head")
    ap.add_argument("--heads", type=int, default=None,
                    help="override the workload's number of heads (a study of a partly filled device; "
                         "such a line is not the named workload and carries no profile constants)")
    ap.add_argument("--decay", action="store_true",
                    help="run the step with scalar decay, per-head factors 1 - 2^(-5-h) (not the headline "
                         "workload; the CPU baseline, which is the undecayed oracle, is then left out)")
    ap.add_argument("--softmax", action="store_true",
                    help="time the standard-attention layer of the hybrid model instead (not the headline "
                         "workload): causal softmax attention forward + backward, B=1 H=16 d=128")
    ap.add_argument("--softmax-len", type=int, default=32768, help="number of queries for --softmax")
    ap.add_argument("--softmax-total", type=int, default=None,
                    help="for --softmax: length of the whole gathered sequence; the call then computes one "
                         "rank's share, the sequence's last --softmax-len queries against all keys "
                         "(default: the queries are the whole sequence)")
    ap.add_argument("--cpu-sample-tokens", type=int, default=131072)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--graph", action="store_true",
                    help="also record the step into a HIP graph and time its replays (added as "
                         "`graph_ms_per_step`; `value` stays the eager step's)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="kept for older command lines: the 1 GiB device-to-device copy (outside the timed "
                         "region) that a counter run scales its counters by is now always run")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    if args.softmax:
        return softmax_main(args)

    import torch
    from paper_2502_07563_amd import binding as bd
    from paper_2502_07563_amd import synth

    cfg = synth.CONFIGS[args.workload]
    B, H, N, d, C, L = (cfg[k] for k in ("B", "H", "N", "d", "C", "L"))
    if args.slot_len is not None:
        L = args.slot_len
    if args.heads is not None:
        H = args.heads
    dtype = cfg["dtype"]
    cu = synth.config_offsets(cfg)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    decay = None
    if args.decay:
        import numpy as np
        decay = (1.0 - 2.0 ** (-5.0 - np.arange(H))).astype(np.float32)
    p = bd.Problem(B, H, N, d, C, L, dtype, cu, decay=decay)
    tdt = p.torch_dtype

    gen = torch.Generator(device=dev)
    gen.manual_seed(cfg["seed"])
    mk = lambda: (torch.randn((B, H, N, d), generator=gen, device=dev, dtype=torch.float32)
                  / math.sqrt(d)).to(tdt)
    Q, K, V, dO = mk(), mk(), mk(), mk()
    O, dQ, dK, dV = (torch.empty_like(Q) for _ in range(4))
    P = bd.alloc_states(p)
    ws = bd.alloc_workspace(p)
    T_s = P.shape[2]
    # One slot per sequence (e.g. --slot-len N): the serial-carry schedule.  Every prefix is zero, so
    # the step makes no chunk_states / state_prefix call and hands P = NULL to both attention calls.
    lone = T_s == (1 if cu is None else len(cu) - 1)
    seg_names = ["attn_fwd", "attn_bwd"] if lone else ["chunk_states", "state_prefix", "attn_fwd", "attn_bwd"]

    ev = lambda: torch.cuda.Event(enable_timing=True)
    marks = []

    def step(record):
        e = [ev() for _ in range(len(seg_names) + 1)] if record else None
        i = 0

        def mark():
            nonlocal i
            if record:
                e[i].record()
                i += 1
        mark()
        if not lone:
            bd.lasp2_chunk_states(p, K, V, P)
            mark()
            bd.lasp2_state_prefix(p, P, P, False)
            mark()
        bd.lasp2_attn_fwd(p, Q, K, V, None if lone else P, O)
        mark()
        bd.lasp2_attn_bwd(p, Q, K, V, dO, None if lone else P, dQ, dK, dV, ws)
        mark()
        if record:
            marks.append(e)

    # The attention kernels may walk several of the caller's slots per workgroup (lasp2_walk_slots):
    # the forward then reads one prefix state per walk, and the backward builds its dM states per walk.
    Leff = L or C
    doc_lens = [N] if cu is None else [int(b - a) for a, b in zip(cu[:-1], cu[1:])]
    walks = lambda w: sum(-(-n // (w * Leff)) for n in doc_lens)
    ws_f, ws_b = bd.lasp2_walk_slots(p), bd.lasp2_walk_slots(p, backward=True)
    Tw_f, Tw_b = walks(ws_f), walks(ws_b)
    lone_f, lone_b = Tw_f == len(doc_lens), Tw_b == len(doc_lens)
    # What lasp2_attn_bwd spends before its attention launch: the walks' own dM_t = Q_t^T dO_t and their
    # suffix combine, timed once here through the public calls on a descriptor whose slots are the walks
    # (the undecayed matrix-core kernels want the dM_t even when every sequence is a single walk).
    pre_ms = 0.0
    mfma = dtype == "bf16" and d == 128
    if not lone_b or (mfma and not args.decay):
        pw = bd.Problem(B, H, N, d, C, ws_b * Leff, dtype, cu, decay=decay) if ws_b > 1 else p

        def pre():
            bd.lasp2_chunk_states(pw, Q, dO, ws)
            if not lone_b:
                bd.lasp2_state_prefix(pw, ws, ws, True)
        pre()
        torch.cuda.synchronize()
        c0, c1 = ev(), ev()
        c0.record()
        for _ in range(5):
            pre()
        c1.record()
        torch.cuda.synchronize()
        pre_ms = c0.elapsed_time(c1) / 5

    # A plain 1 GiB device-to-device copy, outside the timed region: what a streaming kernel
    # reaches on this device next to the published peak (and, under a counter run, a kernel
    # of known traffic to scale the counters by).
    src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    c0, c1 = ev(), ev()
    c0.record()
    for _ in range(5):
        dst.copy_(src)
    c1.record()
    torch.cuda.synchronize()
    copy_gbps = 2.0 * src.numel() * 4 / (c0.elapsed_time(c1) / 5 * 1e-3) / 1e9
    del src, dst

    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(True)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    graph_ms = None
    if args.graph:
        # The library only enqueues kernels on the caller's stream, so the step records as it stands.
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.graph(graph, stream=side):
            step(False)
        for _ in range(max(1, args.warmup)):
            graph.replay()
        torch.cuda.synchronize()
        g0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - g0) * 1e3 / args.steps

    ms_per_step = dt * 1e3 / args.steps
    tokens = B * N
    value = tokens / (dt / args.steps)
    nseg = len(seg_names)
    per_step = [[m[i].elapsed_time(m[i + 1]) for m in marks] for i in range(nseg)]
    stat = lambda v: {"mean": sum(v) / len(v), "median": sorted(v)[len(v) // 2], "min": min(v)}
    seg = {n: stat(v) for n, v in zip(seg_names, per_step)}

    esz = 2 if dtype == "bf16" else 4
    mfma_path = dtype == "bf16" and d == 128
    pair_kernel = mfma_path and ws_b * Leff > 128 and not args.decay   # dV and dK of a walk in one workgroup
    # Dominant kernels: the attention launches, one per direction.  Algorithmic bytes:
    #   forward launch : Q, K, V read, O written, one state array read            (4 passes)
    #   backward launch: Q, K, V, dO read once, dQ, dK, dV written, P read once and the suffix states
    #                    once (dV and dK in one workgroup) or twice (one workgroup each)   (7 passes)
    # With one slot per sequence no prefix state is read.
    tensor = B * H * N * d * esz
    state = B * H * d * d * 4
    bytes_fwd = 4 * tensor + (0 if lone_f else Tw_f * state)
    bytes_bwd = 7 * tensor + ((0 if lone_b else 1) + (1 if pair_kernel else 2)) * Tw_b * state
    # HIP events bracket the forward launch exactly.  The backward launch sits inside
    # lasp2_attn_bwd behind a states kernel and a combine kernel, timed before the loop (pre_ms),
    # so its time is attn_bwd minus those.
    fwd_v = per_step[seg_names.index("attn_fwd")]
    bwd_v = [t - pre_ms for t in per_step[seg_names.index("attn_bwd")]]
    wide_f, wide_b = ws_f * Leff > 128, ws_b * Leff > 128
    if not mfma_path:
        kern_fwd = kern_bwd = "attn_generic_kernel"
    elif args.decay:
        kern_fwd = "attn_skew_mfma_kernel<decay>" if wide_f else "attn_decay_mfma_kernel<128>"
        kern_bwd = "attn_skew_mfma_kernel<decay>" if wide_b else "attn_decay_mfma_kernel<128>"
    else:
        kern_fwd = "attn_skew_mfma_kernel" if wide_f else "attn_mfma_kernel<128>"
        kern_bwd = "attn_bwd_pair_mfma_kernel" if wide_b else "attn_mfma_kernel<128>"
    consts = {} if (args.decay or args.slot_len is not None or args.heads is not None) else PROFILE_CONSTANTS.get(args.workload, {})

    def launch(v, nbytes, traffic):
        st = stat(v)
        gbps = nbytes / (st["mean"] * 1e-3) / 1e9
        return {"ms": st["mean"], "ms_median": st["median"], "ms_min": st["min"], "algorithmic_bytes": nbytes,
                "GBps": gbps, "frac": gbps / HBM_PEAK_GBS, "traffic": traffic}
    lf = launch(fwd_v, bytes_fwd, consts.get("traffic_fwd_bytes"))
    lb = launch(bwd_v, bytes_bwd, consts.get("traffic_bwd_bytes"))
    # the headline is the longer launch's own figure, not a blend of the two
    head, which = (lb, f"{kern_bwd}, the backward's attention launch (dQ, dV, dK of every slot)") \
        if lb["ms"] >= lf["ms"] else (lf, f"{kern_fwd}, the forward's attention launch")
    flops_nominal = nominal_flops_per_token_head(d, C) * tokens * H
    out = {
        "metric": "fwd+bwd tokens/s per layer",
        "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": dtype, "data": "synthetic",
        "config": {"workload": f"{args.workload}: B={B} H={H} N={N} d={d} C={C} L={L or C}"
                               + (f" packed {cfg['n_docs']} docs" if cu is not None else "")
                               + (" decay 1-2^(-5-h)" if args.decay else "")
                               + (" serial carry: one slot per sequence, no state arrays in the forward" if lone else ""),
                   "state_slots": int(T_s), "slots_per_walk": {"fwd": ws_f, "bwd": ws_b}},
        "ms": {n: seg[n]["mean"] for n in seg_names},
        "ms_median": {n: seg[n]["median"] for n in seg_names},
        "ms_min": {n: seg[n]["min"] for n in seg_names},
        "mfma_frac_nominal": flops_nominal / (dt / args.steps) / (MFMA_BF16_PEAK_TFLOPS * 1e12),
        "roofline": {"bound": "hbm", "kernel": f"{which}: the longer of the step's two attention launches",
                     "achieved": head["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": head["frac"], "traffic": head["traffic"],
                     "launch_ms": head["ms"],
                     "launches": {"fwd": dict(lf, kernel=kern_fwd),
                                  "bwd": dict(lb, kernel=kern_bwd,
                                              **({"note": "priced against HBM as the contract asks; what limits this launch "
                                                          "is the LDS instruction rate inside its fused dV/dK workgroups"}
                                                 if pair_kernel else {}))},
                     "device_copy_GBps": copy_gbps},
    }
    if graph_ms is not None:
        out["graph_ms_per_step"] = graph_ms
    if "mfma_insts_fwd" in consts:
        # executed matrix-core work: the attention launches from the SQ_INSTS_MFMA counter, the two
        # chunk-state launches from their tiling (2 d^2 flop per token and head, no padding at this size)
        executed = (consts["mfma_insts_fwd"] + consts["mfma_insts_bwd"]) * MFMA_FLOP + 2 * 2.0 * d * d * tokens * H
        out["mfma_frac_executed"] = executed / (dt / args.steps) / (MFMA_BF16_PEAK_TFLOPS * 1e12)
    if not args.no_cpu_baseline and not args.decay:
        out["cpu_baseline"] = cpu_baseline(cfg, args.cpu_sample_tokens)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
