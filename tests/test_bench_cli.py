"""Host-side checks of bench.py that need no GPU: the one-GPU guard and the flop/byte bookkeeping."""
import importlib.util
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_nominal_flop_count():
    spec = importlib.util.spec_from_file_location("bench", os.path.join(ROOT, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    # 7 triangular C x C products (2 d per pair, C (C+1) / 2 pairs per chunk of C tokens: d (C+1) per token)
    # and 6 state products of 2 d^2 per token, forward 2 and backward 4
    d, C = 128, 256
    assert bench.nominal_flops_per_token_head(d, C) == 7 * d * (C + 1) + 6 * 2 * d * d
    assert bench.HBM_PEAK_GBS == 8000.0 and bench.MFMA_BF16_PEAK_TFLOPS == 2500.0


def _bench_module():
    spec = importlib.util.spec_from_file_location("bench", os.path.join(ROOT, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    return bench


def test_counter_figures_in_bench_match_the_committed_profile_summaries():
    """bench.py cannot read hardware counters, so `roofline.traffic` and `mfma_frac_executed` come
    from literals copied out of the rocprofv3 summaries under profiles/.  The literals must be the
    numbers those summaries print."""
    import re
    consts = _bench_module().PROFILE_CONSTANTS["cfg3"]
    GiB = float(1 << 30)
    text = open(os.path.join(ROOT, "profiles", "lasp2_kernels_cfg3_hbm_traffic.txt")).read()
    fwd = float(re.search(r"attention pass, forward launch\s*:\s*([0-9.]+) GiB moved", text).group(1))
    bwd = float(re.search(r"attention pass, backward launch\s*:\s*([0-9.]+) GiB moved", text).group(1))
    # the summaries print GiB with three decimals
    assert abs(consts["traffic_fwd_bytes"] - fwd * GiB) <= 0.001 * GiB
    assert abs(consts["traffic_bwd_bytes"] - bwd * GiB) <= 0.001 * GiB
    text = open(os.path.join(ROOT, "profiles", "attn_kernels_cfg3_sq_counters.txt")).read()
    assert consts["mfma_insts_fwd"] == int(re.search(r"forward\s+SQ_INSTS_MFMA\s+(\d+)", text).group(1))
    assert consts["mfma_insts_bwd"] == int(re.search(r"backward\s+SQ_INSTS_MFMA\s+(\d+)", text).group(1))
