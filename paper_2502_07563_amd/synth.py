"""Seeded synthetic inputs shaped like the paper's Linear-Llama3 layers.

This module only draws random numbers and rounds them to the storage type; it
contains none of the attention arithmetic, so the GPU tests, the bench and the
CPU oracle can all take their inputs from here.

Recipe: tensor `name` in {Q, K, V, dO}, group g = b*H + h (one (batch, head)
pair) is `default_rng([seed, tensor_id, g]).standard_normal((N, d), float32)
/ sqrt(d)`.  Every group has its own stream, so any single head of a large
configuration can be regenerated alone.  For bf16 configurations the fp32
draws are rounded to bf16 (round to nearest even) and those rounded values are
what both the GPU and the oracle see.
"""
from concurrent.futures import ThreadPoolExecutor
import math

import numpy as np

TENSOR_IDS = {"Q": 0, "K": 1, "V": 2, "dO": 3}

# Workloads named by the build's baseline (index = config number - 1).
CONFIGS = {
    "cfg1": dict(B=1, H=2, N=1024, d=64, C=128, L=0, dtype="f32", seed=0, packed=False),
    "cfg2": dict(B=1, H=16, N=32768, d=128, C=256, L=0, dtype="bf16", seed=1, packed=False),
    "cfg3": dict(B=1, H=16, N=262144, d=128, C=256, L=4096, dtype="bf16", seed=2, packed=False),
    "cfg4": dict(B=8, H=32, N=8192, d=128, C=256, L=0, dtype="bf16", seed=3, packed=False),
    "cfg5": dict(B=1, H=32, N=131072, d=128, C=256, L=0, dtype="bf16", seed=4, packed=True,
                 n_docs=40, mean_len=3277, min_len=64),
}


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16), round to nearest even.  Finite inputs only."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_round(x: np.ndarray) -> np.ndarray:
    """fp32 values rounded to the nearest bf16, returned as fp32."""
    return bf16_bits_to_f32(bf16_bits(x))


def gen_group(seed: int, name: str, g: int, N: int, d: int, dtype: str = "f32") -> np.ndarray:
    """One (batch, head) group of tensor `name`: fp32 [N, d], already rounded to `dtype`."""
    rng = np.random.default_rng([seed, TENSOR_IDS[name], g])
    x = rng.standard_normal((N, d), dtype=np.float32)
    x *= np.float32(1.0 / math.sqrt(d))
    if dtype == "bf16":
        x = bf16_round(x)
    return x


def gen_tensor(seed: int, name: str, G: int, N: int, d: int, dtype: str = "f32",
               workers: int = 8) -> np.ndarray:
    """All G groups of tensor `name`: fp32 [G, N, d] (values representable in `dtype`)."""
    out = np.empty((G, N, d), dtype=np.float32)

    def one(g):
        out[g] = gen_group(seed, name, g, N, d, dtype)

    if G == 1 or workers <= 1:
        for g in range(G):
            one(g)
    else:
        with ThreadPoolExecutor(max_workers=workers) as ex:
            list(ex.map(one, range(G)))
    return out


def doc_offsets(seed: int, total: int, n_docs: int, mean_len: float, min_len: int,
                sigma: float = 1.0) -> np.ndarray:
    """Document offsets cu[0..n_docs] for a packed batch of `total` tokens.

    Lengths are lognormal(mu = ln(mean_len) - sigma^2/2, sigma) draws scaled to
    sum to `total`, floored, clamped below at `min_len`; the rounding remainder
    goes to (or is taken from) the longest document.
    """
    rng = np.random.default_rng([seed, 1000])
    r = rng.lognormal(math.log(mean_len) - 0.5 * sigma * sigma, sigma, n_docs)
    lens = np.maximum(min_len, np.floor(r * total / r.sum())).astype(np.int64)
    lens[np.argmax(lens)] += total - lens.sum()
    assert lens.min() >= min_len and lens.sum() == total
    return np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)


def config_offsets(cfg: dict):
    """cu offsets of a packed configuration, or None."""
    if not cfg.get("packed"):
        return None
    return doc_offsets(cfg["seed"], cfg["N"], cfg["n_docs"], cfg["mean_len"], cfg["min_len"])
