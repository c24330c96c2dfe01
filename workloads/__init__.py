"""Seeded synthetic inputs shared by the oracle-side tests and the GPU path.

This module only draws random numbers and names shapes.  It contains none of
the method's arithmetic (no scale statistic, no quantizer, no packing): the
activation-aware scale and the inverse-scaled activations are computed by
whichever side is under test from the raw arrays produced here.

The arrays stand in for the Llama-2 weights and the Pile calibration
activations used in the paper's experiments (Sec. 4.1, Sec. 5), which are not
available: shapes are the Llama-2-7B / 70B linear-layer shapes, weights are
N(0, sigma^2) in fp16, activations are N(0,1) in fp16 with 1 % of the input
channels (a seeded choice) multiplied by 20 to mimic the activation outlier
channels the method protects (Sec. 3.1).
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

BASE_SEED = 20230601
ROLE_W, ROLE_CALIB, ROLE_X, ROLE_OUTLIER = 0, 1, 2, 3

# (name, N, K) of the seven projections of one decoder layer
LLAMA2_7B_LAYER = [
    ("q_proj", 4096, 4096), ("k_proj", 4096, 4096), ("v_proj", 4096, 4096),
    ("o_proj", 4096, 4096), ("gate_proj", 11008, 4096), ("up_proj", 11008, 4096),
    ("down_proj", 4096, 11008),
]
LLAMA2_70B_LAYER = [
    ("q_proj", 8192, 8192), ("k_proj", 1024, 8192), ("v_proj", 1024, 8192),
    ("o_proj", 8192, 8192), ("gate_proj", 28672, 8192), ("up_proj", 28672, 8192),
    ("down_proj", 8192, 28672),
]
SIGMA_7B = 0.02
SIGMA_70B = 0.015
OUTLIER_FRACTION = 0.01
OUTLIER_GAIN = 20.0
CALIB_TOKENS = 64
PREFILL_M = 2048

# the full stack: 32 decoder layers, 128 decode steps, calibration set of 128 sequences of 512
# tokens (the size the paper calibrates on, Sec. 5 "Settings")
STACK_LAYERS = 32
STACK_STEPS = 128
CALIB_SEQUENCES = 128
CALIB_SEQ_LEN = 512
# distinct inputs of a decoder layer and the input each of the seven projections reads:
# 0 = attention input (q,k,v), 1 = attention output (o), 2 = MLP input (gate, up), 3 = down's input
LAYER_INPUT_OF_PROJ = (0, 0, 0, 1, 2, 2, 3)


def rng(cfg: int, layer: int, proj: int, role: int, *more: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence(
        [BASE_SEED, int(cfg), int(layer), int(proj), int(role)] + [int(v) for v in more])))


def weights(N: int, K: int, sigma: float, cfg: int, layer: int, proj: int) -> np.ndarray:
    """W[N,K] fp16 ~ N(0, sigma^2), drawn in fp32 and rounded to fp16."""
    g = rng(cfg, layer, proj, ROLE_W)
    out = np.empty((N, K), dtype=np.float16)
    step = max(1, (1 << 22) // K)
    for n0 in range(0, N, step):          # chunked: keeps the fp32 temporary small
        n1 = min(N, n0 + step)
        out[n0:n1] = (g.standard_normal((n1 - n0, K), dtype=np.float32) * np.float32(sigma)
                      ).astype(np.float16)
    return out


def outlier_channels(K: int, cfg: int, layer: int, proj: int) -> np.ndarray:
    """Indices of the round(1 % * K) outlier input channels (sorted)."""
    g = rng(cfg, layer, proj, ROLE_OUTLIER)
    cnt = int(round(OUTLIER_FRACTION * K))
    return np.sort(g.choice(K, size=cnt, replace=False))


def activations(T: int, K: int, cfg: int, layer: int, proj: int, role: int,
                outliers: np.ndarray) -> np.ndarray:
    """X[T,K] fp16 ~ N(0,1) with the outlier channels multiplied by 20."""
    g = rng(cfg, layer, proj, role)
    X = g.standard_normal((T, K), dtype=np.float32)
    X[:, outliers] *= np.float32(OUTLIER_GAIN)
    return X.astype(np.float16)


def calibration_sequences(n_seq: int, K: int, cfg: int, layer: int, inp: int,
                          outliers: np.ndarray, threads: int = 1) -> np.ndarray:
    """X[n_seq * 512, K] fp16: calibration sequences of 512 rows each, every sequence from a
    generator of its own (so they can be drawn in parallel and the result does not depend on
    the number of threads)."""
    X = np.empty((n_seq * CALIB_SEQ_LEN, K), dtype=np.float16)

    def one(i):
        g = rng(cfg, layer, inp, ROLE_CALIB, i)
        blk = g.standard_normal((CALIB_SEQ_LEN, K), dtype=np.float32)
        blk[:, outliers] *= np.float32(OUTLIER_GAIN)
        X[i * CALIB_SEQ_LEN:(i + 1) * CALIB_SEQ_LEN] = blk.astype(np.float16)

    if threads > 1:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(threads) as ex:
            list(ex.map(one, range(n_seq)))
    else:
        for i in range(n_seq):
            one(i)
    return X


@dataclass
class LinearCase:
    """Raw inputs of one linear layer: weight, calibration rows, test rows."""
    name: str
    N: int
    K: int
    W: np.ndarray          # [N,K] fp16
    calib: np.ndarray      # [T,K] fp16
    x: np.ndarray          # [M,K] fp16 (not yet divided by s)
    outliers: np.ndarray


def linear_case(name: str, N: int, K: int, M: int, sigma: float, cfg: int, layer: int = 0,
                proj: int = 0, calib_tokens: int = CALIB_TOKENS) -> LinearCase:
    out = outlier_channels(K, cfg, layer, proj)
    return LinearCase(
        name=name, N=N, K=K,
        W=weights(N, K, sigma, cfg, layer, proj),
        calib=activations(calib_tokens, K, cfg, layer, proj, ROLE_CALIB, out),
        x=activations(M, K, cfg, layer, proj, ROLE_X, out),
        outliers=out,
    )


def algorithmic_bytes(M: int, N: int, K: int, group: int = 128) -> int:
    """Bytes one W4A16 linear must move: codes + fp16 scales + uint4 zeros + x + y."""
    G = K // group
    return N * K // 2 + N * G * 2 + N * G // 2 + 2 * M * K + 2 * M * N


def flops(M: int, N: int, K: int) -> int:
    return 2 * M * N * K
