"""Seeded synthetic inputs with the shapes and outlier structure of the paper's
workloads.  They stand in for LLaMA / OPT weights and Wikitext-2 activations,
which are not available here.

This module only draws numbers: it holds none of the quantizers, products or
encodings of the method, and is the one piece of code that both the GPU tests
and the CPU oracle's tests may share.

Recipe (Section 3.2 of the paper: outliers sit in the same few channels of
every token; Section 5.4: sequence length 2048; Section 3.1: most tokens
attend to the start token):
  activations  X ~ N(0,1) [M,K], `n_outlier` channels picked without
               replacement and multiplied by 20, cast to fp16;
  weights      W ~ N(0, 0.02) [N,K] float32; the 4-bit stand-in for GPTQ is
               symmetric round-to-nearest per output channel (scale =
               fp16(max|row|/7));
  attention    logits = Q K^T / sqrt(D) + a[h,i] on column 0, a ~ N(4,2),
               causal mask, float32 softmax, cast to fp16; V ~ N(0,1).
"""
from __future__ import annotations

import numpy as np

# (name, K, N) of the seven projections of one LLaMA-7B block
LLAMA7B_PROJ = [
    ("q_proj", 4096, 4096), ("k_proj", 4096, 4096), ("v_proj", 4096, 4096),
    ("o_proj", 4096, 4096), ("gate_proj", 4096, 11008), ("up_proj", 4096, 11008),
    ("down_proj", 11008, 4096),
]
LLAMA7B_LAYERS = 32
# LLaMA-13B-shaped attention block and the two projections that follow it
LLAMA13B_ATTN = dict(H=40, D=128, S=2048)
LLAMA13B_TAIL = [("o_proj", 5120, 5120), ("gate_proj", 5120, 13824)]


def make_activation(M: int, K: int, n_outlier: int, seed: int) -> np.ndarray:
    """fp16 [M,K]: N(0,1) with `n_outlier` whole channels scaled by 20."""
    rng = np.random.default_rng([seed, 0xAC7])
    x = rng.standard_normal((M, K), dtype=np.float32)
    if n_outlier > 0:
        ch = rng.choice(K, size=min(n_outlier, K), replace=False)
        x[:, ch] *= 20.0
    return x.astype(np.float16)


def make_weight(N: int, K: int, seed: int) -> np.ndarray:
    """float32 [N,K] drawn from N(0, 0.02)."""
    rng = np.random.default_rng([seed, 0x3E1])
    return (rng.standard_normal((N, K), dtype=np.float32) * np.float32(0.02))


def make_weight_q4(N: int, K: int, seed: int) -> tuple[np.ndarray, np.ndarray]:
    """(Wq int8 [N,K] in [-8,7], sw fp16 [N]): the 4-bit weights handed to both
    the library and the oracle.  Symmetric round-to-nearest per output channel
    stands in for GPTQ, which needs calibration data."""
    w = make_weight(N, K, seed).astype(np.float64)
    sw = (np.abs(w).max(axis=1) / 7.0).astype(np.float16)
    sw[sw == 0] = np.float16(1.0)
    wq = np.clip(np.rint(w / sw.astype(np.float64)[:, None]), -8, 7).astype(np.int8)
    return wq, sw


def make_attention(H: int, S: int, D: int, seed: int):
    """(P fp16 [H,S,S] causal softmax probabilities, V fp16 [H,S,D])."""
    rng = np.random.default_rng([seed, 0xA77])
    p = np.zeros((H, S, S), dtype=np.float16)
    causal = np.tril(np.ones((S, S), dtype=bool))
    for h in range(H):
        q = rng.standard_normal((S, D), dtype=np.float32)
        k = rng.standard_normal((S, D), dtype=np.float32)
        logits = (q @ k.T) / np.float32(np.sqrt(D))
        logits[:, 0] += (4.0 + 2.0 * rng.standard_normal(S)).astype(np.float32)
        logits = np.where(causal, logits, -np.inf).astype(np.float32)
        logits -= logits.max(axis=1, keepdims=True)
        ex = np.exp(logits)
        p[h] = (ex / ex.sum(axis=1, keepdims=True)).astype(np.float16)
    v = rng.standard_normal((H, S, D), dtype=np.float32).astype(np.float16)
    return p, v


def make_qkv_int8(H: int, S: int, D: int, seed: int):
    """int8 codes of Q, K, V [H,S,D] for the attention-from-Q-and-K path: unit normals in
    steps of 1/32 (|x| < 4), with a direction shared by every query and the first key so
    that most tokens attend to the start token (Section 4.3)."""
    rng = np.random.default_rng([seed, 0x9B1])
    q = rng.standard_normal((H, S, D))
    k = rng.standard_normal((H, S, D))
    u = rng.standard_normal((H, 1, D)) / np.sqrt(D)
    q += u * (4.0 + rng.standard_normal((H, S, 1)))
    k[:, :1] += 8.0 * u
    v = rng.standard_normal((H, S, D))
    to8 = lambda t: np.clip(np.rint(t * 32.0), -127, 127).astype(np.int8)
    return to8(q), to8(k), to8(v)


def rope_tables(P: int, D: int, base: float = 10000.0):
    """(cos, sin) float32 [P, D/2]: the angle of position p and pair i is p * base^(-2i/D)."""
    inv = base ** (-np.arange(0, D, 2, dtype=np.float64) / D)
    ang = np.arange(P, dtype=np.float64)[:, None] * inv[None, :]
    return np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)


def make_block_weights(d: int, H: int, F: int, seed: int) -> dict:
    """Weights of one LLaMA-shaped block: 4-bit `w_<name>` int8 [N,K] with fp16 scales
    `s_<name>` for q, k, v, o (d -> d), gate, up (d -> F), down (F -> d), and the two
    normalisation gains (1 + N(0, 0.1), fp16).  The projections are drawn as in
    `make_weight_q4` with a standard deviation of 1/sqrt(K), which keeps the residual
    stream of a random block at unit scale."""
    rng = np.random.default_rng([seed, 0xB10C])
    w = {}
    shapes = dict(q=(d, d), k=(d, d), v=(d, d), o=(d, d), gate=(F, d), up=(F, d), down=(d, F))
    for i, (name, (N, K)) in enumerate(shapes.items()):
        wq, sw = make_weight_q4(N, K, seed * 16 + i)
        w["w_" + name] = wq
        w["s_" + name] = (sw.astype(np.float64) / (0.02 * np.sqrt(K))).astype(np.float16)
    w["g_attn"] = (1.0 + 0.1 * rng.standard_normal(d)).astype(np.float16)
    w["g_mlp"] = (1.0 + 0.1 * rng.standard_normal(d)).astype(np.float16)
    return w


def n_outlier_channels(K: int, frac: float = 0.01) -> int:
    """About 1 % outlier channels, rounded up (prefill configurations)."""
    return int(np.ceil(frac * K))
