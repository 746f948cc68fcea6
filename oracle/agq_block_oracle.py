"""CPU oracle for one transformer block of the quantized model (Section 4.2's
activation quantization pipeline, Figure 3) with activation-aware token pruning
after attention (Section 4.3) and the cascade schedule of Section 5.2 (Eq.9).

TEST INFRASTRUCTURE ONLY, like `agq_oracle`, on which it builds: only the tests,
the smoke check and the benchmark's `cpu_baseline` leg may import it.

The pipeline keeps the non-linear operators in fp16 and quantizes the operand of
every matrix product.  The block is LLaMA's (the model family the paper
evaluates first): RMSNorm, rotary position embedding, SwiGLU, two residual
additions.  Readings taken where the paper is silent (each repeated below):
  * a non-linear operator takes fp16 tensors and returns an fp16 tensor; its
    arithmetic is done in float64 and rounded once to fp16;
  * the rotary embedding pairs element i of a head with element i + D/2 and takes
    the angles from tables the caller supplies (float32 cos / sin per position);
  * q, k and v are quantized to int8 with static layer-wise exponents, the input
    of the projection after attention to 4 or 8 bits (Section 4.2 allows 4);
  * tokens are pruned right after the attention product: the projection after
    attention, the residual stream and the positions keep the surviving rows;
  * every exponent is static (post-training calibration): they are given, or,
    with `exps=None`, derived from this very input.
"""
from __future__ import annotations

import numpy as np

from . import agq_oracle as O


def to_f16(a) -> np.ndarray:
    """float64 -> fp16, round to nearest even in one step (overflow -> +-Inf)."""
    with np.errstate(over="ignore"):
        return np.asarray(a, dtype=np.float64).astype(np.float16)


def _f64(x) -> np.ndarray:
    x = np.asarray(x)
    if x.dtype != np.float16:
        raise TypeError("non-linear operators take fp16")
    return x.astype(np.float64)


# --------------------------------------------------------------------------
# the fp16 non-linear operators the pipeline leaves unquantized (Section 4.2)
# --------------------------------------------------------------------------

def rmsnorm(x, g, eps: float) -> np.ndarray:
    """Root-mean-square normalisation of every row:
    y[t,c] = x[t,c] * g[c] / sqrt(mean_c(x[t,:]^2) + eps), fp16 in, fp16 out."""
    x64, g64 = _f64(x), _f64(g)
    ms = (x64 * x64).sum(axis=1, keepdims=True) / x64.shape[1]
    return to_f16((x64 * g64[None, :]) * (1.0 / np.sqrt(ms + float(eps))))


def rope(x, pos, cos, sin, H: int) -> np.ndarray:
    """Rotary position embedding on fp16 [S, H*D]: inside every head the pair
    (x[i], x[i + D/2]) is rotated by the angle of (pos[t], i):
      y[i]       = x[i] cos - x[i + D/2] sin
      y[i + D/2] = x[i + D/2] cos + x[i] sin
    cos, sin: float32 [P, D/2] tables indexed by position.  fp16 out."""
    x64 = _f64(x)
    S, d = x64.shape
    D = d // H
    pos = np.asarray(pos, dtype=np.int64)
    cos, sin = np.asarray(cos), np.asarray(sin)
    if cos.dtype != np.float32 or sin.dtype != np.float32 or cos.shape[1] != D // 2:
        raise TypeError("tables are float32 [P, D/2]")
    c = cos[pos].astype(np.float64)[:, None, :]
    s = sin[pos].astype(np.float64)[:, None, :]
    xh = x64.reshape(S, H, D)
    lo, hi = xh[:, :, : D // 2], xh[:, :, D // 2:]
    y = np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=2)
    return to_f16(y.reshape(S, d))


def swiglu(gate, up) -> np.ndarray:
    """a = silu(gate) * up with silu(z) = z / (1 + exp(-z)), fp16 in and out."""
    g64, u64 = _f64(gate), _f64(up)
    with np.errstate(over="ignore"):
        return to_f16(g64 / (1.0 + np.exp(-g64)) * u64)


def residual_add(a, b) -> np.ndarray:
    """fp16(a + b): the sum of two fp16 values is exact in float64."""
    return to_f16(_f64(a) + _f64(b))


def heads_int8(x, H: int, e: int, S_pad: int | None = None) -> np.ndarray:
    """Eq.2 (8 bit, signed grid, step 2^e) on fp16 [S, H*D], returned per head as
    int8 [H, S, D].  S_pad (a test aid for comparing against a padded buffer): [H, S_pad, D]
    with zero rows from S on; the block itself never pads."""
    q = O.quantize_act(x, 8, e, 0)
    S, d = q.shape
    out = np.zeros((H, S_pad or S, d // H), dtype=np.int8)
    out[:, :S] = q.reshape(S, H, d // H).transpose(1, 0, 2)
    return out


# --------------------------------------------------------------------------
# Eq.9: cascade schedule
# --------------------------------------------------------------------------

def cascade_keep(S: int, beta: float, m: int) -> list[int]:
    """Section 5.2, Eq.9: m pruning stages, each with the progressive ratio
    gamma = 1 - (1 - beta)^(1/m); returns the tokens left after each stage."""
    gamma = O.progressive_ratio(beta, m)
    keep, out = int(S), []
    for _ in range(m):
        keep = O.n_keep(keep, gamma)
        out.append(keep)
    return out


# --------------------------------------------------------------------------
# the block
# --------------------------------------------------------------------------

EXP_NAMES = ("e_attn_in", "e_q", "e_k", "e_v", "e_attn_out", "e_mlp_in", "e_mlp_act")


SITES = ("attn_in", "attn_out", "mlp_in", "mlp_act")      # the four activations that feed projections


def block_forward(x, pos, cos, sin, w: dict, H: int, qmax: int, eps: float, keep: int,
                  bits_attn_out: int = 4, exps: dict | None = None, alphas: dict | None = None,
                  trip_kmax: int | None = None) -> dict:
    """One block of the pipeline of Section 4.2 on fp16 x [S,d] with positions pos [S].
    w holds g_attn, g_mlp (fp16 [d]) and for each of q, k, v, o, gate, up, down
    the 4-bit weights `w_<name>` (int8 [N,K]) with their scales `s_<name>`.
    exps: the static exponents (EXP_NAMES); None calibrates them on this input.
    alphas: TRIP factors (Section 4.3, Eq.5) per site of SITES, int [K] each, for the
    activations that feed projections; a site without an entry uses Eq.2.  With a site's
    factors its exponent is Eq.6's base step.  trip_kmax (only with exps None): derive
    base step and factors of every site on the way (Eq.6, Eq.8 with K = trip_kmax).
    keep: tokens that survive the pruning after attention (== S: none pruned).
    Returns every intermediate tensor by name, `x_out` [keep,d], `pos_out`, `idx`
    and the exponents used."""
    x = np.asarray(x)
    S, d = x.shape
    D = d // H
    e = dict(exps) if exps is not None else {}

    al = dict(alphas) if alphas is not None else {}

    def exp_of(name, t, bits, site=None):
        if exps is None:
            if site is not None and trip_kmax is not None:
                e[name] = O.trip_base_exp(t, bits, trip_kmax)
                al[site] = O.trip_search(t, bits, e[name], 0, trip_kmax)
            else:
                e[name] = O.calibrate_act_exp(t, bits)
        return e[name]

    def linear(t, bits, ee, site, name):
        if al.get(site) is not None:
            return O.linear_w4_trip(t, bits, ee, 0, al[site], w["w_" + name], w["s_" + name])[1]
        return O.linear_w4(t, bits, ee, 0, w["w_" + name], w["s_" + name])[1]

    r = {}
    r["h1"] = rmsnorm(x, w["g_attn"], eps)
    ea = exp_of("e_attn_in", r["h1"], 8, "attn_in")
    for n in ("q", "k", "v"):
        r[n] = linear(r["h1"], 8, ea, "attn_in", n)
    r["q_rot"] = rope(r["q"], pos, cos, sin, H)
    r["k_rot"] = rope(r["k"], pos, cos, sin, H)
    eq, ek, ev = exp_of("e_q", r["q_rot"], 8), exp_of("e_k", r["k_rot"], 8), exp_of("e_v", r["v"], 8)
    r["q_q"] = heads_int8(r["q_rot"], H, eq)
    r["k_q"] = heads_int8(r["k_rot"], H, ek)
    r["v_q"] = heads_int8(r["v"], H, ev)
    r["codes"], r["margin"] = O.qk_log2_codes(r["q_q"], r["k_q"], eq, ek, qmax, causal=True)
    _, r["o"] = O.attn_v_from_codes(r["codes"], r["v_q"], ev, qmax, causal=True)
    r["score"] = O.start_token_score_codes(r["codes"], qmax)
    idx = O.prune_select(r["score"], keep)
    r["idx"] = idx
    r["o_kept"] = r["o"][idx]
    eo = exp_of("e_attn_out", r["o_kept"], bits_attn_out, "attn_out")
    r["attn_out"] = linear(r["o_kept"], bits_attn_out, eo, "attn_out", "o")
    r["x1"] = residual_add(x[idx], r["attn_out"])
    r["pos_out"] = np.asarray(pos, dtype=np.int32)[idx]
    r["h2"] = rmsnorm(r["x1"], w["g_mlp"], eps)
    em = exp_of("e_mlp_in", r["h2"], 8, "mlp_in")
    r["gate"] = linear(r["h2"], 8, em, "mlp_in", "gate")
    r["up"] = linear(r["h2"], 8, em, "mlp_in", "up")
    r["act"] = swiglu(r["gate"], r["up"])
    ed = exp_of("e_mlp_act", r["act"], 8, "mlp_act")
    r["down"] = linear(r["act"], 8, ed, "mlp_act", "down")
    r["x_out"] = residual_add(r["x1"], r["down"])
    r["alphas"] = al
    r["exps"] = e
    return r


def stack_forward(x, pos, cos, sin, weights: list, H: int, qmax: int, eps: float, keep: list,
                  bits_attn_out: int = 4, exps: list | None = None) -> list:
    """A stack of blocks with the cascade pruning of Section 5.2: block l receives what block l-1
    kept (tokens and positions) and keeps keep[l] of them.  weights, keep and exps are per block.
    Returns the per-block results of `block_forward`; the last one's x_out / pos_out are the stack's."""
    out = []
    for l, (w, k) in enumerate(zip(weights, keep)):
        r = block_forward(x, pos, cos, sin, w, H, qmax, eps, int(k), bits_attn_out,
                          None if exps is None else exps[l])
        out.append(r)
        x, pos = r["x_out"], r["pos_out"]
    return out
