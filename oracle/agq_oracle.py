"""CPU oracle for the Agile-Quant W4A8 / W4A4 linear layer and its log2-softmax path.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain definition that the
GPU library is checked against.  Only the tests, the smoke check and the
`cpu_baseline` leg of the benchmark may import it; the product path never does.
It shares no code with the HIP kernels and imports nothing from the package.

Every function states the passage of the paper (arxiv 2312.05693) it follows.
Floating point is done in float64, where every product below is exact, and is
rounded once at the end; integer work is done in int64 and asserted to fit the
int32 accumulator the method uses.

Readings taken where the paper is silent (each is repeated at its function):
  * activation scale is a power of two, s = 2^e, one per tensor (layer-wise);
  * round-to-nearest with ties to even;
  * zp == 0 selects the signed grid of Eq.1, zp > 0 the unsigned grid of Eq.2;
  * weights: symmetric round-to-nearest per output channel stands in for GPTQ;
  * Eq.3 is applied to softmax probabilities with max|X| taken as 1.0;
  * token importance is the attention paid to the first token, summed over heads;
  * TRIP: Eq.6's step is the layer-wise one divided by 2^K (K the largest
    refinement), and Eq.8's rounding term includes Eq.5's clip.
NaN inputs are outside every quantizer's domain: the oracle raises on them.
"""
from __future__ import annotations

import numpy as np

# --------------------------------------------------------------------------
# Eq.1  integer grids
# --------------------------------------------------------------------------

def grid_bounds(bits: int, zp: int = 0) -> tuple[int, int]:
    """Section 4.1, Eq.1: the signed grid {-2^(b-1) .. 2^(b-1)-1} (taken when
    zp == 0) or the unsigned grid {0 .. 2^b-1} (taken when zp > 0)."""
    if bits < 2 or bits > 8:
        raise ValueError("bits must be in 2..8")
    if zp == 0:
        return -(1 << (bits - 1)), (1 << (bits - 1)) - 1
    if zp < 0 or zp > (1 << bits) - 1:
        raise ValueError("zp outside the unsigned grid")
    return 0, (1 << bits) - 1


def _as_f64(x) -> np.ndarray:
    x = np.asarray(x)
    if x.dtype != np.float16:
        raise TypeError("activations are fp16")
    x64 = x.astype(np.float64)          # exact
    if np.isnan(x64).any():
        raise ValueError("NaN is outside the quantizer's domain")
    return x64


# --------------------------------------------------------------------------
# Eq.2  uniform quantizer with s = 2^e
# --------------------------------------------------------------------------

def quantize_act(x, bits: int, e: int, zp: int = 0) -> np.ndarray:
    """Section 4.1, Eq.2: q = CLIP(round(x / s) + zp, lo, hi) with s = 2^e.

    x / 2^e is exact in float64; `np.rint` rounds ties to even; +-Inf land on
    the clip bounds.  Returns int32 codes on the grid of `grid_bounds`."""
    lo, hi = grid_bounds(bits, zp)
    r = np.ldexp(_as_f64(x), -int(e))               # exact scaling by 2^-e
    t = np.rint(r)                                   # ties to even
    q = np.clip(t + float(zp), float(lo), float(hi))
    return q.astype(np.int32)


def dequantize_act(q, e: int, zp: int = 0) -> np.ndarray:
    """Inverse map of Eq.2: x_hat = (q - zp) * 2^e (exact in float64)."""
    return np.ldexp((np.asarray(q, dtype=np.int64) - int(zp)).astype(np.float64), int(e))


def calibrate_act_exp(x, bits: int) -> int:
    """Layer-wise power-of-two scale (Section 4.4, one scale for all channels):
    the smallest integer e with max|x| <= qmax * 2^e, qmax = 2^(b-1)-1.
    An all-zero tensor gives e = 0.  Non-finite entries count as magnitude 2^16
    (above every finite fp16), so the result is always defined."""
    x = np.asarray(x)
    if x.dtype != np.float16:
        raise TypeError("activations are fp16")
    a = np.abs(x.astype(np.float64))
    a = np.where(np.isfinite(a), a, 65536.0)
    amax = float(a.max()) if a.size else 0.0
    if amax == 0.0:
        return 0
    qmax = (1 << (bits - 1)) - 1
    e = -64
    while amax > qmax * (2.0 ** e):                  # predicate, never a log
        e += 1
    return e


# --------------------------------------------------------------------------
# 4-bit storage: two codes per byte
# --------------------------------------------------------------------------

def pack_nibbles(q) -> np.ndarray:
    """Two 4-bit codes per byte along the last axis: the low nibble holds the
    even index, the high nibble the odd one; signed codes are stored in two's
    complement (Section 4.4 packs two adjacent 4-bit values into one byte)."""
    q = np.asarray(q, dtype=np.int64)
    if q.shape[-1] % 2:
        raise ValueError("last axis must be even")
    if q.min(initial=0) < -8 or q.max(initial=0) > 15:
        raise ValueError("code does not fit four bits")
    u = (q & 0xF).astype(np.uint8)
    return (u[..., 0::2] | (u[..., 1::2] << 4)).astype(np.uint8)


def unpack_nibbles(b, signed: bool = True) -> np.ndarray:
    """Inverse of `pack_nibbles`; returns int32 codes."""
    b = np.asarray(b, dtype=np.uint8)
    lo = (b & 0xF).astype(np.int32)
    hi = (b >> 4).astype(np.int32)
    out = np.empty(b.shape[:-1] + (b.shape[-1] * 2,), dtype=np.int32)
    out[..., 0::2] = lo
    out[..., 1::2] = hi
    if signed:
        out = np.where(out >= 8, out - 16, out)
    return out


# --------------------------------------------------------------------------
# weights: per-output-channel symmetric 4-bit (stand-in for GPTQ, Section 5.1)
# --------------------------------------------------------------------------

def quantize_weight_rtn(w) -> tuple[np.ndarray, np.ndarray]:
    """Per-output-channel weight parameters (Section 4.4: engines take per-channel
    scales for weights).  sw[n] = fp16(max_k |W[n,k]| / 7), 1 where the row is
    zero; Wq = CLIP(round(W / sw), -8, 7) with ties to even.  W is [N, K]."""
    w = np.asarray(w, dtype=np.float64)
    amax = np.abs(w).max(axis=1)
    sw = (amax / 7.0).astype(np.float16)
    sw = np.where(sw == 0, np.float16(1.0), sw).astype(np.float16)
    q = np.rint(w / sw.astype(np.float64)[:, None])
    q = np.clip(q, -8, 7).astype(np.int8)
    return q, sw


# --------------------------------------------------------------------------
# integer contraction and dequantisation
# --------------------------------------------------------------------------

INT32_MAX = (1 << 31) - 1


def gemm_int(q, zp: int, wq) -> np.ndarray:
    """acc[m,n] = sum_k (q[m,k] - zp) * Wq[n,k]: the product of the quantized
    activation with the 4-bit weight matrix, accumulated in integers
    (Section 4.4: layer-wise activation, per-channel weight).  int64 here,
    asserted to fit the 32-bit accumulator."""
    a = np.asarray(q, dtype=np.int64) - int(zp)
    b = np.asarray(wq, dtype=np.int64)
    if a.shape[-1] != b.shape[-1]:
        raise ValueError("K mismatch")
    acc = a @ b.T
    if acc.size and max(int(acc.max()), -int(acc.min())) > INT32_MAX:
        raise OverflowError("accumulator leaves int32")
    return acc


def dequant_out(acc, e: int, sw) -> np.ndarray:
    """y[m,n] = fp16( acc[m,n] * 2^e * sw[n] ): the layer-wise activation scale
    times the per-channel weight scale (Section 4.4).  The product is exact in
    float64 (32 + 11 significant bits) and is rounded once, to fp16."""
    sw = np.asarray(sw)
    if sw.dtype != np.float16:
        raise TypeError("weight scales are fp16")
    g = np.ldexp(sw.astype(np.float64), int(e))              # exact
    y = np.asarray(acc, dtype=np.int64).astype(np.float64) * g[None, :]
    with np.errstate(over="ignore"):
        return y.astype(np.float16)


def linear_w4(x, bits: int, e: int, zp: int, wq, sw):
    """The whole linear layer: Eq.2 on the activation, integer product with the
    4-bit weights, per-channel dequantisation.  Returns (acc int64, y fp16)."""
    q = quantize_act(x, bits, e, zp)
    acc = gemm_int(q, zp, wq)
    return acc, dequant_out(acc, e, sw)


# --------------------------------------------------------------------------
# Eq.5-8  TRIP: per-channel power-of-two factors on top of the layer-wise step
# --------------------------------------------------------------------------

def _check_alpha(alpha, K: int) -> np.ndarray:
    alpha = np.asarray(alpha, dtype=np.int64)
    if alpha.shape != (K,):
        raise ValueError("one factor per channel")
    if alpha.size and (alpha.min() < 0 or alpha.max() > 4):
        raise ValueError("factors lie in 0..4")
    return alpha


def trip_base_exp(x, bits: int, kmax: int) -> int:
    """Section 4.3, Eq.6 with s a power of two.  As printed the equation makes
    2^alpha * s independent of alpha; it is read with the largest refinement K
    in the denominator: s is the layer-wise step that covers the whole range,
    divided by 2^K, so that a channel with factor alpha_c = K gets the
    layer-wise step back and the others a finer one.  Returns e with s = 2^e."""
    if kmax < 0 or kmax > 4:
        raise ValueError("K lies in 0..4")
    return calibrate_act_exp(x, bits) - int(kmax)


def trip_quantize(x, bits: int, e: int, zp: int, alpha) -> np.ndarray:
    """Section 4.3, Eq.5: q[m,c] = CLIP(round(x[m,c] / (2^alpha[c] * s)) + zp, lo, hi)
    with s = 2^e shared by all channels and one factor alpha[c] per channel
    (column) of x.  Grid and rounding as in Eq.2."""
    x64 = _as_f64(x)
    alpha = _check_alpha(alpha, x64.shape[-1])
    lo, hi = grid_bounds(bits, zp)
    r = np.ldexp(x64, -(int(e) + alpha))             # exact; the factors run along the last axis
    q = np.clip(np.rint(r) + float(zp), float(lo), float(hi))
    return q.astype(np.int32)


def trip_dequantize(q, e: int, zp: int, alpha) -> np.ndarray:
    """Inverse map of Eq.5: x_hat[m,c] = (q[m,c] - zp) * 2^(e + alpha[c]), exact."""
    q = np.asarray(q, dtype=np.int64)
    alpha = _check_alpha(alpha, q.shape[-1])
    return np.ldexp((q - int(zp)).astype(np.float64), int(e) + alpha)


def trip_search(x, bits: int, e: int, zp: int, kmax: int) -> np.ndarray:
    """Section 4.3, Eq.8: alpha_c = argmin over {0..K} of
    || X_c - dequant(quant(X_c | alpha_c)) ||_2  for every channel c of x [M, C].

    The rounding term of Eq.8 is read as Eq.5's quantizer (clip included)
    followed by its inverse: without the clip the finest step would win for
    every channel and the search would be vacuous.  The squared norm is
    summed in float64 over the tokens m = 0, 1, .. in that order (every
    residual is exact; each square and each addition is rounded once), equal
    errors go to the smaller factor.  Returns int8 [C]."""
    if kmax < 0 or kmax > 4:
        raise ValueError("K lies in 0..4")
    x64 = _as_f64(x)
    if x64.ndim != 2:
        raise ValueError("x is [tokens, channels]")
    M, C = x64.shape
    err = np.zeros((kmax + 1, C), dtype=np.float64)
    for a in range(kmax + 1):
        al = np.full(C, a, dtype=np.int64)
        xh = trip_dequantize(trip_quantize(x, bits, e, zp, al), e, zp, al)
        with np.errstate(invalid="ignore", over="ignore"):
            r = x64 - xh                                  # exact; +-Inf stays +-Inf
            for m in range(M):
                err[a] = err[a] + r[m] * r[m]
    best = np.zeros(C, dtype=np.int8)
    best_err = err[0].copy()
    for a in range(1, kmax + 1):
        better = err[a] < best_err                        # strict: ties keep the smaller factor
        best = np.where(better, np.int8(a), best)
        best_err = np.where(better, err[a], best_err)
    return best


def gemm_int_trip(q, zp: int, wq, alpha) -> np.ndarray:
    """Section 4.4, the TRIP matrix product: the factor of input channel k moves
    onto row k of the weights,
        acc[m,n] = sum_k (q[m,k] - zp) * 2^alpha[k] * Wq[n,k],
    so that the activation keeps one layer-wise step.  int64, asserted to fit
    the 32-bit accumulator."""
    a = np.asarray(q, dtype=np.int64) - int(zp)
    b = np.asarray(wq, dtype=np.int64)
    if a.shape[-1] != b.shape[-1]:
        raise ValueError("K mismatch")
    alpha = _check_alpha(alpha, a.shape[-1])
    acc = (a << alpha[None, :]) @ b.T
    if acc.size and max(int(acc.max()), -int(acc.min())) > INT32_MAX:
        raise OverflowError("accumulator leaves int32")
    return acc


def linear_w4_trip(x, bits: int, e: int, zp: int, alpha, wq, sw):
    """The linear layer with TRIP factors: Eq.5 on the activation, the integer
    product with the factors folded in, and the per-channel dequantisation with
    the base step 2^e.  Returns (acc int64, y fp16)."""
    q = trip_quantize(x, bits, e, zp, alpha)
    acc = gemm_int_trip(q, zp, wq, alpha)
    return acc, dequant_out(acc, e, sw)


# --------------------------------------------------------------------------
# Eq.3  log2 quantizer on softmax probabilities, and the product with V
# --------------------------------------------------------------------------

def log2_quant(p, qmax: int) -> np.ndarray:
    """Section 4.1, Eq.3 with max|X| = 1: c = CLIP(round(-log2 p), 0, qmax).
    p = 0 gives +Inf before the clip, hence qmax.  -log2 p is never half-way
    between integers for a rational p, so the tie rule cannot matter; float64's
    log2 error is many orders below the distance of any fp16 value from a
    half-way point.  p must lie in [0, 1]."""
    p64 = _as_f64(p)
    if p64.size and (p64.min() < 0.0 or p64.max() > 1.0):
        raise ValueError("probabilities must lie in [0, 1]")
    with np.errstate(divide="ignore"):
        t = np.rint(-np.log2(p64))
    return np.clip(t, 0.0, float(qmax)).astype(np.int32)


def attn_v_rows(p_rows, n_valid, vq_h, qmax: int) -> np.ndarray:
    """Rows of the product of Eq.3's codes with one head's value matrix:
    A[r,d] = sum_{j < n_valid[r]} 2^(qmax - c[r,j]) * vq_h[j,d], c = Eq.3 of
    p_rows[r,j].  p_rows fp16 [R,S], vq_h int8 [S,D], n_valid int [R].
    The matrix product runs in float64, where it is exact: every term is an
    integer below 2^23 and a row has at most 2^30 of them.  Returned as int64,
    asserted to fit int32."""
    p_rows = np.asarray(p_rows)
    R, S = p_rows.shape
    if S >= (1 << 30):
        raise ValueError("row too long for an exact float64 sum")
    c = log2_quant(p_rows, qmax)
    wgt = np.ldexp(1.0, qmax - c)                             # 2^(qmax-c), exact
    keep = np.arange(S)[None, :] < np.asarray(n_valid, dtype=np.int64)[:, None]
    wgt = np.where(keep, wgt, 0.0)
    A = wgt @ np.asarray(vq_h, dtype=np.float64)
    if A.size and float(np.abs(A).max()) > INT32_MAX:
        raise OverflowError("accumulator leaves int32")
    return A.astype(np.int64)


def attn_v_log2(p, vq, e_v: int, qmax: int, causal: bool = True):
    """Softmax output quantized by Eq.3 and multiplied with the int8 value matrix
    (Section 5.1: log2 quantization for the softmax activation; Section 3.3:
    the attention-times-V product).

    p  : fp16 [H, S, S], row i = query i.  With `causal`, entries j > i are
         neither quantized nor multiplied.
    vq : int8 [H, S, D] on the grid of Eq.2 with scale 2^e_v.
    Returns (A, O):  A[h,i,d] = sum_j 2^(qmax - c[h,i,j]) * vq[h,j,d]  (int64,
    asserted < 2^31), and O[i, h*D + d] = fp16( A * 2^(e_v - qmax) )."""
    p = np.asarray(p)
    vq = np.asarray(vq)
    H, S, S2 = p.shape
    if S != S2 or vq.shape[:2] != (H, S):
        raise ValueError("shape mismatch")
    D = vq.shape[2]
    n_valid = np.arange(1, S + 1) if causal else np.full(S, S)
    A = np.stack([attn_v_rows(p[h], n_valid, vq[h], qmax) for h in range(H)])
    O = np.ldexp(A.astype(np.float64), int(e_v) - int(qmax))  # exact
    with np.errstate(over="ignore"):
        O = O.astype(np.float16)
    return A, np.ascontiguousarray(O.transpose(1, 0, 2).reshape(S, H * D))


def log2_codes_packed(p, qmax: int, causal: bool = True) -> np.ndarray:
    """The 4-bit codes of Eq.3, two per byte (low nibble = even j).  With
    `causal`, entries j > i carry code qmax (they stand for probability 0)."""
    p = np.asarray(p)
    c = log2_quant(p, qmax)
    if causal:
        S = p.shape[-1]
        c = np.where(np.tril(np.ones((S, S), dtype=bool))[None], c, qmax)
    return pack_nibbles(c)


# --------------------------------------------------------------------------
# attention from quantized Q and K: integer QK^T, softmax, Eq.3, times V
# --------------------------------------------------------------------------

def qk_scores(qq, kq) -> np.ndarray:
    """Section 4.2 lists QK among the quantized matrix products: s[h,i,j] =
    sum_d qq[h,i,d] * kq[h,j,d] on the integer codes of Eq.2 (int8: qq [H,S,D],
    kq [H,T,D]; T = S in the attention block).  int64, asserted to fit int32."""
    qq = np.asarray(qq, dtype=np.int64)
    kq = np.asarray(kq, dtype=np.int64)
    if qq.ndim != 3 or kq.ndim != 3 or qq.shape[0] != kq.shape[0] or qq.shape[2] != kq.shape[2]:
        raise ValueError("qq is [H, S, D], kq [H, T, D]")
    s = np.einsum("hid,hjd->hij", qq, kq)
    if s.size and max(int(s.max()), -int(s.min())) > INT32_MAX:
        raise OverflowError("score leaves int32")
    return s


def qk_log2_codes(qq, kq, e_q: int, e_k: int, qmax: int, causal: bool = True):
    """Softmax of the dequantized scores followed by Eq.3, without ever rounding
    the probabilities to fp16 (non-linear operators stay in floating point,
    Section 3.3; Eq.3 is used for the softmax output, Section 5.1):
        z[h,i,j] = s[h,i,j] * 2^(e_q + e_k) / sqrt(D)
        p        = softmax_j z        (over j <= i when causal)
        c        = CLIP(round(-log2 p), 0, qmax)
    computed in float64 as t = -log2 p = log2(sum_j 2^(z_j log2 e)) - z log2 e with
    the row maximum taken out.  Returns (c int32 [H,S,S], margin float64 [H,S,S]):
    margin is the distance of t from the nearest rounding boundary that can
    change the code (half-integers below qmax); an implementation that evaluates
    t in lower precision may differ from c only where margin is below its error.
    Masked entries (j > i, causal) carry code qmax and margin +Inf."""
    s = qk_scores(qq, kq).astype(np.float64)
    H, S, T = s.shape
    if causal and S != T:
        raise ValueError("the causal mask needs as many queries as keys")
    D = np.asarray(qq).shape[2]
    z2 = s * (2.0 ** (int(e_q) + int(e_k)) / np.sqrt(float(D)) * np.log2(np.e))   # logits in base-2 units
    if causal:
        z2 = np.where(np.tril(np.ones((S, S), dtype=bool))[None], z2, -np.inf)
    m = z2.max(axis=2, keepdims=True)
    L = m + np.log2(np.exp2(z2 - m).sum(axis=2, keepdims=True))
    with np.errstate(invalid="ignore"):
        t = L - z2                                               # -log2 p >= 0; +Inf where masked
    c = np.clip(np.rint(t), 0.0, float(qmax))
    # boundaries that matter: k + 0.5 for k = 0 .. qmax-1
    with np.errstate(invalid="ignore"):
        frac = np.abs(t - np.floor(t) - 0.5)
        margin = np.where(t < qmax, frac, t - (qmax - 0.5))
    margin = np.where(np.isfinite(t), margin, np.inf)
    return c.astype(np.int32), margin


def attn_v_from_codes(codes, vq, e_v: int, qmax: int, causal: bool = True):
    """The product of Eq.3's weights with the value matrix, from given codes:
    A[h,i,d] = sum_j 2^(qmax - c[h,i,j]) * vq[h,j,d] (j <= i when causal),
    O[i, h*D+d] = fp16(A * 2^(e_v - qmax)).  Same arithmetic as `attn_v_log2`."""
    codes = np.asarray(codes, dtype=np.int64)
    vq = np.asarray(vq)
    H, S, _ = codes.shape
    D = vq.shape[2]
    wgt = np.ldexp(1.0, (int(qmax) - codes).astype(np.int64))
    if causal:
        wgt = np.where(np.tril(np.ones((S, S), dtype=bool))[None], wgt, 0.0)
    A = np.einsum("hij,hjd->hid", wgt, vq.astype(np.float64))     # exact: integers below 2^53
    if A.size and float(np.abs(A).max()) > INT32_MAX:
        raise OverflowError("accumulator leaves int32")
    O = np.ldexp(A, int(e_v) - int(qmax))
    with np.errstate(over="ignore"):
        O = O.astype(np.float16)
    return A.astype(np.int64), np.ascontiguousarray(O.transpose(1, 0, 2).reshape(S, H * D))


def start_token_score_codes(codes, qmax: int) -> np.ndarray:
    """Token importance on the quantized attention map (Section 4.3: attention to
    the first token): score[i] = sum_h 2^(qmax - c[h,i,0]), an exact integer."""
    c0 = np.asarray(codes, dtype=np.int64)[:, :, 0]
    return (np.int64(1) << (int(qmax) - c0)).sum(axis=0)


# --------------------------------------------------------------------------
# token importance and pruning (Section 4.3, Eq.4; Section 5.2, Eq.9)
# --------------------------------------------------------------------------

def start_token_score(p) -> np.ndarray:
    """Importance of token i = its attention to the first (start) token
    (Section 4.3), summed over heads on the unquantized map.  Returned as the
    exact integer sum_h p[h,i,0] * 2^24 (every fp16 value times 2^24 is an
    integer), so the ranking has no rounding in it."""
    col = np.ldexp(_as_f64(np.asarray(p)[:, :, 0]), 24)
    t = col.sum(axis=0)
    assert np.all(t == np.floor(t))
    return t.astype(np.int64)


def progressive_ratio(beta: float, m: int) -> float:
    """Section 5.2, Eq.9: gamma = 1 - (1 - beta)^(1/m)."""
    return 1.0 - (1.0 - beta) ** (1.0 / m)


def n_keep(S: int, gamma: float) -> int:
    """Tokens that survive one pruning stage of ratio gamma: S - floor(S*gamma)."""
    return S - int(np.floor(S * gamma))


def prune_select(score, keep: int) -> np.ndarray:
    """Section 4.3, Eq.4: indices of the `keep` most important tokens; equal
    scores go to the lower index; the survivors stay in their original order."""
    score = np.asarray(score, dtype=np.int64)
    S = score.shape[0]
    if keep < 0 or keep > S:
        raise ValueError("keep outside 0..S")
    order = sorted(range(S), key=lambda i: (-int(score[i]), i))
    return np.array(sorted(order[:keep]), dtype=np.int32)


def prune_tokens(score, keep: int, x):
    """Eq.4: X^P = F^P(X), the rows of x at `prune_select`'s indices."""
    idx = prune_select(score, keep)
    return idx, np.asarray(x)[idx]


# --------------------------------------------------------------------------
# the same integer contraction in plain C (for sizes numpy's int64 is slow at)
# --------------------------------------------------------------------------

def gemm_int_c(q, wq, threads: int = 1) -> np.ndarray:
    """`gemm_int` with zp = 0 through the plain-C loops of agq_oracle_gemm.c
    (loop order m, n, k; 64-bit running sum checked against int32).  Needs
    oracle/build.py to have been run.  Returns int32 [M, N]."""
    import ctypes
    import os
    lib = ctypes.CDLL(os.path.join(os.path.dirname(os.path.abspath(__file__)), "libagq_oracle.so"))
    q = np.ascontiguousarray(q, dtype=np.int8)
    wq = np.ascontiguousarray(wq, dtype=np.int8)
    M, K = q.shape
    N, K2 = wq.shape
    if K != K2:
        raise ValueError("K mismatch")
    acc = np.empty((M, N), dtype=np.int32)
    fn = lib.agq_oracle_gemm_i8
    fn.restype = ctypes.c_int
    fn.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64,
                   ctypes.c_int64, ctypes.c_void_p, ctypes.c_int]
    bad = fn(q.ctypes.data, wq.ctypes.data, M, N, K, acc.ctypes.data, int(threads))
    if bad:
        raise OverflowError("accumulator leaves int32")
    return acc


def c_max_threads() -> int:
    import ctypes
    import os
    lib = ctypes.CDLL(os.path.join(os.path.dirname(os.path.abspath(__file__)), "libagq_oracle.so"))
    lib.agq_oracle_max_threads.restype = ctypes.c_int
    return int(lib.agq_oracle_max_threads())
