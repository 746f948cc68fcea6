"""Pins for the CPU oracle: each function is checked against something other
than itself - hand-worked values (tests/golden, with their citations), exact
integer / rational arithmetic, brute force on tiny inputs, invariants, and
special cases that reduce to a textbook product.  No GPU is used here."""
from __future__ import annotations

import os
from fractions import Fraction

import numpy as np
import pytest

from paper_2312_05693_amd import synth

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _rows(name):
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                yield line.split()


ALL_F16 = np.arange(0x10000, dtype=np.uint16).view(np.float16)
FINITE_F16 = ALL_F16[np.isfinite(ALL_F16.astype(np.float32))]


def f16_parts(h):
    """(sign, integer mantissa, exponent) with value = sign * mant * 2^exp, from
    the bit pattern alone."""
    b = int(np.asarray(h, dtype=np.float16).view(np.uint16))
    s = -1 if b >> 15 else 1
    ex = (b >> 10) & 0x1F
    fr = b & 0x3FF
    if ex == 0:
        return s, fr, -24
    return s, fr | 0x400, ex - 25


def f16_fraction(h) -> Fraction:
    s, m, x = f16_parts(h)
    return s * Fraction(m) * (Fraction(2) ** x)


def round_half_even(fr: Fraction) -> int:
    fl = fr.numerator // fr.denominator
    rem = fr - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        return fl + 1
    return fl


# ---------------------------------------------------------------- Eq.1 / Eq.2

def test_grid_bounds_eq1(oracle):
    assert oracle.grid_bounds(8, 0) == (-128, 127)
    assert oracle.grid_bounds(4, 0) == (-8, 7)
    assert oracle.grid_bounds(8, 128) == (0, 255)
    assert oracle.grid_bounds(4, 8) == (0, 15)


def test_quantize_golden_eq2(oracle):
    n = 0
    for x, e, bits, zp, want in _rows("eq2_uniform_examples.txt"):
        got = oracle.quantize_act(np.array([float(x)], dtype=np.float16), int(bits), int(e), int(zp))
        assert int(got[0]) == int(want), (x, e, bits, zp)
        n += 1
    assert n >= 25


def test_quantize_exact_rational_sample(oracle):
    # exact rational arithmetic with an explicit tie rule, on a stride of all
    # finite fp16 patterns plus every pattern near the clip points
    pick = FINITE_F16[::53]
    for bits in (4, 8):
        lo, hi = -(1 << (bits - 1)), (1 << (bits - 1)) - 1
        for e in (-8, -3, -1, 0, 1, 2, 5, 8):
            got = oracle.quantize_act(pick, bits, e, 0)
            for h, g in zip(pick, got):
                want = min(max(round_half_even(f16_fraction(h) / Fraction(2) ** e), lo), hi)
                assert int(g) == want


def test_quantize_exhaustive_integer_arithmetic(oracle):
    # all 63 488 finite fp16 values, e in -8..8, both widths, against a bit-level
    # integer implementation: value = mant * 2^ex, shift, round half to even
    bits16 = FINITE_F16.view(np.uint16).astype(np.int64)
    sign = np.where(bits16 >> 15, -1, 1)
    ex = (bits16 >> 10) & 0x1F
    fr = bits16 & 0x3FF
    mant = np.where(ex == 0, fr, fr | 0x400)
    p2 = np.where(ex == 0, -24, ex - 25)
    for bits in (4, 8):
        lo, hi = -(1 << (bits - 1)), (1 << (bits - 1)) - 1
        for e in range(-8, 9):
            sh = p2 - e                                  # value/2^e = mant * 2^sh
            up = np.where(sh >= 0, mant << np.clip(sh, 0, 40), 0)
            d = np.clip(-sh, 0, 62)
            fl = mant >> d
            rem = mant - (fl << d)
            half = np.where(d > 0, np.int64(1) << np.clip(d - 1, 0, 62), 0)
            rnd = fl + ((rem > half) | ((rem == half) & (d > 0) & (fl & 1 == 1))).astype(np.int64)
            mag = np.where(sh >= 0, up, rnd)
            want = np.clip(sign * mag, lo, hi)
            got = oracle.quantize_act(FINITE_F16, bits, e, 0)
            assert np.array_equal(got, want), (bits, e)


def test_quantize_invariants(oracle):
    x = np.sort(FINITE_F16.astype(np.float32)).astype(np.float16)
    for bits in (4, 8):
        qmax = (1 << (bits - 1)) - 1
        for e in (-4, 0, 3):
            q = oracle.quantize_act(x, bits, e, 0)
            assert np.all(np.diff(q) >= 0)                        # monotone
            x64 = x.astype(np.float64)
            inside = np.abs(x64) <= qmax * 2.0 ** e
            err = np.abs(x64 - oracle.dequantize_act(q, e))
            assert np.all(err[inside] <= 2.0 ** (e - 1))          # half a step
            qn = oracle.quantize_act((-x).astype(np.float16), bits, e, 0)
            assert np.array_equal(qn[inside], -q[inside])         # odd symmetry
            assert int(oracle.quantize_act(np.zeros(1, np.float16), bits, e, 0)[0]) == 0
            # unsigned grid with zp = 2^(b-1) is the signed grid shifted
            qu = oracle.quantize_act(x, bits, e, 1 << (bits - 1))
            assert np.array_equal(qu, q + (1 << (bits - 1)))
            # dequantised codes are fixed points of the quantizer
            xr = oracle.dequantize_act(q, e)
            ok = np.abs(xr) <= 65504
            q2 = oracle.quantize_act(xr[ok].astype(np.float16), bits, e, 0)
            assert np.array_equal(q2, q[ok])
    inf = np.array([np.inf, -np.inf], dtype=np.float16)
    assert oracle.quantize_act(inf, 8, 0, 0).tolist() == [127, -128]
    with pytest.raises(ValueError):
        oracle.quantize_act(np.array([np.nan], dtype=np.float16), 8, 0, 0)


def test_calibrate_bruteforce(oracle):
    rng = np.random.default_rng(5)
    cases = [synth.make_activation(8, 64, 2, s) for s in range(6)]
    cases += [(rng.standard_normal(50) * 10.0 ** rng.integers(-6, 4)).astype(np.float16) for _ in range(40)]
    cases += [np.array([v], dtype=np.float16) for v in (127.0, 127.5, 128.0, 63.5, 64.0, 7.0, 7.5, 6e-8, 65504.0)]
    for x in cases:
        amax = Fraction(float(np.abs(x.astype(np.float64)).max()))
        for bits in (4, 8):
            qmax = (1 << (bits - 1)) - 1
            e = oracle.calibrate_act_exp(x, bits)
            if amax == 0:
                assert e == 0
                continue
            want = next(c for c in range(-64, 64) if amax <= qmax * Fraction(2) ** c)
            assert e == want
            q = oracle.quantize_act(x, bits, e, 0)
            assert np.abs(q).max() <= qmax                        # nothing clips
            assert np.abs(q).max() >= (qmax + 1) // 2             # and e is tight
    assert oracle.calibrate_act_exp(np.zeros(4, np.float16), 8) == 0
    assert oracle.calibrate_act_exp(np.array([np.inf], np.float16), 8) == 10   # 2^16 <= 127*2^10


# ---------------------------------------------------------------- nibbles, weights

def test_nibble_roundtrip_all_values(oracle):
    for a in range(-8, 8):
        for b in range(-8, 8):
            byte = oracle.pack_nibbles(np.array([a, b]))
            assert int(byte[0]) == ((a & 0xF) | ((b & 0xF) << 4))
            assert oracle.unpack_nibbles(byte, signed=True).tolist() == [a, b]
    u = np.arange(16)
    assert oracle.unpack_nibbles(oracle.pack_nibbles(u), signed=False).tolist() == u.tolist()
    rng = np.random.default_rng(1)
    q = rng.integers(-8, 8, size=(5, 64))
    assert np.array_equal(oracle.unpack_nibbles(oracle.pack_nibbles(q)), q)
    with pytest.raises(ValueError):
        oracle.pack_nibbles(np.array([16, 0]))


def test_weight_rtn(oracle):
    # hand-worked row: max 0.7 -> sw = fp16(0.1) = 0.0999755859375
    wq, sw = oracle.quantize_weight_rtn(np.array([[0.7, -0.31, 0.12, 0.0], [0, 0, 0, 0]]))
    assert float(sw[0]) == 0.0999755859375 and float(sw[1]) == 1.0
    assert wq.tolist() == [[7, -3, 1, 0], [0, 0, 0, 0]]
    w = synth.make_weight(48, 256, 3)
    wq, sw = oracle.quantize_weight_rtn(w)
    assert wq.dtype == np.int8 and sw.dtype == np.float16
    assert np.all(np.abs(wq).max(axis=1) == 7) and wq.min() >= -8
    err = np.abs(w.astype(np.float64) - wq * sw.astype(np.float64)[:, None])
    assert np.all(err <= sw.astype(np.float64)[:, None] / 2 * (1 + 1e-12))
    wq2, sw2 = oracle.quantize_weight_rtn(w * 2)
    assert np.array_equal(wq2, wq) and np.array_equal(sw2.astype(np.float64), 2 * sw.astype(np.float64))
    # the input recipe's 4-bit weights are this quantizer applied to its float weights
    gq, gs = synth.make_weight_q4(48, 256, 3)
    assert np.array_equal(gq, wq) and np.array_equal(gs, sw)


# ---------------------------------------------------------------- integer product

def test_gemm_bruteforce_bigint(oracle):
    rng = np.random.default_rng(7)
    M, K, N = 5, 64, 12
    for zp, (lo, hi) in ((0, (-128, 128)), (128, (0, 256))):
        q = rng.integers(lo, hi, size=(M, K))
        w = rng.integers(-8, 8, size=(N, K))
        want = [[sum((int(q[m, k]) - zp) * int(w[n, k]) for k in range(K)) for n in range(N)] for m in range(M)]
        assert oracle.gemm_int(q, zp, w).tolist() == want
        if zp == 0:
            assert oracle.gemm_int_c(q, w, 1).tolist() == want
            assert oracle.gemm_int_c(q, w, 3).tolist() == want


def test_gemm_invariants(oracle):
    rng = np.random.default_rng(8)
    M, K, N = 33, 384, 80
    q = rng.integers(-128, 128, size=(M, K)).astype(np.int8)
    q2 = rng.integers(-60, 60, size=(M, K)).astype(np.int8)
    w = rng.integers(-8, 8, size=(N, K)).astype(np.int8)
    acc = oracle.gemm_int(q, 0, w)
    assert acc.shape == (M, N)
    assert np.array_equal(acc, oracle.gemm_int_c(q, w, 2))                  # C loops == numpy int64
    assert np.array_equal(acc, (q.astype(np.float64) @ w.T.astype(np.float64)).astype(np.int64))  # BLAS, exact here
    # linear in the activation
    assert np.array_equal(oracle.gemm_int(q.astype(np.int64) + q2, 0, w), acc + oracle.gemm_int(q2, 0, w))
    # one-hot weight rows pick activation columns (catches a transposed operand)
    cols = rng.choice(K, size=N, replace=False)
    eye = np.zeros((N, K), dtype=np.int8)
    eye[np.arange(N), cols] = 1
    assert np.array_equal(oracle.gemm_int(q, 0, eye), q[:, cols].astype(np.int64))
    assert np.array_equal(oracle.gemm_int_c(q, eye, 1), q[:, cols].astype(np.int32))
    # permuting K on both operands changes nothing
    perm = rng.permutation(K)
    assert np.array_equal(oracle.gemm_int(q[:, perm], 0, w[:, perm]), acc)
    # extreme operands reach the bound 128 * 8 * K exactly; it is below 2^24 for K < 16384
    Kb = 13824
    qe = np.full((1, Kb), -128, dtype=np.int8)
    we = np.full((2, Kb), -8, dtype=np.int8)
    assert oracle.gemm_int(qe, 0, we).tolist() == [[128 * 8 * Kb] * 2]
    assert oracle.gemm_int_c(qe, we, 1).tolist() == [[128 * 8 * Kb] * 2]
    assert 128 * 8 * Kb < 2 ** 24
    # zero point: (q - zp) enters the product, so shifting codes and zp together is neutral
    assert np.array_equal(oracle.gemm_int(q.astype(np.int64) + 128, 128, w), acc)


def test_gemm_overflow_is_caught(oracle):
    q = np.full((1, 1 << 22), -128, dtype=np.int8)
    w = np.full((1, 1 << 22), -8, dtype=np.int8)
    with pytest.raises(OverflowError):
        oracle.gemm_int_c(q, w, 1)


# ---------------------------------------------------------------- dequantisation

_F16_SORTED = np.sort(FINITE_F16.astype(np.float64))


def fraction_to_f16(v: Fraction) -> float:
    """Correctly rounded (nearest, ties to even mantissa) fp16 of a rational,
    by exact comparison with the two neighbouring fp16 values."""
    if v == 0:
        return 0.0
    i = int(np.searchsorted(_F16_SORTED, float(v)))
    cands = [_F16_SORTED[j] for j in range(max(i - 2, 0), min(i + 2, len(_F16_SORTED)))]
    best = min(cands, key=lambda c: abs(Fraction(float(c)) - v))
    ties = [c for c in cands if abs(Fraction(float(c)) - v) == abs(Fraction(float(best)) - v)]
    if len(ties) > 1:
        best = next(c for c in ties if (int(np.float16(c).view(np.uint16)) & 1) == 0)
    top = Fraction(65504) + Fraction(16)          # half-way to 2^16
    if abs(v) >= top:
        return float("inf") if v > 0 else float("-inf")
    return float(best)


def test_dequant_exact_rational(oracle):
    rng = np.random.default_rng(11)
    n = 400
    acc = np.concatenate([rng.integers(-2 ** 24, 2 ** 24, size=n - 8), [0, 1, -1, 3, 2 ** 24 - 1, -2 ** 24, 2047, 2049]])
    sw = np.abs(rng.standard_normal(n) * 0.02).astype(np.float16)
    sw[:5] = [1.0, 0.5, 6e-8, 65504.0, 0.010002]
    for e in (-6, -1, 0, 4):
        y = oracle.dequant_out(acc.reshape(1, n), e, sw)[0]
        for a, s, got in zip(acc, sw, y):
            want = fraction_to_f16(Fraction(int(a)) * f16_fraction(s) * Fraction(2) ** e)
            assert float(got) == want, (a, float(s), e)
    # one step of e doubles the result exactly (no overflow here); zero stays +0
    acc2 = rng.integers(-1000, 1000, size=(3, 16))
    sw2 = np.full(16, 0.01, dtype=np.float16)
    y0 = oracle.dequant_out(acc2, -2, sw2).astype(np.float64)
    y1 = oracle.dequant_out(acc2, -1, sw2).astype(np.float64)
    assert np.array_equal(y1, 2 * y0)
    z = oracle.dequant_out(np.zeros((1, 16), np.int64), 3, sw2)
    assert np.all(z.view(np.uint16) == 0)


def test_linear_power_of_two_is_exact_shift(oracle):
    # with unit weight scales the layer reproduces x_hat @ Wq^T exactly:
    # a power-of-two activation scale makes dequantisation a pure exponent shift
    x = synth.make_activation(6, 128, 2, 21)
    wq = np.random.default_rng(2).integers(-8, 8, size=(16, 128)).astype(np.int8)
    e = oracle.calibrate_act_exp(x, 8)
    acc, y = oracle.linear_w4(x, 8, e, 0, wq, np.ones(16, np.float16))
    xhat = oracle.dequantize_act(oracle.quantize_act(x, 8, e, 0), e)
    exact = xhat @ wq.T.astype(np.float64)
    assert np.array_equal(exact, np.ldexp(acc.astype(np.float64), e))
    assert np.array_equal(y, exact.astype(np.float16))


# ---------------------------------------------------------------- Eq.3

def test_log2_golden_eq3(oracle):
    n = 0
    for p, qmax, want in _rows("eq3_log2_examples.txt"):
        got = oracle.log2_quant(np.array([float(p)], dtype=np.float16), int(qmax))
        assert int(got[0]) == int(want), (p, qmax)
        n += 1
    assert n >= 14


def test_log2_exhaustive_bigint(oracle):
    # every fp16 in [0,1]: round(-log2 p) = n  <=>  2^-(2n+1) < p^2 < 2^-(2n-1),
    # decided with integers only (p = mant * 2^ex)
    ps = ALL_F16[: 0x3C00 + 1]
    assert float(ps[-1]) == 1.0
    for qmax in (15, 7):
        got = oracle.log2_quant(ps, qmax)
        for h, g in zip(ps, got):
            _, mant, ex = f16_parts(h)
            if mant == 0:
                want = qmax
            else:
                sq, sx = mant * mant, 2 * ex                 # p^2 = sq * 2^sx
                n = 0
                while not (sq << max(sx + 2 * n + 1, 0) > 1 << max(-(sx + 2 * n + 1), 0)):
                    n += 1                                    # first n with p^2 > 2^-(2n+1)
                want = min(n, qmax)
            assert int(g) == want, (float(h), qmax)
    with pytest.raises(ValueError):
        oracle.log2_quant(np.array([1.5], np.float16), 15)


def test_attn_v_special_cases(oracle):
    rng = np.random.default_rng(13)
    H, S, D, qmax = 2, 24, 8, 15
    vq = rng.integers(-128, 128, size=(H, S, D)).astype(np.int8)
    # probabilities that are exact powers of two >= 2^-qmax: Eq.3 loses nothing,
    # so the result is the textbook product P @ V
    k = rng.integers(0, qmax + 1, size=(H, S, S))
    p = np.ldexp(1.0, -k).astype(np.float16)
    A, O = oracle.attn_v_log2(p, vq, -3, qmax, causal=False)
    exact = np.einsum("hij,hjd->hid", p.astype(np.float64), vq.astype(np.float64))
    assert np.array_equal(np.ldexp(A.astype(np.float64), -qmax), exact)
    assert np.array_equal(O, np.ldexp(exact, -3).transpose(1, 0, 2).reshape(S, H * D).astype(np.float16))
    # causal: entries above the diagonal are ignored whatever they hold
    Ac, _ = oracle.attn_v_log2(p, vq, -3, qmax, causal=True)
    p_low = np.where(np.tril(np.ones((S, S), bool))[None], p, np.float16(0))
    want = np.einsum("hij,hjd->hid", np.where(np.tril(np.ones((S, S), bool))[None], p_low.astype(np.float64), 0.0),
                     vq.astype(np.float64))
    assert np.array_equal(np.ldexp(Ac.astype(np.float64), -qmax), want)
    # one-hot row returns that row of V times 2^qmax; row 0 of a causal map is V[0]
    onehot = np.zeros((1, 4, 4), np.float16)
    onehot[0, np.arange(4), [0, 1, 0, 2]] = 1.0
    v4 = rng.integers(-128, 128, size=(1, 4, 3)).astype(np.int8)
    A1, O1 = oracle.attn_v_log2(onehot, v4, 0, 7, causal=True)
    # zeros carry code qmax, i.e. weight 1 (probability 2^-qmax), inside the causal part
    for i, j in enumerate([0, 1, 0, 2]):
        want = 128 * v4[0, j].astype(np.int64) + sum(v4[0, jj].astype(np.int64) for jj in range(i + 1) if jj != j)
        assert np.array_equal(A1[0, i], want)
    # brute force, pure Python, tiny
    pr = synth.make_attention(1, 6, 4, 3)[0]
    vv = rng.integers(-128, 128, size=(1, 6, 4)).astype(np.int8)
    Ab, _ = oracle.attn_v_log2(pr, vv, 0, 15, causal=True)
    codes = oracle.log2_quant(pr, 15)
    for i in range(6):
        for d in range(4):
            assert int(Ab[0, i, d]) == sum((1 << (15 - int(codes[0, i, j]))) * int(vv[0, j, d]) for j in range(i + 1))


def test_attn_v_rowsum_bound(oracle):
    # for a genuine softmax row, sum_j 2^-c_j <= sqrt(2) * sum_j p_j + n * 2^-qmax,
    # which keeps the accumulator far inside int32 (and inside 2^24)
    p, _ = synth.make_attention(2, 96, 16, 9)
    c = oracle.log2_quant(p, 15)
    w = np.where(np.tril(np.ones((96, 96), bool))[None], np.ldexp(1.0, -c), 0.0)
    assert np.all(w.sum(axis=2) <= np.sqrt(2) * 1.001 + np.arange(1, 97)[None] * 2.0 ** -15)


def test_log2_codes_packed(oracle):
    p, _ = synth.make_attention(1, 8, 4, 2)
    b = oracle.log2_codes_packed(p, 15, causal=True)
    c = oracle.unpack_nibbles(b, signed=False)
    full = oracle.log2_quant(p, 15)
    for i in range(8):
        assert c[0, i, : i + 1].tolist() == full[0, i, : i + 1].tolist()
        assert np.all(c[0, i, i + 1:] == 15)


# ---------------------------------------------------------------- importance, pruning

def test_start_token_score_exact(oracle):
    p, _ = synth.make_attention(3, 16, 4, 5)
    t = oracle.start_token_score(p)
    for i in range(16):
        want = sum(f16_fraction(p[h, i, 0]) for h in range(3)) * 2 ** 24
        assert want.denominator == 1 and int(t[i]) == int(want)
    assert int(t[0]) == 3 << 24          # the first token attends only to itself


def test_prune_select(oracle):
    rng = np.random.default_rng(17)
    for _ in range(30):
        S = int(rng.integers(1, 40))
        score = rng.integers(0, 6, size=S)          # many ties
        keep = int(rng.integers(0, S + 1))
        idx = oracle.prune_select(score, keep)
        assert len(idx) == keep and np.all(np.diff(idx) > 0)
        # brute force: token i survives iff fewer than `keep` tokens beat it
        beats = [sum(1 for j in range(S) if score[j] > score[i] or (score[j] == score[i] and j < i)) for i in range(S)]
        assert idx.tolist() == [i for i in range(S) if beats[i] < keep]
    # against a stable library sort
    score = rng.integers(0, 1000, size=200)
    want = np.sort(np.argsort(-score, kind="stable")[:77])
    assert np.array_equal(oracle.prune_select(score, 77), want)
    x = rng.standard_normal((200, 5)).astype(np.float16)
    idx, xo = oracle.prune_tokens(score, 77, x)
    assert np.array_equal(xo, x[want])
    # the start token always survives a causal map (its own score is maximal)
    p, _ = synth.make_attention(2, 32, 4, 1)
    t = oracle.start_token_score(p)
    assert 0 in oracle.prune_select(t, 1).tolist()


def test_progressive_ratio_eq9(oracle):
    for beta, m, want in _rows("eq9_progressive_ratio.txt"):
        g = oracle.progressive_ratio(float(beta), int(m))
        assert abs(g - float(want)) < 1e-12
        assert abs((1 - g) ** int(m) - (1 - float(beta))) < 1e-12
    assert oracle.n_keep(2048, 0.5) == 1024
    assert oracle.n_keep(10, 0.25) == 8          # 10 - floor(2.5)
    assert oracle.n_keep(7, 0.0) == 7


# ---------------------------------------------------------------- Eq.5 - Eq.8 (TRIP)

def test_trip_golden_eq5_eq8(oracle):
    rows = [[float(v) for v in r] for r in _rows("eq8_trip_examples.txt")]
    x = np.array([r[:3] for r in rows], dtype=np.float16).T          # [3 tokens, 4 channels]
    bits, e, zp, kmax = 4, -2, 0, 2
    for a in range(kmax + 1):
        al = np.full(x.shape[1], a)
        xh = oracle.trip_dequantize(oracle.trip_quantize(x, bits, e, zp, al), e, zp, al)
        err = ((x.astype(np.float64) - xh) ** 2).sum(axis=0)
        assert err.tolist() == [r[3 + a] for r in rows]
    assert oracle.trip_search(x, bits, e, zp, kmax).tolist() == [int(r[6]) for r in rows]


def test_trip_quantize_reduces_to_eq2(oracle):
    rng = np.random.default_rng(21)
    x = (rng.standard_normal((7, 40)) * 6).astype(np.float16)
    for bits, zp in ((8, 0), (4, 0), (8, 100), (4, 9)):
        # all factors zero: Eq.5 is Eq.2
        assert np.array_equal(oracle.trip_quantize(x, bits, -3, zp, np.zeros(40, dtype=int)),
                              oracle.quantize_act(x, bits, -3, zp))
        # one common factor a: Eq.2 with the step 2^(e+a)
        for a in (1, 4):
            assert np.array_equal(oracle.trip_quantize(x, bits, -3, zp, np.full(40, a)),
                                  oracle.quantize_act(x, bits, -3 + a, zp))
        # mixed factors: every column on its own against Eq.2 with that column's step
        alpha = rng.integers(0, 5, size=40)
        q = oracle.trip_quantize(x, bits, -3, zp, alpha)
        for c in range(40):
            assert np.array_equal(q[:, c], oracle.quantize_act(x[:, c], bits, -3 + int(alpha[c]), zp))
        xh = oracle.trip_dequantize(q, -3, zp, alpha)
        for c in range(40):
            assert np.array_equal(xh[:, c], oracle.dequantize_act(q[:, c], -3 + int(alpha[c]), zp))


def test_trip_base_exp(oracle):
    x = np.array([[1.0, -100.0], [0.5, 3.0]], dtype=np.float16)
    e_layer = oracle.calibrate_act_exp(x, 8)
    assert 127 * 2.0 ** e_layer >= 100.0 > 127 * 2.0 ** (e_layer - 1)
    for k in range(5):
        assert oracle.trip_base_exp(x, 8, k) == e_layer - k
    # a channel with the factor K gets the layer-wise step back
    assert np.array_equal(oracle.trip_quantize(x, 8, e_layer - 3, 0, np.array([3, 3])), oracle.quantize_act(x, 8, e_layer, 0))


def test_trip_search_bruteforce_rational(oracle):
    """Eq.8 in exact rational arithmetic, pure Python, on small inputs."""
    rng = np.random.default_rng(22)
    M, C = 9, 24
    x = (rng.standard_normal((M, C)) * np.where(rng.random(C) < 0.3, 12.0, 1.0)).astype(np.float16)
    for bits, e, zp, kmax in ((8, -7, 0, 4), (4, -3, 0, 3), (8, -6, 77, 4), (4, -2, 5, 2)):
        lo, hi = oracle.grid_bounds(bits, zp)
        got = oracle.trip_search(x, bits, e, zp, kmax)
        for c in range(C):
            errs = []
            for a in range(kmax + 1):
                step = Fraction(2) ** (e + a)
                tot = Fraction(0)
                for m in range(M):
                    v = f16_fraction(x[m, c])
                    q = min(max(round_half_even(v / step) + zp, lo), hi)
                    tot += (v - (q - zp) * step) ** 2
                errs.append(tot)
            best = min(errs)
            # the float64 sums of the oracle may differ from the exact ones in the last
            # bits: the factor it picked must be optimal up to that, and exactly the
            # first optimum when the optimum is separated
            assert errs[int(got[c])] <= best * (1 + Fraction(1, 10 ** 12))
            sep = [a for a in range(kmax + 1) if errs[a] <= best * (1 + Fraction(1, 10 ** 9))]
            if len(sep) == 1 or all(errs[a] == best for a in sep):
                assert int(got[c]) == sep[0]


def test_trip_search_properties(oracle):
    rng = np.random.default_rng(23)
    M, C, bits, kmax = 64, 32, 8, 4
    base = rng.standard_normal((M, C))
    x = base.astype(np.float16)
    e = oracle.trip_base_exp(x, bits, kmax)
    a0 = oracle.trip_search(x, bits, e, 0, kmax)
    # values that all sit on the finest grid without clipping: factor 0 for every channel
    on_grid = (rng.integers(-127, 128, size=(M, C)) * 2.0 ** e).astype(np.float16)
    assert oracle.trip_search(on_grid, bits, e, 0, kmax).tolist() == [0] * C
    # scaling a channel up by 2^j moves its best factor up by exactly j (the residuals
    # scale with it), as long as the result still lies in 0..K
    x2 = x.copy()
    x2[:, :8] = (base[:, :8].astype(np.float16).astype(np.float64) * 4.0).astype(np.float16)
    a2 = oracle.trip_search(x2, bits, e, 0, kmax)
    for c in range(8):
        if a0[c] + 2 <= kmax:
            assert a2[c] == a0[c] + 2
    assert np.array_equal(a2[8:], a0[8:])                     # channels are independent
    # a channel whose magnitudes need the layer-wise step picks the largest factor
    big = x.copy()
    big[:, 3] = (base[:, 3] * 30).astype(np.float16)
    eb = oracle.trip_base_exp(big, bits, kmax)
    ab = oracle.trip_search(big, bits, eb, 0, kmax)
    assert ab[3] == kmax and ab.max() == kmax and (ab[np.arange(C) != 3] < kmax).all()
    # token order matters only through float64 rounding: a reversed tensor gives the same factors here
    assert np.array_equal(oracle.trip_search(x[::-1].copy(), bits, e, 0, kmax), a0)
    # +-Inf makes every candidate's error infinite: the smaller factor is kept
    xi = x.copy()
    xi[5, 2] = np.inf
    assert oracle.trip_search(xi, bits, e, 0, kmax)[2] == 0


def test_trip_gemm_folding_identity(oracle):
    """Section 4.4: the factors move onto the weight rows.  The folded product through
    the plain integer contraction, a pure-Python big-integer sum, and the factor-free
    special case pin `gemm_int_trip`."""
    rng = np.random.default_rng(24)
    M, K, N = 6, 96, 10
    w = rng.integers(-8, 8, size=(N, K))
    alpha = np.where(rng.random(K) < 0.2, rng.integers(1, 5, size=K), 0)
    for zp, (lo, hi) in ((0, (-128, 128)), (128, (0, 256))):
        q = rng.integers(lo, hi, size=(M, K))
        got = oracle.gemm_int_trip(q, zp, w, alpha)
        assert np.array_equal(got, oracle.gemm_int(q, zp, w * (1 << alpha)[None, :]))
        want = [[sum((int(q[m, k]) - zp) * (1 << int(alpha[k])) * int(w[n, k]) for k in range(K)) for n in range(N)]
                for m in range(M)]
        assert got.tolist() == want
        assert np.array_equal(oracle.gemm_int_trip(q, zp, w, np.zeros(K, dtype=int)), oracle.gemm_int(q, zp, w))
    with pytest.raises(ValueError):
        oracle.gemm_int_trip(q, 0, w, np.full(K, 5))


def test_trip_linear_approximates_the_real_product(oracle):
    """With outlier channels the TRIP layer must be closer to the float product than the
    layer-wise quantizer at the same bits: the reason the factors exist (Section 4.3)."""
    x = synth.make_activation(32, 512, 4, seed=3)
    w = synth.make_weight(48, 512, seed=3)
    wq, sw = oracle.quantize_weight_rtn(w)
    ref = x.astype(np.float64) @ (wq.astype(np.float64) * sw.astype(np.float64)[:, None]).T
    bits, kmax = 8, 4
    e_layer = oracle.calibrate_act_exp(x, bits)
    _, y_plain = oracle.linear_w4(x, bits, e_layer, 0, wq, sw)
    e = oracle.trip_base_exp(x, bits, kmax)
    alpha = oracle.trip_search(x, bits, e, 0, kmax)
    acc, y_trip = oracle.linear_w4_trip(x, bits, e, 0, alpha, wq, sw)
    # the folded accumulator equals the dequantized activation times the integer weights
    xh = oracle.trip_dequantize(oracle.trip_quantize(x, bits, e, 0, alpha), e, 0, alpha)
    assert np.array_equal(np.ldexp(acc.astype(np.float64), e), xh @ wq.astype(np.float64).T)
    err_plain = np.abs(y_plain.astype(np.float64) - ref).mean()
    err_trip = np.abs(y_trip.astype(np.float64) - ref).mean()
    assert err_trip < 0.5 * err_plain
    assert 0 < (alpha > 0).sum() < 64                         # the outlier channels and few others


# ---------------------------------------------------------------- attention from quantized Q and K

def test_qk_scores_bruteforce(oracle):
    rng = np.random.default_rng(31)
    H, S, D = 2, 5, 12
    q = rng.integers(-128, 128, size=(H, S, D)).astype(np.int8)
    k = rng.integers(-128, 128, size=(H, S, D)).astype(np.int8)
    want = [[[sum(int(q[h, i, d]) * int(k[h, j, d]) for d in range(D)) for j in range(S)] for i in range(S)] for h in range(H)]
    assert oracle.qk_scores(q, k).tolist() == want
    # one-hot keys pick query components (catches a transposed operand)
    eye = np.zeros((1, 4, 12), dtype=np.int8)
    eye[0, np.arange(4), [3, 0, 7, 11]] = 1
    assert np.array_equal(oracle.qk_scores(q[:1, :4], eye)[0], q[0, :4][:, [3, 0, 7, 11]].astype(np.int64))


def test_qk_log2_codes_closed_forms(oracle):
    H, S, D, qmax = 1, 40, 16, 15
    # equal scores: p = 1/n over the n allowed keys, code = round(log2 n) (n = i + 1 when causal)
    q = np.zeros((H, S, D), dtype=np.int8)
    k = np.ones((H, S, D), dtype=np.int8)
    c, margin = oracle.qk_log2_codes(q, k, 0, 0, qmax, causal=True)
    for i in range(S):
        want = min(int(np.rint(np.log2(i + 1))), qmax)
        assert (c[0, i, : i + 1] == want).all() and (c[0, i, i + 1:] == qmax).all()
        assert np.isinf(margin[0, i, i + 1:]).all()
    c, _ = oracle.qk_log2_codes(q, k, 0, 0, qmax, causal=False)
    assert (c == int(np.rint(np.log2(S)))).all()
    # one key far ahead of the rest: its code is 0, the others' the clipped distance in bits
    q = np.full((H, S, D), 8, dtype=np.int8)
    k = np.zeros((H, S, D), dtype=np.int8)
    k[0, 3] = 8                                            # s = 8 * 8 * 16 = 1024 for key 3, 0 elsewhere
    e = -2                                                 # z = 1024 * 2^-4 / 4 = 16 nats = 23.08 bits
    c, margin = oracle.qk_log2_codes(q, k, e, e, qmax, causal=False)
    assert (c[0, :, 3] == 0).all() and (np.delete(c[0], 3, axis=1) == qmax).all()
    c, _ = oracle.qk_log2_codes(q, k, e - 1, e, 31, causal=False)   # half the logit: 11.54 bits
    assert (c[0, :, 3] == 0).all() and (np.delete(c[0], 3, axis=1) == 12).all()


def test_qk_log2_codes_against_library_and_rationals(oracle):
    from scipy.special import log_softmax
    rng = np.random.default_rng(32)
    H, S, D, qmax = 3, 24, 32, 15
    q = rng.integers(-40, 40, size=(H, S, D)).astype(np.int8)
    k = rng.integers(-40, 40, size=(H, S, D)).astype(np.int8)
    e_q, e_k = -3, -4
    for causal in (True, False):
        c, margin = oracle.qk_log2_codes(q, k, e_q, e_k, qmax, causal)
        z = oracle.qk_scores(q, k).astype(np.float64) * 2.0 ** (e_q + e_k) / np.sqrt(D)
        if causal:
            z = np.where(np.tril(np.ones((S, S), dtype=bool))[None], z, -np.inf)
        t = -log_softmax(z, axis=2) / np.log(2.0)           # library route to -log2 p
        want = np.clip(np.rint(t), 0, qmax)
        sure = margin > 1e-9
        assert np.array_equal(c[sure], want[sure].astype(np.int32)) and sure.mean() > 0.999
        # margin is what it says: moving t by less than the margin never changes the code
        fin = np.isfinite(t) & (margin < np.inf)
        for sign in (-1.0, 1.0):
            moved = np.clip(np.rint(t[fin] + sign * 0.999 * margin[fin]), 0, qmax)
            assert np.array_equal(moved, c[fin])
        # softmax is invariant to a per-row shift of the scores: add a constant vector to every key
        # of a head whose query components sum to zero -> s changes by 0; instead check scaling:
        # doubling e_q + e_k by two steps equals quadrupling the scores
        c2, _ = oracle.qk_log2_codes((q.astype(np.int16) * 2).clip(-128, 127).astype(np.int8), (k.astype(np.int16) * 2).astype(np.int8),
                                     e_q - 1, e_k - 1, qmax, causal)
        assert np.array_equal(c2, c)
    # exact rational check of one row: p_j = 2^(a_j) / sum with integer bit-logits
    qq = np.zeros((1, 4, 16), dtype=np.int8)
    kk = np.zeros((1, 4, 16), dtype=np.int8)
    qq[0, :, 0] = 1
    kk[0, :, 0] = [0, 1, 2, 3]
    # choose scale so that z log2 e is an integer number of bits: impossible exactly; so compare via fractions of exp
    c, _ = oracle.qk_log2_codes(qq, kk, 2, 0, 15, causal=False)    # z = s * 4 / 4 = s nats
    from math import e as E, log2
    denom = sum(E ** s for s in range(4))
    assert c[0, 0].tolist() == [min(int(np.rint(-log2(E ** s / denom))), 15) for s in range(4)]


def test_attn_v_from_codes(oracle):
    rng = np.random.default_rng(33)
    H, S, D, qmax = 2, 9, 8, 15
    codes = rng.integers(0, qmax + 1, size=(H, S, S))
    v = rng.integers(-128, 128, size=(H, S, D)).astype(np.int8)
    for causal in (True, False):
        A, O = oracle.attn_v_from_codes(codes, v, -4, qmax, causal)
        for h in range(H):
            for i in range(S):
                js = range(i + 1) if causal else range(S)
                for d in range(D):
                    want = sum((1 << (qmax - int(codes[h, i, j]))) * int(v[h, j, d]) for j in js)
                    assert int(A[h, i, d]) == want
                    assert O[i, h * D + d] == np.float16(want * 2.0 ** (-4 - qmax))
    # consistent with the fp16-probability path when the codes are the same
    p = synth.make_attention(2, 16, 8, seed=5)[0]
    c = oracle.log2_quant(p, qmax)
    vq = rng.integers(-128, 128, size=(2, 16, 8)).astype(np.int8)
    A1, O1 = oracle.attn_v_log2(p, vq, -3, qmax, causal=True)
    A2, O2 = oracle.attn_v_from_codes(c, vq, -3, qmax, causal=True)
    assert np.array_equal(A1, A2) and np.array_equal(O1.view(np.uint16), O2.view(np.uint16))
    # importance on the quantized map
    sc = oracle.start_token_score_codes(codes, qmax)
    assert sc.tolist() == [sum(1 << (qmax - int(codes[h, i, 0])) for h in range(H)) for i in range(S)]


def test_start_token_score_codes_pins(oracle):
    """Section 4.3: importance = attention paid to the first token, here read on the quantized map.
    Pinned by a hand-worked map with literal scores (other columns, heads and rows carry different
    codes, so a wrong column, axis or sign of the exponent changes the numbers), by probabilities that
    are exact powers of two (the score must be the unquantized map's score, rescaled), and by the two
    extreme heads."""
    # codes[h, i, j]; column 0 is what counts.  qmax = 15:
    #   token 0: heads give 2^15 + 2^15           = 65536
    #   token 1: 2^(15-3) + 2^(15-1)              = 20480
    #   token 2: 2^(15-15) + 2^(15-14)            = 3
    codes = np.array([[[0, 9, 2], [3, 0, 9], [15, 1, 0]],
                      [[0, 4, 4], [1, 7, 7], [14, 0, 3]]])
    assert oracle.start_token_score_codes(codes, 15).tolist() == [65536, 20480, 3]
    # qmax = 7 (Eq.3's signed 4-bit range): 2^7 + 2^7, 2^4 + 2^6, 2^0 + 2^1 with codes 7 and 6 in the last row
    codes7 = np.array([[[0, 5], [3, 0], [7, 1]], [[0, 2], [1, 7], [6, 0]]])
    assert oracle.start_token_score_codes(codes7, 7).tolist() == [256, 80, 3]
    # one head only, one token only: shapes must not be confused
    assert oracle.start_token_score_codes(np.array([[[2, 0, 0, 0]]]), 15).tolist() == [8192]
    # probabilities that are powers of two no smaller than 2^-qmax quantize without error (Eq.3), so the
    # score on the codes is the score on the probabilities, 2^24 p summed over heads, in units of 2^qmax
    rng = np.random.default_rng(71)
    for qmax in (15, 7):
        H, S = 5, 12
        c = rng.integers(0, qmax + 1, size=(H, S, S))
        p = np.ldexp(1.0, -c).astype(np.float16)
        assert np.array_equal(oracle.log2_quant(p, qmax), c)
        got = oracle.start_token_score_codes(oracle.log2_quant(p, qmax), qmax)
        assert np.array_equal(got << (24 - qmax), oracle.start_token_score(p))
        # and both equal the plain column sum of the map
        assert np.array_equal(got, (p[:, :, 0].astype(np.float64).sum(axis=0) * 2.0 ** qmax).astype(np.int64))
    # every head looks only at the first token: H * 2^qmax; no head does (p = 0 -> code qmax): H
    H, S = 4, 6
    p = np.zeros((H, S, S), dtype=np.float16)
    assert oracle.start_token_score_codes(oracle.log2_quant(p, 15), 15).tolist() == [H] * S
    p[:, :, 0] = 1.0
    assert oracle.start_token_score_codes(oracle.log2_quant(p, 15), 15).tolist() == [H << 15] * S
    # monotone: lowering one head's code for a token raises that token's score and no other's
    base = oracle.start_token_score_codes(codes, 15)
    codes2 = codes.copy()
    codes2[1, 1, 0] = 0
    moved = oracle.start_token_score_codes(codes2, 15)
    assert moved[1] == base[1] - (1 << 14) + (1 << 15) and moved[0] == base[0] and moved[2] == base[2]
