"""GPU parity of one block of the quantized pipeline (agq_block_forward /
agq_block_calibrate) against the block oracle.

Every stage is checked on the tensors that actually flowed through the GPU call:
the oracle's single function, applied to the GPU's own input of that stage, must
reproduce the GPU's output of that stage - bit for bit for integers and, because
the fp16 operators round a float64 result once on both sides, bit for bit for
fp16 as well (the bar is 1e-3 relative; exact equality is what is observed and
asserted).  The attention codes are compared where the oracle's -log2 p is
further than CODE_MARGIN from a rounding boundary (the kernel evaluates it in
fp32); everything after them follows exactly from the GPU's own codes.  When no
code differs, the whole chain equals the oracle's chain bit for bit."""
from __future__ import annotations

import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from paper_2312_05693_amd import synth  # noqa: E402
from test_gpu_parity import CODE_MARGIN, dev, host, unpack_codes  # noqa: E402

EPS = 1e-5


@pytest.fixture(scope="module")
def agq():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2312_05693_amd import binding
    binding.lib()
    return binding


@pytest.fixture(scope="module")
def blk_oracle(oracle):
    from oracle import agq_block_oracle
    return agq_block_oracle


def same(a, b):
    a, b = np.asarray(a), np.asarray(b)
    return a.shape == b.shape and np.array_equal(a.view(np.uint16) if a.dtype == np.float16 else a,
                                                 b.view(np.uint16) if b.dtype == np.float16 else b)


def make_inputs(S, d, H, F, seed, pos=None, P=None):
    x = synth.make_activation(S, d, max(1, d // 128), seed)
    pos = np.arange(S, dtype=np.int32) if pos is None else np.asarray(pos, dtype=np.int32)
    cos, sin = synth.rope_tables(P or int(pos.max()) + 1, d // H)
    return x, pos, cos, sin, synth.make_block_weights(d, H, F, seed)


SITE_OF = dict(q="attn_in", k="attn_in", v="attn_in", o="attn_out", gate="mlp_in", up="mlp_in", down="mlp_act")


def upload_weights(agq, w, alphas=None):
    """Device weights; with `alphas` (site -> factors) the projections of those sites become TRIP blobs.
    Returns the dict for make_block and, per site with factors, the number of extra chunks."""
    out = {"g_attn": dev(w["g_attn"]), "g_mlp": dev(w["g_mlp"])}
    trip = {}
    for n in agq.BLOCK_PROJ:
        alpha = (alphas or {}).get(SITE_OF[n])
        if alpha is None:
            out["w_" + n] = agq.pack_w4(dev(w["w_" + n]))
        else:
            out["w_" + n], trip[SITE_OF[n]] = agq.pack_w4_trip(dev(w["w_" + n]), alpha)
        out["s_" + n] = dev(w["s_" + n])
    return (out, trip) if alphas is not None else out


def gpu_tensors(agq, blk, L, ws, S, keep, names=None):
    torch.cuda.synchronize()
    return {n: agq.block_tensor(blk, L, ws, n, S, keep).cpu().numpy() for n in (names or agq.BLOCK_TENSORS)
            if n not in ("q_rot", "k_rot")}


def check_stages(agq, oracle, B, w, H, qmax, bits_o, x, pos, cos, sin, keep, exps, g, x_out, pos_out, alphas=None):
    """g: the GPU's intermediates.  Returns True when the GPU's attention codes equal the oracle's."""
    S, d = x.shape
    D, sp = d // H, g["o"].shape[0]

    def lin(t, bits, e, n):
        alpha = (alphas or {}).get(SITE_OF[n])
        if alpha is not None:
            return oracle.linear_w4_trip(t, bits, e, 0, alpha, w["w_" + n], w["s_" + n])[1]
        return oracle.linear_w4(t, bits, e, 0, w["w_" + n], w["s_" + n])[1]
    assert same(g["h1"], B.rmsnorm(x, w["g_attn"], EPS)), "h1"
    for n in ("q", "k", "v"):
        assert same(g[n], lin(g["h1"], 8, exps["e_attn_in"], n)), n
    assert same(g["q_q"], B.heads_int8(B.rope(g["q"], pos, cos, sin, H), H, exps["e_q"], sp)), "q_q"
    assert same(g["k_q"], B.heads_int8(B.rope(g["k"], pos, cos, sin, H), H, exps["e_k"], sp)), "k_q"
    assert same(g["v_q"], B.heads_int8(g["v"], H, exps["e_v"], sp)), "v_q"
    # attention: the block's o and score are what the attention entry point returns for these operands ...
    o2, codes, score2 = agq.qk_log2_softmax(dev(g["q_q"]), dev(g["k_q"]), dev(g["v_q"]), exps["e_q"], exps["e_k"],
                                            exps["e_v"], qmax=qmax, causal=True, want_codes=True, want_score=True)
    assert same(g["o"], host(o2)) and same(g["score"], host(score2)), "attention"
    # ... whose codes are the oracle's outside the margin, and o / score follow exactly from the codes
    got_c = unpack_codes(host(codes), sp)
    want_c, margin = oracle.qk_log2_codes(g["q_q"], g["k_q"], exps["e_q"], exps["e_k"], qmax, True)
    sure = margin > CODE_MARGIN
    assert np.array_equal(got_c[sure], want_c[sure]) and np.abs(got_c - want_c).max() <= 1, "codes"
    tri = np.tril(np.ones((sp, sp), dtype=bool))[None]
    got_cm = np.where(tri, got_c, qmax)
    assert same(g["o"], oracle.attn_v_from_codes(got_cm, g["v_q"], exps["e_v"], qmax, True)[1]), "o"
    assert np.array_equal(g["score"].astype(np.int64), oracle.start_token_score_codes(got_cm, qmax)), "score"
    # pruning
    idx = oracle.prune_select(g["score"][:S], keep)
    assert np.array_equal(g["idx"], idx), "idx"
    assert same(g["o_kept"][:keep], g["o"][idx]), "o_kept"
    assert same(g["attn_out"], lin(g["o_kept"][:keep], bits_o, exps["e_attn_out"], "o")), "attn_out"
    assert same(g["x1"], B.residual_add(x[idx], g["attn_out"])), "x1"
    assert np.array_equal(pos_out, pos[idx]), "pos_out"
    assert same(g["h2"], B.rmsnorm(g["x1"], w["g_mlp"], EPS)), "h2"
    assert same(g["gate"], lin(g["h2"], 8, exps["e_mlp_in"], "gate")), "gate"
    assert same(g["up"], lin(g["h2"], 8, exps["e_mlp_in"], "up")), "up"
    assert same(g["act"], B.swiglu(g["gate"], g["up"])), "act"
    assert same(g["down"], lin(g["act"], 8, exps["e_mlp_act"], "down")), "down"
    assert same(x_out, B.residual_add(g["x1"], g["down"])), "x_out"
    return bool(np.array_equal(np.where(tri, got_c, 0), np.where(tri, want_c, 0)))


CASES = [
    # S, d, H, F, keep, qmax, bits_attn_out
    (200, 512, 4, 1408, 150, 15, 4),     # D = 128, ragged S (padded to 256), pruning, 4-bit after attention
    (130, 256, 4, 384, 130, 7, 8),       # D = 64, nothing pruned, literal Eq.3 range, 8-bit after attention
    (16, 128, 2, 256, 9, 15, 4),         # few tokens: the weight-streaming kernels serve every projection
    (1, 128, 1, 128, 1, 15, 8),          # a single token
    (300, 1024, 8, 2816, 77, 15, 4),     # heavy pruning
]


@pytest.mark.parametrize("S,d,H,F,keep,qmax,bits_o", CASES)
def test_block_stage_by_stage(agq, oracle, blk_oracle, S, d, H, F, keep, qmax, bits_o):
    B = blk_oracle
    rng = np.random.default_rng(S)
    pos = np.sort(rng.choice(3 * S + 5, size=S, replace=False)).astype(np.int32)   # as after earlier pruning
    x, pos, cos, sin, w = make_inputs(S, d, H, F, seed=100 + S, pos=pos)
    ref = B.block_forward(x, pos, cos, sin, w, H, qmax, EPS, keep, bits_attn_out=bits_o)   # calibrates
    exps = ref["exps"]
    wd = upload_weights(agq, w)
    blk = agq.make_block(d, H, F, wd, qmax=qmax, bits_attn_out=bits_o, rms_eps=EPS, exps=exps)
    x_out, pos_out, ws, L = agq.block_forward(blk, dev(x), dev(pos), dev(cos), dev(sin), n_keep=keep)
    g = gpu_tensors(agq, blk, L, ws, S, keep)
    codes_equal = check_stages(agq, oracle, B, w, H, qmax, bits_o, x, pos, cos, sin, keep, exps, g, host(x_out),
                               host(pos_out))
    if codes_equal:      # then nothing separates the two chains
        assert same(host(x_out), ref["x_out"]) and np.array_equal(g["idx"], ref["idx"])
    # the same call again into the same workspace gives the same bits (no state, no uninitialised reads)
    x_out2, _, _, _ = agq.block_forward(blk, dev(x), dev(pos), dev(cos), dev(sin), n_keep=keep, workspace=ws)
    assert same(host(x_out2), host(x_out))


@pytest.mark.parametrize("S,keep,sites,kmax", [(200, 150, ("attn_in", "mlp_in"), 4), (12, 7, ("attn_in", "mlp_in"), 4),
                                               (160, 160, ("attn_in", "attn_out", "mlp_in", "mlp_act"), 1),
                                               (40, 30, ("mlp_act",), 2)])
def test_block_with_trip_sites(agq, oracle, blk_oracle, S, keep, sites, kmax):
    """TRIP (Eq.5-8) at chosen activations of the block: their projections are TRIP blobs, the exponent is Eq.6's
    base step; q, k, v (and gate, up) share the gathered pre-pass.  Checked stage by stage like the plain block."""
    d, H, F = 512, 4, 1408
    x, pos, cos, sin, w = make_inputs(S, d, H, F, seed=300 + S)
    full = blk_oracle.block_forward(x, pos, cos, sin, w, H, 15, EPS, keep, trip_kmax=kmax)     # factors at every site
    alphas = {s_: full["alphas"][s_] for s_ in sites}
    # exponents: base step at the chosen sites, the plain calibration elsewhere
    ref = blk_oracle.block_forward(x, pos, cos, sin, w, H, 15, EPS, keep)
    exps = dict(ref["exps"])
    for s_ in sites:
        exps["e_" + s_] = full["exps"]["e_" + s_]
    ref = blk_oracle.block_forward(x, pos, cos, sin, w, H, 15, EPS, keep, exps=exps, alphas=alphas)
    wd, trip = upload_weights(agq, w, alphas)
    assert set(trip) == set(sites)          # a site whose factors are all zero is a TRIP blob without extra chunks
    blk = agq.make_block(d, H, F, wd, rms_eps=EPS, exps=exps, trip=trip)
    x_out, pos_out, ws, L = agq.block_forward(blk, dev(x), dev(pos), dev(cos), dev(sin), n_keep=keep)
    g = gpu_tensors(agq, blk, L, ws, S, keep)
    same_codes = check_stages(agq, oracle, blk_oracle, w, H, 15, 4, x, pos, cos, sin, keep, exps, g, host(x_out),
                              host(pos_out), alphas=alphas)
    if same_codes:
        assert same(host(x_out), ref["x_out"])
    # the calibration pass wants plain blobs
    with pytest.raises(agq.AgqError):
        agq.block_forward(blk, dev(x), dev(pos), dev(cos), dev(sin), n_keep=keep, calibrate=True)


def test_block_calibrate_finds_the_oracle_exponents(agq, oracle, blk_oracle):
    S, d, H, F, keep = 160, 512, 4, 1408, 120
    x, pos, cos, sin, w = make_inputs(S, d, H, F, seed=7)
    ref = blk_oracle.block_forward(x, pos, cos, sin, w, H, 15, EPS, keep)
    wd = upload_weights(agq, w)
    blk = agq.make_block(d, H, F, wd, rms_eps=EPS)
    x_cal, _, ws, L = agq.block_forward(blk, dev(x), dev(pos), dev(cos), dev(sin), n_keep=keep, calibrate=True)
    got = agq.block_exps(blk)
    g = gpu_tensors(agq, blk, L, ws, S, keep)
    # each exponent is the oracle's calibration of the tensor the GPU's quantizer reads
    q_rot = host(agq.block_tensor(blk, L, ws, "q_rot", S, keep))
    k_rot = host(agq.block_tensor(blk, L, ws, "k_rot", S, keep))
    assert same(q_rot, blk_oracle.rope(g["q"], pos, cos, sin, H)) and same(k_rot, blk_oracle.rope(g["k"], pos, cos, sin, H))
    want = dict(e_attn_in=oracle.calibrate_act_exp(g["h1"], 8), e_q=oracle.calibrate_act_exp(q_rot, 8),
                e_k=oracle.calibrate_act_exp(k_rot, 8), e_v=oracle.calibrate_act_exp(g["v"], 8),
                e_attn_out=oracle.calibrate_act_exp(g["o_kept"][:keep], 4),
                e_mlp_in=oracle.calibrate_act_exp(g["h2"], 8), e_mlp_act=oracle.calibrate_act_exp(g["act"], 8))
    assert got == want
    # the calibration pass itself is a forward pass with those exponents
    x_fwd, _, _, _ = agq.block_forward(blk, dev(x), dev(pos), dev(cos), dev(sin), n_keep=keep)
    assert same(host(x_fwd), host(x_cal))
    assert got == ref["exps"] or not same(host(x_cal), ref["x_out"])   # equal chains imply equal exponents


def test_cascade_of_blocks(agq, oracle, blk_oracle):
    """Eq.9: three blocks, the last two pruning with the progressive ratio; every block checked stage by stage on
    the tokens and positions the previous one handed over."""
    S, d, H, F = 256, 256, 2, 640
    keeps = [S] + agq.cascade_keep(S, 0.5, 2)
    assert keeps == [S] + blk_oracle.cascade_keep(S, 0.5, 2) and keeps[-1] in (128, 129)
    x, pos, cos, sin, _ = make_inputs(S, d, H, F, seed=11)
    xg, pg = dev(x), dev(pos)
    for layer, keep in enumerate(keeps):
        w = synth.make_block_weights(d, H, F, 50 + layer)
        x_in, pos_in = host(xg), host(pg)
        ref = blk_oracle.block_forward(x_in, pos_in, cos, sin, w, H, 15, EPS, keep)
        blk = agq.make_block(d, H, F, upload_weights(agq, w), rms_eps=EPS, exps=ref["exps"])
        xg, pg, ws, L = agq.block_forward(blk, xg, pg, dev(cos), dev(sin), n_keep=keep)
        g = gpu_tensors(agq, blk, L, ws, x_in.shape[0], keep)
        check_stages(agq, oracle, blk_oracle, w, H, 15, 4, x_in, pos_in, cos, sin, keep, ref["exps"], g, host(xg),
                     host(pg))
    assert xg.shape == (keeps[-1], d) and host(pg)[0] == 0


def test_stack_with_cascade_equals_block_by_block(agq, oracle, blk_oracle):
    """agq_stack_forward: five blocks, Eq.9's schedule (two pruning stages, beta = 0.6) applied in blocks 1 and 3; the
    call equals the same blocks run one by one (each of which is checked stage by stage above), bit for bit."""
    S, d, H, F, n = 300, 256, 2, 640, 5
    stages = agq.cascade_keep(S, 0.6, 2)
    keep = [S, stages[0], stages[0], stages[1], stages[1]]
    x, pos, cos, sin, _ = make_inputs(S, d, H, F, seed=41)
    xd, pd, cd, sd = dev(x), dev(pos), dev(cos), dev(sin)
    blocks, xg, pg, s_in = [], xd, pd, S
    for layer in range(n):                      # calibrate every block on the tokens it will receive
        w = synth.make_block_weights(d, H, F, 60 + layer)
        blk = agq.make_block(d, H, F, upload_weights(agq, w), rms_eps=EPS)
        agq.block_forward(blk, xg, pg, cd, sd, n_keep=keep[layer], calibrate=True)
        xg, pg, _, _ = agq.block_forward(blk, xg, pg, cd, sd, n_keep=keep[layer])
        blocks.append(blk)
    x_seq, p_seq = host(xg).copy(), host(pg).copy()
    x_st, p_st, ws = agq.stack_forward(blocks, keep, xd, pd, cd, sd)
    assert x_st.shape == (keep[-1], d) and same(host(x_st), x_seq) and np.array_equal(host(p_st), p_seq)
    assert host(p_st)[0] == 0 and np.all(np.diff(host(p_st)) > 0)
    # captured into a graph and replayed into a dirty workspace
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        agq.stack_forward(blocks, keep, xd, pd, cd, sd, workspace=ws, out=(x_st, p_st))
    for rep in range(2):
        x_st.fill_(3.0)
        ws.fill_(0xA5)
        torch.cuda.synchronize()
        graph.replay()
        assert same(host(x_st), x_seq) and np.array_equal(host(p_st), p_seq)
    # argument errors: a count that grows, a block of another width
    with pytest.raises(agq.AgqError):
        agq.stack_forward(blocks, [S, 200, 210, 100, 100], xd, pd, cd, sd)
    other = agq.make_block(512, 4, 640, blocks[0]._keepalive, rms_eps=EPS)
    with pytest.raises(agq.AgqError):
        agq.stack_forward(blocks[:1] + [other], keep[:2], xd, pd, cd, sd)


def test_block_graph_replay(agq, oracle, blk_oracle):
    """agq_block_forward enqueues kernels only (no memset nodes, no allocation): captured into a HIP graph after an
    eager call, every replay reproduces the eager result bit for bit, with eager work in between."""
    S, d, H, F, keep = 200, 256, 2, 640, 120
    x, pos, cos, sin, w = make_inputs(S, d, H, F, seed=31)
    blk = agq.make_block(d, H, F, upload_weights(agq, w), rms_eps=EPS)
    xd, pd, cd, sd = dev(x), dev(pos), dev(cos), dev(sin)
    x_out, pos_out, ws, L = agq.block_forward(blk, xd, pd, cd, sd, n_keep=keep, calibrate=True)
    agq.block_forward(blk, xd, pd, cd, sd, n_keep=keep, workspace=ws, out=(x_out, pos_out))
    eager_x, eager_p = host(x_out).copy(), host(pos_out).copy()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        agq.block_forward(blk, xd, pd, cd, sd, n_keep=keep, workspace=ws, out=(x_out, pos_out))
    for rep in range(3):
        x_out.fill_(rep + 1)
        pos_out.fill_(-1)
        ws.fill_(0x5A if rep else 0)          # the call may not depend on what the workspace held
        torch.cuda.synchronize()
        graph.replay()
        assert same(host(x_out), eager_x) and np.array_equal(host(pos_out), eager_p), rep


SPECIAL = np.array([0.0, -0.0, 6e-8, -6e-8, 6.1e-5, -6.1e-5, 65504.0, -65504.0, 1024.0, 0.5, 2048.0, 1.0, 0.333, 12.0,
                    -12.0, 20.0, -20.0, 1e-3, -1e-3, 3.0, -7.0, 0.25, 1e4, -1e4], dtype=np.float16)


def test_elementwise_operators_on_special_values(agq, blk_oracle):
    """SwiGLU and the residual addition on every pair of values that stress the single rounding (ties such as
    1024 + 0.5 and 2048 + 1, subnormal sums, overflow to Inf, both tails of the exponential), and on random data."""
    a, b = np.meshgrid(SPECIAL, SPECIAL)
    a, b = np.ascontiguousarray(a.ravel()), np.ascontiguousarray(b.ravel())      # 576 = 72 * 8 values
    rng = np.random.default_rng(5)
    ra = (rng.standard_normal(8 * 4099) * 4).astype(np.float16)
    rb = (rng.standard_normal(8 * 4099) * np.exp(rng.uniform(-8, 6, 8 * 4099))).astype(np.float16)
    for u, v in ((a, b), (ra, rb)):
        with np.errstate(over="ignore", invalid="ignore"):
            assert same(host(agq.residual_add(dev(u), dev(v))), blk_oracle.residual_add(u, v))
            assert same(host(agq.swiglu(dev(u), dev(v))), blk_oracle.swiglu(u, v))
    L = agq.lib()
    t = dev(ra)
    assert L.agq_swiglu(t.data_ptr(), t.data_ptr(), t.data_ptr(), 12, None) == agq.AGQ_EINVAL
    assert L.agq_residual_add(t.data_ptr(), None, t.data_ptr(), 16, None) == agq.AGQ_EINVAL
    assert L.agq_residual_add(None, None, None, 0, None) == agq.AGQ_OK


@pytest.mark.parametrize("rows,d", [(5, 8), (3, 128), (7, 5120), (2, 8200), (2, 16384)])
def test_rmsnorm_operator(agq, blk_oracle, rows, d):
    rng = np.random.default_rng(d)
    x = (rng.standard_normal((rows, d)) * np.exp(rng.uniform(-6, 6, (rows, 1)))).astype(np.float16)
    x[0, : min(d, SPECIAL.size)] = SPECIAL[: min(d, SPECIAL.size)]
    g = (1 + 0.3 * rng.standard_normal(d)).astype(np.float16)
    for eps in (1e-5, 1e-6, 0.0):
        assert same(host(agq.rmsnorm(dev(x), dev(g), eps)), blk_oracle.rmsnorm(x, g, eps)), eps
    # fused with the residual addition and the row gather
    res = (rng.standard_normal((rows + 9, d)) * 3).astype(np.float16)
    idx = np.sort(rng.choice(rows + 9, size=rows, replace=False)).astype(np.int32)
    xs = (x.astype(np.float32) * np.float32(2.0 ** -6)).astype(np.float16) if d > 8 else x
    xs = np.where(np.isfinite(xs), xs, np.float16(1.0)).astype(np.float16)
    xs[np.abs(xs.astype(np.float32)) > 1000] = np.float16(7.0)
    t, y = agq.rmsnorm(dev(xs), dev(g), 1e-5, res=dev(res), idx=dev(idx))
    want_t = blk_oracle.residual_add(res[idx], xs)
    assert same(host(t), want_t) and same(host(y), blk_oracle.rmsnorm(want_t, g, 1e-5))
    t, y = agq.rmsnorm(dev(xs), dev(g), 1e-5, res=dev(res[:rows].copy()))
    want_t = blk_oracle.residual_add(res[:rows], xs)
    assert same(host(t), want_t) and same(host(y), blk_oracle.rmsnorm(want_t, g, 1e-5))


@pytest.mark.parametrize("S,H,D,S_pad", [(5, 3, 16, 5), (130, 4, 64, 256), (77, 2, 128, 128), (128, 1, 128, 128)])
def test_rope_quantize_operator(agq, blk_oracle, S, H, D, S_pad):
    rng = np.random.default_rng(S)
    P = 300
    cos, sin = synth.rope_tables(P, D)
    q, k, v = [(rng.standard_normal((S, H * D)) * sc).astype(np.float16) for sc in (1.0, 3.0, 0.5)]
    q[0, : SPECIAL.size] = SPECIAL
    pos = rng.integers(0, P, size=S).astype(np.int32)
    pos[-1] = P + 50                       # outside the table: clamped to its last row
    pos[0] = -3                            # and to its first
    pc = np.clip(pos, 0, P - 1)
    for e_q, e_k, e_v in ((-5, -3, -6), (0, -9, 2)):
        got = agq.rope_quantize(dev(q), dev(k), dev(v), H, dev(pos), dev(cos), dev(sin), e_q, e_k, e_v, S_pad=S_pad)
        want = [blk_oracle.heads_int8(blk_oracle.rope(q, pc, cos, sin, H), H, e_q, S_pad),
                blk_oracle.heads_int8(blk_oracle.rope(k, pc, cos, sin, H), H, e_k, S_pad),
                blk_oracle.heads_int8(v, H, e_v, S_pad)]
        for gt, wt, n in zip(got, want, "qkv"):
            assert same(host(gt), wt), (n, e_q, e_k, e_v)
    # no tokens at all: the padding rows are still cleared
    junk = [torch.full((H, 128, D), 77, dtype=torch.int8, device="cuda") for _ in range(3)]
    t = dev(q)
    assert agq.lib().agq_rope_quantize(t.data_ptr(), t.data_ptr(), t.data_ptr(), 0, H, D, dev(pos).data_ptr(),
                                       dev(cos).data_ptr(), dev(sin).data_ptr(), P, 0, 0, 0, 128, junk[0].data_ptr(),
                                       junk[1].data_ptr(), junk[2].data_ptr(), None) == agq.AGQ_OK
    assert all(not host(j).any() for j in junk)


def check_block_sampled(agq, oracle, B, S, d, H, F, keep, seed):
    """A calibration pass and a forward pass at a size the oracle cannot do whole: rows sampled for the oracle at
    every stage, the pruning indices, the element-wise operators and the attention relations in full."""
    qmax = 15
    x, pos, cos, sin, w = make_inputs(S, d, H, F, seed=seed)
    wd = upload_weights(agq, w)
    blk = agq.make_block(d, H, F, wd, qmax=qmax, bits_attn_out=4, rms_eps=EPS)
    x_out, pos_out, ws, L = agq.block_forward(blk, dev(x), dev(pos), dev(cos), dev(sin), n_keep=keep, calibrate=True)
    exps = agq.block_exps(blk)
    x_fwd, _, _, _ = agq.block_forward(blk, dev(x), dev(pos), dev(cos), dev(sin), n_keep=keep, workspace=ws)
    assert same(host(x_fwd), host(x_out))
    g = gpu_tensors(agq, blk, L, ws, S, keep)
    x_out, pos_out = host(x_out), host(pos_out)
    rows = np.array(sorted({0, 1, S // 3 + 94, (5 * S) // 8 + 20, S - 1}))
    lin = lambda t, bits, e, n: oracle.linear_w4(t, bits, e, 0, w["w_" + n], w["s_" + n])[1]
    assert same(g["h1"][rows], B.rmsnorm(x[rows], w["g_attn"], EPS))
    assert exps["e_attn_in"] == oracle.calibrate_act_exp(g["h1"], 8)
    for n in ("q", "k", "v"):
        assert same(g[n][rows], lin(g["h1"][rows], 8, exps["e_attn_in"], n)), n
    for n in ("q", "k"):
        rot = B.rope(g[n][rows], pos[rows], cos, sin, H)
        assert same(g[n + "_q"][:, rows], B.heads_int8(rot, H, exps["e_" + n])), n
    assert same(g["v_q"][:, rows], B.heads_int8(g["v"][rows], H, exps["e_v"]))
    assert not g["q_q"][:, S:].any() and not g["k_q"][:, S:].any() and not g["v_q"][:, S:].any()
    o2, _, score2 = agq.qk_log2_softmax(dev(g["q_q"]), dev(g["k_q"]), dev(g["v_q"]), exps["e_q"], exps["e_k"],
                                        exps["e_v"], qmax=qmax, causal=True, want_codes=False, want_score=True)
    assert same(g["o"], host(o2)) and same(g["score"], host(score2))
    idx = oracle.prune_select(g["score"][:S], keep) if keep < S else np.arange(S, dtype=np.int32)
    assert np.array_equal(g["idx"], idx) and idx[0] == 0 and np.array_equal(pos_out, pos[idx])
    assert same(g["o_kept"][:keep], g["o"][idx])
    kr = np.array(sorted({0, 1, keep // 2 - 12, keep - 1}))
    assert exps["e_attn_out"] == oracle.calibrate_act_exp(g["o_kept"][:keep], 4)
    assert same(g["attn_out"][kr], lin(g["o_kept"][kr], 4, exps["e_attn_out"], "o"))
    assert same(g["x1"], B.residual_add(x[idx], g["attn_out"]))
    assert same(g["h2"][kr], B.rmsnorm(g["x1"][kr], w["g_mlp"], EPS))
    assert same(g["gate"][kr], lin(g["h2"][kr], 8, exps["e_mlp_in"], "gate"))
    assert same(g["up"][kr], lin(g["h2"][kr], 8, exps["e_mlp_in"], "up"))
    assert same(g["act"], B.swiglu(g["gate"], g["up"]))
    assert exps["e_mlp_act"] == oracle.calibrate_act_exp(g["act"], 8)
    assert same(g["down"][kr], lin(g["act"][kr], 8, exps["e_mlp_act"], "down"))
    assert same(x_out, B.residual_add(g["x1"], g["down"]))


def test_block_llama13b_full_size_sampled(agq, oracle, blk_oracle):
    """The benchmark's block (d = 5120, H = 40, F = 13824, S = 2048, half of the tokens pruned)."""
    check_block_sampled(agq, oracle, blk_oracle, 2048, 5120, 40, 13824, 1024, seed=13)


def test_block_with_few_tokens_on_wide_layers(agq, oracle, blk_oracle):
    """Few tokens on wide layers: the projections after the pruning have few output tiles and a long K, so the
    tiled kernel splits K over workgroups (partial tiles in the block's GEMM scratch)."""
    check_block_sampled(agq, oracle, blk_oracle, 300, 2048, 16, 4096, 200, seed=16)
    check_block_sampled(agq, oracle, blk_oracle, 520, 1024, 8, 8192, 130, seed=17)


def test_block_longest_sequences(agq, oracle, blk_oracle):
    """The largest token counts a call accepts: 8192 with pruning (the selection's limit), and beyond it without
    (here 8200, padded to 8320 for the attention call), on a narrow block."""
    check_block_sampled(agq, oracle, blk_oracle, 8192, 128, 2, 128, 5000, seed=14)
    check_block_sampled(agq, oracle, blk_oracle, 8200, 128, 2, 128, 8200, seed=15)
