"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on
the same seeded inputs.  Integer results (codes, packed bytes, accumulators,
indices) must be bit-exact; fp16 outputs must agree within 1e-3 relative (plus
one fp16 subnormal step absolute), the tolerance of the benchmark spec - the
kernel's float(acc) * g is rounded to fp32 and then to fp16, the oracle rounds
the exact product once, so they differ by at most one fp16 ulp, rarely."""
from __future__ import annotations

import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from paper_2312_05693_amd import synth  # noqa: E402

REL_TOL = 1e-3
ABS_TOL = 2.0 ** -24


@pytest.fixture(scope="module")
def agq():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2312_05693_amd import binding
    binding.lib()          # must load: there is no fallback
    return binding


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def assert_f16_close(got, want, what=""):
    got = np.asarray(got, dtype=np.float16)
    want = np.asarray(want, dtype=np.float16)
    assert got.shape == want.shape, what
    g64, w64 = got.astype(np.float64), want.astype(np.float64)
    fin = np.isfinite(w64)
    assert np.array_equal(np.isfinite(g64), fin), what
    assert np.array_equal(g64[~fin], w64[~fin]), what
    err = np.abs(g64[fin] - w64[fin])
    bound = REL_TOL * np.abs(w64[fin]) + ABS_TOL
    assert np.all(err <= bound), "%s: max excess %g" % (what, float((err - bound).max()))
    # and the disagreements are single-ulp, rare double-rounding cases
    diff = got.view(np.int16).astype(np.int32)[fin] - want.view(np.int16).astype(np.int32)[fin]
    assert np.abs(diff).max(initial=0) <= 1, what
    assert (diff != 0).mean() <= 2e-3 if diff.size > 2000 else True, what


def make_case(M, K, N, seed, n_out=4):
    x = synth.make_activation(M, K, n_out, seed)
    wq, sw = synth.make_weight_q4(N, K, seed)
    return x, wq, sw


# ------------------------------------------------------------------ pack / unpack

def test_pack_roundtrip(agq, oracle):
    rng = np.random.default_rng(0)
    # every nibble value at every position of one 16 x 128 chunk, and ragged N
    for N, K in ((16, 128), (40, 256), (256, 384), (300, 128)):
        wq = rng.integers(-8, 8, size=(N, K)).astype(np.int8)
        if N == 16:
            wq = ((np.arange(N * K).reshape(N, K) * 7 + np.arange(N)[:, None]) % 16 - 8).astype(np.int8)
        packed = agq.pack_w4(dev(wq))
        assert packed.numel() == agq.pack_w4_bytes(N, K)
        assert np.array_equal(host(agq.unpack_w4(packed, N, K)), wq)
        # the nibble part of the blob holds exactly the multiset of nibbles of W (plus zero padding) ...
        npad = (N + 255) // 256 * 256
        nib = host(packed)[: npad * K // 2]
        counts = np.bincount(np.concatenate([nib & 0xF, nib >> 4]), minlength=16)
        want = np.bincount((wq.astype(np.int64) & 0xF).ravel(), minlength=16)
        want[0] += nib.size * 2 - wq.size
        assert np.array_equal(counts, want)
        # ... and its tail the sum of every output channel's weights, padded channels 0
        wsum = host(packed)[npad * K // 2:].view(np.int32)
        assert wsum.size == npad
        assert np.array_equal(wsum[:N], wq.astype(np.int64).sum(axis=1)) and not wsum[N:].any()
    # out-of-range values are saturated and counted
    wq = rng.integers(-8, 8, size=(16, 128)).astype(np.int8)
    wq[3, 5], wq[9, 100], wq[0, 0] = 9, -100, 127
    bad = torch.zeros(1, dtype=torch.int32, device="cuda")
    packed = agq.pack_w4(dev(wq), bad_count=bad)
    assert int(host(bad)[0]) == 3
    assert np.array_equal(host(agq.unpack_w4(packed, 16, 128)), np.clip(wq, -8, 7))


# ------------------------------------------------------------------ Eq.2

def test_quantize_all_fp16_patterns(agq, oracle):
    allh = np.arange(0x10000, dtype=np.uint16).view(np.float16)
    x = allh[np.isfinite(allh.astype(np.float32)) | np.isinf(allh.astype(np.float32))]
    x = x[~np.isnan(x.astype(np.float32))]
    x = np.concatenate([x, np.zeros((-x.size) % 64, np.float16)]).reshape(-1, 64)
    xd = dev(x)
    for bits in (8, 4):
        for e in (-8, -3, -1, 0, 1, 2, 7):
            for zp in (0, 1 << (bits - 1), 3):
                want = oracle.quantize_act(x, bits, e, zp)
                got = host(agq.quantize_act(xd, bits, e, zp))
                if bits == 8:
                    got = got.astype(np.int32) if zp == 0 else got.view(np.uint8).astype(np.int32)
                    assert np.array_equal(got, want), (bits, e, zp)
                else:
                    assert np.array_equal(got.view(np.uint8), oracle.pack_nibbles(want)), (bits, e, zp)


def test_quantize_strided_and_edges(agq, oracle):
    x = synth.make_activation(37, 200, 3, 4)            # K % 8 == 0, ragged rows
    big = torch.zeros((37, 256), dtype=torch.float16, device="cuda")
    big[:, :200] = dev(x)
    view = big[:, :200]
    got = host(agq.quantize_act(view, 8, -2, 0))
    assert np.array_equal(got.astype(np.int32), oracle.quantize_act(x, 8, -2, 0))
    empty = torch.zeros((0, 64), dtype=torch.float16, device="cuda")
    assert agq.quantize_act(empty, 8, 0).shape == (0, 64)


def test_calibrate(agq, oracle):
    cases = [synth.make_activation(128, 768, 4, 0), synth.make_activation(1, 4096, 4, 1),
             synth.make_activation(300, 1024, 11, 2), np.zeros((4, 64), np.float16),
             (synth.make_activation(8, 64, 0, 3).astype(np.float32) * 1e-4).astype(np.float16),
             np.full((2, 8), 127.0, np.float16), np.full((2, 8), 127.5, np.float16),
             np.array([[np.inf] + [0] * 7], np.float16), np.full((1, 8), 6e-8, np.float16)]
    for x in cases:
        for bits in (8, 4):
            e = int(host(agq.calibrate_act_exp(dev(x), bits))[0])
            assert e == oracle.calibrate_act_exp(x, bits), (x.shape, bits)


# ------------------------------------------------------------------ the linear layer

def run_linear(agq, oracle, x, wq, sw, bits, x_kind="f16", e=None, check_y=True, zp=0):
    M, K = x.shape
    N = wq.shape[0]
    if e is None:
        e = oracle.calibrate_act_exp(x, bits) if M else 0
    acc_want, y_want = oracle.linear_w4(x, bits, e, zp, wq, sw)
    packed = agq.pack_w4(dev(wq))
    acc = torch.full((M, N), -12345, dtype=torch.int32, device="cuda")
    fn = agq.gemm_w4a8 if bits == 8 else agq.gemm_w4a4
    if x_kind == "f16":
        xin, kind = dev(x), agq.AGQ_X_F16
    elif x_kind == "dot":
        xin, kind = dev(x), agq.AGQ_X_F16_DOT
    else:
        xin, kind = agq.quantize_act(dev(x), bits, e, zp), agq.AGQ_X_Q
    y = fn(xin, e, packed, dev(sw), N, K, x_kind=kind, acc_out=acc, zp=zp)
    assert np.array_equal(host(acc).astype(np.int64), acc_want), "accumulators differ"
    if check_y:
        assert_f16_close(host(y), y_want, "y")
    return e


@pytest.mark.parametrize("M", [1, 2, 3, 4, 5, 8, 13, 16])
@pytest.mark.parametrize("K,N", [(128, 16), (256, 40), (768, 768), (1408, 272), (4096, 64)])
def test_decode_small(agq, oracle, M, K, N):
    x, wq, sw = make_case(M, K, N, seed=100 + M + K + N)
    run_linear(agq, oracle, x, wq, sw, 8)


@pytest.mark.parametrize("bits,x_kind", [(8, "q"), (4, "f16"), (4, "q")])
@pytest.mark.parametrize("M,K,N", [(1, 256, 48), (7, 1024, 100), (16, 768, 256)])
def test_decode_variants(agq, oracle, bits, x_kind, M, K, N):
    x, wq, sw = make_case(M, K, N, seed=7 * M + K + N + bits)
    run_linear(agq, oracle, x, wq, sw, bits, x_kind)


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("K,N", [(128, 16), (256, 40), (1408, 272), (4096, 4096), (4096, 11008), (11008, 4096), (16384, 48)])
def test_decode_vector_alu_form(agq, oracle, K, N, bits):
    """One token row on the vector ALU (AGQ_X_F16_DOT: Eq.2 in registers, v_dot4_i32_i8 / v_dot8_i32_i4, no matrix
    core): the accumulators against the oracle bit for bit, and the fp16 output identical to the matrix-core form's."""
    x, wq, sw = make_case(1, K, N, seed=900 + K + N + bits)
    e = run_linear(agq, oracle, x, wq, sw, bits, "dot")
    packed, xd, swd = agq.pack_w4(dev(wq)), dev(x), dev(sw)
    fn = agq.gemm_w4a8 if bits == 8 else agq.gemm_w4a4
    y_dot = fn(xd, e, packed, swd, N, K, x_kind=agq.AGQ_X_F16_DOT)
    y_mfma = fn(xd, e, packed, swd, N, K)
    assert np.array_equal(host(y_dot).view(np.uint16), host(y_mfma).view(np.uint16))
    # clipping codes (a too small exponent) saturate the same way
    run_linear(agq, oracle, x, wq, sw, bits, "dot", e=e - 3)
    # several projections of the row in one launch
    wq2, sw2 = synth.make_weight_q4(N + 16, K, seed=77)
    mfn = agq.gemm_w4a8_multi if bits == 8 else agq.gemm_w4a4_multi
    accs = [torch.zeros((1, n), dtype=torch.int32, device="cuda") for n in (N, N + 16)]
    mfn(xd, e, [(packed, swd, N, None, accs[0]), (agq.pack_w4(dev(wq2)), dev(sw2), N + 16, None, accs[1])], K,
        x_kind=agq.AGQ_X_F16_DOT)
    assert np.array_equal(host(accs[0]).astype(np.int64), oracle.linear_w4(x, bits, e, 0, wq, sw)[0])
    assert np.array_equal(host(accs[1]).astype(np.int64), oracle.linear_w4(x, bits, e, 0, wq2, sw2)[0])
    # only for one row on the signed grid
    L = agq.lib()
    two = torch.zeros((2, K), dtype=torch.float16, device="cuda")
    y2 = torch.zeros((2, N), dtype=torch.float16, device="cuda")
    assert L.agq_gemm_w4a8(two.data_ptr(), agq.AGQ_X_F16_DOT, 2, K, K, 0, 0, packed.data_ptr(), swd.data_ptr(), N,
                           y2.data_ptr(), N, None, None, 0, None) == agq.AGQ_EINVAL
    assert L.agq_gemm_w4a8(xd.data_ptr(), agq.AGQ_X_F16_DOT, 1, K, K, 0, 128, packed.data_ptr(), swd.data_ptr(), N,
                           y2.data_ptr(), N, None, None, 0, None) == agq.AGQ_EINVAL


@pytest.mark.parametrize("M", [17, 64, 128, 129, 200, 257, 300, 333, 400])
@pytest.mark.parametrize("K,N", [(128, 16), (384, 272), (768, 768), (1024, 500)])
def test_tiled_small(agq, oracle, M, K, N):
    # up to 256 rows of fp16 input these small layers run as row groups of the weight-streaming kernel,
    # beyond that through the pre-pass and the tiled kernel (ragged last tiles in both directions)
    x, wq, sw = make_case(M, K, N, seed=200 + M + K + N)
    run_linear(agq, oracle, x, wq, sw, 8)


@pytest.mark.parametrize("M,K,N,bits,zp", [(17, 4096, 4096, 8, 0), (64, 4096, 4096, 8, 0), (80, 4096, 4096, 8, 0),
                                             (32, 4096, 11008, 8, 0), (48, 4096, 11008, 8, 0), (64, 11008, 4096, 8, 0),
                                             (250, 2048, 512, 4, 0), (256, 768, 768, 8, 131), (100, 1408, 272, 4, 9),
                                             (31, 13824, 48, 8, 0)])
def test_row_groups_and_the_switch_to_tiles(agq, oracle, M, K, N, bits, zp):
    """17..256 rows: sixteen rows per workgroup of the weight-streaming kernel while the weights re-read per row
    group stay cheap, else the tiled path; shapes on both sides of the switch, both grids, ragged last groups.
    The accumulators are compared on sampled rows where the full product would take the oracle too long."""
    x, wq, sw = make_case(M, K, N, seed=400 + M + N, n_out=6)
    e = oracle.calibrate_act_exp(x, bits) + (1 if zp else 0)
    acc = torch.full((M, N), -3, dtype=torch.int32, device="cuda")
    fn = agq.gemm_w4a8 if bits == 8 else agq.gemm_w4a4
    y = fn(dev(x), e, agq.pack_w4(dev(wq)), dev(sw), N, K, acc_out=acc, zp=zp)
    rows = sorted({0, 1, 15, 16, min(17, M - 1), M // 2, M - 2, M - 1})
    acc_w, y_w = oracle.linear_w4(x[rows], bits, e, zp, wq, sw)
    assert np.array_equal(host(acc)[rows].astype(np.int64), acc_w)
    assert_f16_close(host(y)[rows], y_w, "y")
    # every row was written, and row groups do not leak into each other: a second activation that differs in one
    # row changes that row only
    x2 = x.copy()
    x2[M // 2] = x[0]
    acc2 = torch.full((M, N), -3, dtype=torch.int32, device="cuda")
    fn(dev(x2), e, agq.pack_w4(dev(wq)), dev(sw), N, K, acc_out=acc2, zp=zp)
    a1, a2 = host(acc), host(acc2)
    assert np.array_equal(np.delete(a1, M // 2, axis=0), np.delete(a2, M // 2, axis=0))
    assert np.array_equal(a2[M // 2], a1[0])


@pytest.mark.parametrize("M,K,N,bits,zp,x_kind", [(300, 2048, 384, 8, 0, "f16"), (290, 2048, 500, 4, 0, "f16"),
                                                    (700, 2816, 272, 8, 131, "f16"), (260, 2560, 130, 8, 0, "q"),
                                                    (128, 4096, 4096, 8, 0, "f16"), (257, 4096, 4096, 4, 9, "f16"),
                                                    (400, 11008, 4096, 8, 0, "f16"), (300, 13824, 640, 8, 0, "q")])
def test_tiled_split_k(agq, oracle, M, K, N, bits, zp, x_kind):
    """Few 128 x 128 tiles and a long K: the K steps of a tile are shared out over several workgroups, whose int32
    partial tiles a second kernel adds up.  Against the oracle (sampled rows at the large sizes), against the
    same call with a workspace that only has room for the activation (no split), and call after call into the same
    workspace."""
    x, wq, sw = make_case(M, K, N, seed=900 + M + N, n_out=6)
    e = oracle.calibrate_act_exp(x, bits) + (1 if zp else 0)
    full, small = agq.gemm_workspace_bytes(M, N, K), agq.gemm_workspace_bytes(M, 0, K)
    assert full > small == -(-M // 128) * 128 * K       # these shapes are split
    fn = agq.gemm_w4a8 if bits == 8 else agq.gemm_w4a4
    if x_kind == "f16":
        xin, kind = dev(x), agq.AGQ_X_F16
    elif x_kind == "dot":
        xin, kind = dev(x), agq.AGQ_X_F16_DOT
    else:
        xin, kind = agq.quantize_act(dev(x), bits, e, zp), agq.AGQ_X_Q
    packed, swd = agq.pack_w4(dev(wq)), dev(sw)
    ws = torch.empty(full, dtype=torch.uint8, device="cuda")
    ws.fill_(0xA5)                                       # nothing relies on what the workspace held
    outs = []
    for rep in range(3):
        acc = torch.full((M, N), -3, dtype=torch.int32, device="cuda")
        y = fn(xin, e, packed, swd, N, K, x_kind=kind, acc_out=acc, zp=zp, workspace=ws)
        outs.append((host(acc), host(y)))
    acc1 = torch.full((M, N), -3, dtype=torch.int32, device="cuda")
    y1 = fn(xin, e, packed, swd, N, K, x_kind=kind, acc_out=acc1, zp=zp, workspace=ws[:small])
    for a, yy in outs:
        assert np.array_equal(a, host(acc1)) and np.array_equal(yy.view(np.int16), host(y1).view(np.int16))
    rows = list(range(M)) if M * K * N <= 3e8 else sorted({0, 1, 31, 32, 127, M // 2, M - 2, M - 1} & set(range(M)))
    acc_w, y_w = oracle.linear_w4(x[rows], bits, e, zp, wq, sw)
    assert np.array_equal(outs[0][0][rows].astype(np.int64), acc_w)
    assert_f16_close(outs[0][1][rows], y_w, "y")


@pytest.mark.parametrize("M,K,N,bits,zp,x_kind", [(448, 4096, 1000, 8, 0, "f16"), (300, 1024, 2100, 4, 9, "f16"),
                                                    (512, 4096, 4096, 8, 0, "q"), (321, 512, 5000, 8, 131, "f16")])
def test_tiled_64_token_tiles(agq, oracle, M, K, N, bits, zp, x_kind):
    """At most 128 tiles of 128 x 128 and no K split that pays: the tiled kernel runs 64-token tiles (twice the
    workgroups).  Token counts that end inside the first and inside the second half of a 128-token tile."""
    x, wq, sw = make_case(M, K, N, seed=950 + M + N, n_out=6)
    e = oracle.calibrate_act_exp(x, bits) + (1 if zp else 0)
    fn = agq.gemm_w4a8 if bits == 8 else agq.gemm_w4a4
    if x_kind == "f16":
        xin, kind = dev(x), agq.AGQ_X_F16
    elif x_kind == "dot":
        xin, kind = dev(x), agq.AGQ_X_F16_DOT
    else:
        xin, kind = agq.quantize_act(dev(x), bits, e, zp), agq.AGQ_X_Q
    acc = torch.full((M, N), -3, dtype=torch.int32, device="cuda")
    ybuf = torch.full((M, N + 8), 5.0, dtype=torch.float16, device="cuda")
    fn(xin, e, agq.pack_w4(dev(wq)), dev(sw), N, K, x_kind=kind, acc_out=acc, zp=zp, y=ybuf[:, :N])
    rows = sorted({0, 1, 31, 32, 63, 64, 127, 128, 191, 192, M // 2, M - 2, M - 1})
    acc_w, y_w = oracle.linear_w4(x[rows], bits, e, zp, wq, sw)
    got = host(ybuf)
    assert np.array_equal(host(acc)[rows].astype(np.int64), acc_w)
    assert_f16_close(got[rows, :N], y_w, "y")
    assert (got[:, N:] == 5.0).all() and not (host(acc) == -3).all(axis=1).any()     # every row written, nothing beyond


def test_tiled_split_k_multi_and_graph(agq, oracle):
    # q/k/v-style call whose tiles together are still few: one split launch over all projections; replayed as a graph
    M, K, Ns, bits = 300, 2048, [256, 100, 384], 8
    x = synth.make_activation(M, K, 4, seed=910)
    e = oracle.calibrate_act_exp(x, bits)
    xd = dev(x)
    projs, wants = [], []
    for i, N in enumerate(Ns):
        wq, sw = synth.make_weight_q4(N, K, seed=920 + i)
        projs.append((agq.pack_w4(dev(wq)), dev(sw), N, torch.empty((M, N), dtype=torch.float16, device="cuda"),
                      torch.empty((M, N), dtype=torch.int32, device="cuda")))
        wants.append(oracle.linear_w4(x, bits, e, 0, wq, sw))
    full = agq.gemm_workspace_bytes(M, sum(Ns), K)
    assert full > agq.gemm_workspace_bytes(M, 0, K)
    ws = torch.empty(full, dtype=torch.uint8, device="cuda")
    agq.gemm_w4a8_multi(xd, e, projs, K, workspace=ws)
    for (acc_w, y_w), p in zip(wants, projs):
        assert np.array_equal(host(p[4]).astype(np.int64), acc_w)
        assert_f16_close(host(p[3]), y_w, "multi split")
    eager = [host(p[3]).copy() for p in projs]
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        agq.gemm_w4a8_multi(xd, e, projs, K, workspace=ws)
    for rep in range(3):
        for p in projs:
            p[3].zero_()
        g.replay()
        torch.cuda.synchronize()
        for want, p in zip(eager, projs):
            assert np.array_equal(host(p[3]).view(np.int16), want.view(np.int16))


def test_row_groups_strided_multi(agq, oracle):
    # strided input and output, several projections, the 4-bit grid: 100 rows in seven groups (the last with four)
    M, K, Ns, bits = 100, 512, [64, 272, 100], 4
    xs = np.zeros((M, K + 64), dtype=np.float16)
    xs[:, :K] = synth.make_activation(M, K, 3, seed=77)
    xd = dev(xs)[:, :K]
    e = oracle.calibrate_act_exp(xs[:, :K], bits)
    projs, wants, outs = [], [], []
    for i, N in enumerate(Ns):
        wq, sw = synth.make_weight_q4(N, K, seed=80 + i)
        ybuf = torch.full((M, N + 24), 7.0, dtype=torch.float16, device="cuda")
        outs.append(ybuf)
        projs.append((agq.pack_w4(dev(wq)), dev(sw), N, ybuf[:, :N], None))
        wants.append(oracle.linear_w4(xs[:, :K], bits, e, 0, wq, sw)[1])
    agq.gemm_w4a4_multi(xd, e, projs, K)
    for ybuf, want, N in zip(outs, wants, Ns):
        got = host(ybuf)
        assert_f16_close(got[:, :N], want, "y")
        assert (got[:, N:] == 7.0).all()          # nothing written past a row's N columns


@pytest.mark.parametrize("bits,x_kind", [(8, "q"), (4, "f16"), (4, "q")])
def test_tiled_variants(agq, oracle, bits, x_kind):
    x, wq, sw = make_case(150, 512, 300, seed=31 + bits)
    run_linear(agq, oracle, x, wq, sw, bits, x_kind)


@pytest.mark.parametrize("M,bits", [(1, 8), (4, 8), (16, 8), (3, 4), (40, 8), (150, 4), (300, 8), (700, 4)])
def test_multi_projection_equals_single_calls(agq, oracle, M, bits):
    # q/k/v-style: several weight matrices on one activation, one call
    K = 512
    Ns = [64, 272, 100, 16]
    x = synth.make_activation(M, K, 3, seed=50 + M)
    e = oracle.calibrate_act_exp(x, bits)
    projs, wants, accs = [], [], []
    for i, N in enumerate(Ns):
        wq, sw = synth.make_weight_q4(N, K, seed=60 + i)
        acc = torch.full((M, N), -7, dtype=torch.int32, device="cuda")
        projs.append((agq.pack_w4(dev(wq)), dev(sw), N, None, acc))
        accs.append(acc)
        wants.append(oracle.linear_w4(x, bits, e, 0, wq, sw))
    fn = agq.gemm_w4a8_multi if bits == 8 else agq.gemm_w4a4_multi
    ys = fn(dev(x), e, projs, K)
    for (acc_w, y_w), acc, y in zip(wants, accs, ys):
        assert np.array_equal(host(acc).astype(np.int64), acc_w)
        assert_f16_close(host(y), y_w, "multi")
    # three projections, pre-quantized codes as input
    xq = agq.quantize_act(dev(x), bits, e, 0)
    ys = fn(xq, e, projs[:3], K, x_kind=agq.AGQ_X_Q)
    for (acc_w, y_w), y in zip(wants, ys):
        assert_f16_close(host(y), y_w, "multi q")


@pytest.mark.parametrize("M,K,Ns", [(9, 8192, [4100]), (16, 1024, [4096, 4096, 1000]), (13, 4096, [11008, 11008]),
                                     (12, 11008, [272]), (6, 16384, [64, 16]), (16, 8320, [48]),
                                     (5, 1024, [8192, 8200]), (8, 512, [16390]), (7, 512, [16370]), (4, 512, [16400]),
                                     (11, 5120, [4200]), (16, 6144, [2000, 2200]), (9, 2048, [4099, 4102]),
                                     (6, 640, [8200]), (8, 384, [8192]), (16, 128, [4112, 16, 4000]),
                                     (16, 512, [24600]), (6, 512, [24600]), (10, 7168, [12304]), (16, 2048, [24576]),
                                     (16, 256, [49200]), (16, 128, [49152]), (9, 384, [30000, 5000, 77]),
                                     (7, 5120, [6200, 6200])])
def test_decode_many_tiles_per_workgroup(agq, oracle, M, K, Ns):
    """5..16 rows with more channel tiles than compute units: one workgroup per
    compute unit serves several tiles, with K split over its wavefronts and up
    to six of its tiles in flight (K up to 8192; one to four chunks of K per
    wavefront, a K that leaves wavefronts idle, odd widths and pitches, tiles of
    several projections in one workgroup, the largest count it takes in one
    round) or, beyond that, in rounds (one full round and a last one of none,
    one or several tiles; two full rounds and nothing left); K above 8192,
    small tile counts and fewer rows stay on the per-tile kernel."""
    x = synth.make_activation(M, K, 4, seed=70 + M)
    e = oracle.calibrate_act_exp(x, 8)
    projs, wants = [], []
    for i, N in enumerate(Ns):
        wq, sw = synth.make_weight_q4(N, K, seed=80 + i)
        acc = torch.full((M, N), -7, dtype=torch.int32, device="cuda")
        projs.append((agq.pack_w4(dev(wq)), dev(sw), N, None, acc))
        wants.append(oracle.linear_w4(x, 8, e, 0, wq, sw))
    ys = agq.gemm_w4a8_multi(dev(x), e, projs, K)
    for (acc_w, y_w), pr, y in zip(wants, projs, ys):
        assert np.array_equal(host(pr[4]).astype(np.int64), acc_w)
        assert_f16_close(host(y), y_w, "many tiles")


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("e", [-16, -15, -14, -3, 0, 5, 14, 15])
@pytest.mark.parametrize("M", [4, 16])
def test_decode_prologue_every_fp16_value(agq, oracle, M, e, bits):
    """The Eq.2 prologue of the few-token kernels over every finite fp16 bit
    pattern (ties, subnormals, both infinities) at exponents on both sides of
    the range its half-precision arithmetic covers: a single wrong code shows in
    the exact accumulators."""
    pat = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    vals = pat.view(np.float16)
    vals = vals[~np.isnan(vals)]
    K = 128 * ((vals.size + M * 128 - 1) // (M * 128))
    x = np.zeros(M * K, np.float16)
    x[: vals.size] = vals
    x = x.reshape(M, K)
    rng = np.random.default_rng(e + 100)
    wq = rng.integers(-8, 8, size=(32, K)).astype(np.int8)
    wq[wq == 0] = 1                      # every code reaches every accumulator of its row
    sw = np.full(32, 2.0 ** -12, np.float16)
    run_linear(agq, oracle, x, wq, sw, bits, e=e, check_y=False)


@pytest.mark.parametrize("M,K,N,pad", [(1, 4096, 272, 40), (4, 1024, 100, 40), (7, 768, 64, 40), (16, 4096, 64, 40),
                                       (16, 1024, 4200, 40), (150, 512, 300, 40), (16, 1024, 4200, 41),
                                       (12, 384, 24650, 40), (6, 256, 24650, 43)])
def test_strided_input_and_output(agq, oracle, M, K, N, pad):
    """Activation rows and output rows with a pitch larger than their width
    (views into wider buffers): every kernel variant must honour ldx and ldy,
    and must leave the columns beyond N untouched (also with an output pitch
    that rules out the wide stores, and in the multi-round kernel)."""
    x, wq, sw = make_case(M, K, N, seed=300 + M + K + N)
    e = oracle.calibrate_act_exp(x, 8)
    acc_want, y_want = oracle.linear_w4(x, 8, e, 0, wq, sw)
    xbuf = torch.full((M, K + 64), 77.0, dtype=torch.float16, device="cuda")
    xbuf[:, :K] = dev(x)
    ybuf = torch.full((M, N + pad), -5.0, dtype=torch.float16, device="cuda")
    acc = torch.full((M, N), -12345, dtype=torch.int32, device="cuda")
    agq.gemm_w4a8(xbuf[:, :K], e, agq.pack_w4(dev(wq)), dev(sw), N, K, y=ybuf[:, :N], acc_out=acc)
    assert np.array_equal(host(acc).astype(np.int64), acc_want)
    yh = host(ybuf)
    assert_f16_close(yh[:, :N], y_want, "strided y")
    assert np.all(yh[:, N:] == np.float16(-5.0)), "wrote past the row"


def test_graph_replay_matches_eager(agq, oracle):
    """The decode calls are meant to be replayed from a HIP graph (a decode step is
    launch-bound).  Capture one call of each few-token kernel variant after an
    eager warm-up, replay several times with eager work in between, and compare
    every replay with the eager result and with the oracle."""
    cases = []
    for M, K, Ns in ((1, 4096, [272]), (4, 1024, [100, 64]), (16, 4096, [64]), (16, 1024, [4096, 300]),
                     (9, 256, [24700])):
        x = synth.make_activation(M, K, 4, seed=400 + M + K)
        e = oracle.calibrate_act_exp(x, 8)
        projs, wants = [], []
        for i, N in enumerate(Ns):
            wq, sw = synth.make_weight_q4(N, K, seed=410 + i)
            projs.append((agq.pack_w4(dev(wq)), dev(sw), N, torch.zeros((M, N), dtype=torch.float16, device="cuda"), None))
            wants.append(oracle.linear_w4(x, 8, e, 0, wq, sw)[1])
        cases.append((dev(x), e, projs, K, wants))

    def run_all():
        for xd, e, projs, K, _ in cases:
            agq.gemm_w4a8_multi(xd, e, projs, K)

    run_all()                                   # eager: one-time set-up happens here
    eager = [[host(p[3]).copy() for p in projs] for _, _, projs, _, _ in cases]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run_all()
    for rep in range(3):
        for _, _, projs, _, _ in cases:
            for p in projs:
                p[3].fill_(float(rep))          # eager work between replays; also proves the replay writes
        torch.cuda.synchronize()
        graph.replay()
        for (_, _, projs, _, wants), eag in zip(cases, eager):
            for p, y_e, y_w in zip(projs, eag, wants):
                got = host(p[3])
                assert np.array_equal(got.view(np.uint16), y_e.view(np.uint16)), "replay differs from eager"
                assert_f16_close(got, y_w, "graph replay")


@pytest.mark.parametrize("x_kind", ["f16", "q"])
@pytest.mark.parametrize("bits,zp", [(8, 128), (8, 117), (8, 1), (8, 255), (4, 8), (4, 5), (4, 15)])
@pytest.mark.parametrize("M,K,N", [(1, 512, 48), (4, 1024, 100), (7, 768, 64), (16, 768, 4200), (150, 512, 300),
                                   (6, 384, 8300), (16, 256, 24600)])
def test_unsigned_grid_with_zero_point(agq, oracle, M, K, N, bits, zp, x_kind):
    """Eq.2's unsigned grid inside the GEMMs: acc = sum_k (q - zp) w with q in
    [0, 2^b - 1], through every kernel variant and both input kinds, including
    odd zero points (ties) and zero points at both ends of the grid."""
    x, wq, sw = make_case(M, K, N, seed=500 + M + K + N + zp)
    e = oracle.calibrate_act_exp(x, bits) + 1          # the data then spans about half the unsigned grid around zp
    run_linear(agq, oracle, x, wq, sw, bits, x_kind=x_kind, e=e, zp=zp)


def test_unsigned_grid_every_fp16_value(agq, oracle):
    """The unsigned-grid prologue over every finite fp16 bit pattern, for an even
    and an odd zero point, in and out of the range of the half-precision path."""
    pat = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    vals = pat.view(np.float16)
    vals = vals[~np.isnan(vals)]
    M = 16
    K = 128 * ((vals.size + M * 128 - 1) // (M * 128))
    x = np.zeros(M * K, np.float16)
    x[: vals.size] = vals
    x = x.reshape(M, K)
    rng = np.random.default_rng(77)
    wq = rng.integers(-8, 8, size=(32, K)).astype(np.int8)
    wq[wq == 0] = 1
    sw = np.full(32, 2.0 ** -12, np.float16)
    for e, zp in ((-3, 128), (0, 99), (5, 200), (-16, 131)):
        run_linear(agq, oracle, x, wq, sw, 8, e=e, zp=zp, check_y=False)
    run_linear(agq, oracle, x[:4], wq, sw, 4, e=-2, zp=7, check_y=False)


def test_extreme_operands_hit_the_bound(agq, oracle):
    # all codes at -128 and all weights at -8: acc = 128 * 8 * K exactly, the
    # largest value the accumulator can take (times 16 inside the kernel)
    for M in (3, 40):
        K, N = 13824, 32
        x = np.full((M, K), -128.0, np.float16)
        wq = np.full((N, K), -8, np.int8)
        sw = np.full(N, 2.0 ** -10, np.float16)
        run_linear(agq, oracle, x, wq, sw, 8, e=0)


def test_clipping_and_small_exponent(agq, oracle):
    # an exponent that is too small for the data: codes saturate on both sides
    x, wq, sw = make_case(9, 256, 64, seed=5)
    run_linear(agq, oracle, x, wq, sw, 8, e=-4)
    run_linear(agq, oracle, x, wq, sw, 4, e=-2)
    x, wq, sw = make_case(70, 256, 64, seed=6)
    run_linear(agq, oracle, x, wq, sw, 8, e=-4)


def test_empty_batch(agq):
    wq, sw = synth.make_weight_q4(16, 128, 1)
    packed = agq.pack_w4(dev(wq))
    x = torch.zeros((0, 128), dtype=torch.float16, device="cuda")
    y = agq.gemm_w4a8(x, 0, packed, dev(sw), 16, 128)
    assert y.shape == (0, 16)


def test_deterministic_repeat(agq, oracle):
    x, wq, sw = make_case(16, 4096, 4096, seed=9)
    e = oracle.calibrate_act_exp(x, 8)
    packed, xd, swd = agq.pack_w4(dev(wq)), dev(x), dev(sw)
    first = host(agq.gemm_w4a8(xd, e, packed, swd, 4096, 4096)).copy()
    for _ in range(20):
        assert np.array_equal(host(agq.gemm_w4a8(xd, e, packed, swd, 4096, 4096)).view(np.uint16), first.view(np.uint16))


def test_first_call_of_a_process_under_graph_capture(agq):
    """The calls enqueue kernels only, the very first one of a process included (its one-time host-side set-up is
    not a stream operation): a child process captures its first GEMM calls (the shapes that use the kernel with
    the activation in LDS, and the per-tile kernel), replays the graph and compares with eager calls made after."""
    import os
    import subprocess
    import sys
    code = r"""
import sys, numpy as np, torch
sys.path.insert(0, %r)
from paper_2312_05693_amd import binding as agq, synth
agq.lib()
dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
cases = []
for (M, K, N, seed) in ((12, 256, 4352, 1), (3, 512, 80, 2)):
    x = synth.make_activation(M, K, 2, seed)
    wq, sw = synth.make_weight_q4(N, K, seed)
    packed = torch.empty(agq.pack_w4_bytes(N, K), dtype=torch.uint8, device="cuda")
    cases.append((M, K, N, dev(x), dev(wq), dev(sw), packed, torch.zeros((M, N), dtype=torch.float16, device="cuda")))
torch.cuda.synchronize()
side = torch.cuda.Stream()
g = torch.cuda.CUDAGraph()
with torch.cuda.graph(g, stream=side):
    for (M, K, N, xd, wqd, swd, packed, y) in cases:
        agq.pack_w4(wqd, packed=packed)
        agq.gemm_w4a8(xd, -3, packed, swd, N, K, y=y)
g.replay()
torch.cuda.synchronize()
for (M, K, N, xd, wqd, swd, packed, y) in cases:
    want = agq.gemm_w4a8(xd, -3, agq.pack_w4(wqd), swd, N, K)
    torch.cuda.synchronize()
    assert y.abs().sum().item() > 0 and torch.equal(y.view(torch.int16), want.view(torch.int16)), (M, K, N)
print("CAPTURED_FIRST_CALL_OK")
""" % os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=110)
    assert r.returncode == 0 and "CAPTURED_FIRST_CALL_OK" in r.stdout, r.stdout[-2000:] + r.stderr[-2000:]


# ------------------------------------------------------------------ the paper-shaped configurations

def test_config0_opt125m_w4a8(agq, oracle):
    # single W4A8 linear: X fp16 [128,768] with 4 outlier channels, W [768,768], seed 0
    x, wq, sw = make_case(128, 768, 768, seed=0, n_out=4)
    e = run_linear(agq, oracle, x, wq, sw, 8)
    assert e in (-2, -1, 0)


def sampled_linear(agq, oracle, M, K, N, bits, seed, n_out, rows=None):
    """Full-size GEMM on the GPU in the benchmark's launch configuration.  rows: the rows whose accumulators the
    oracle computes (its C loops), compared bit for bit; None = the whole problem.  On top, at any size: the column
    sums and the row sums of the accumulators against what the codes and weights give (a wrong tile shows in at
    least its rows' or its columns' sums unless its errors cancel both ways), and every row's fp16 output against
    the oracle's dequantization of that row's accumulators (the epilogue and its store, everywhere)."""
    x, wq, sw = make_case(M, K, N, seed=seed, n_out=n_out)
    e = oracle.calibrate_act_exp(x, bits)
    packed = agq.pack_w4(dev(wq))
    acc = torch.empty((M, N), dtype=torch.int32, device="cuda")
    fn = agq.gemm_w4a8 if bits == 8 else agq.gemm_w4a4
    y = fn(dev(x), e, packed, dev(sw), N, K, acc_out=acc)
    acc_h, y_h = host(acc), host(y)
    qall = oracle.quantize_act(x, bits, e, 0).astype(np.int8)
    rows = list(range(M)) if rows is None else sorted(set(min(r, M - 1) for r in rows))
    want = oracle.gemm_int_c(qall[rows], wq, threads=oracle.c_max_threads())
    assert np.array_equal(acc_h[rows], want)
    assert_f16_close(y_h[rows], oracle.dequant_out(want, e, sw), "y")
    q64, w64 = qall.astype(np.int64), wq.astype(np.int64)
    assert np.array_equal(acc_h.astype(np.int64).sum(axis=0), q64.sum(axis=0) @ w64.T)      # per column
    assert np.array_equal(acc_h.astype(np.int64).sum(axis=1), q64 @ w64.sum(axis=0))        # per row
    assert_f16_close(y_h, oracle.dequant_out(acc_h, e, sw), "y of every row from its accumulators")


def tile_rows(M):
    """One row in every 32-token block (the MFMA tile height of the tiled kernel), at a position inside the block
    that changes from block to block, plus the edges of the 128-token tiles."""
    rows = [32 * b + (11 * b + 5) % 32 for b in range((M + 31) // 32)]
    return rows + [0, 1, 31, 32, 127, 128, M // 2 - 1, M // 2, M - 129, M - 128, M - 1]


@pytest.mark.parametrize("M", [1, 4, 16])
@pytest.mark.parametrize("K,N", [(4096, 4096), (4096, 11008), (11008, 4096)])
def test_config1_llama7b_decode(agq, oracle, M, K, N):
    sampled_linear(agq, oracle, M, K, N, 8, seed=1, n_out=4, rows=range(M))


@pytest.mark.parametrize("K,N", [(4096, 4096), (4096, 11008), (11008, 4096)])
def test_config2_llama7b_prefill_w4a8(agq, oracle, K, N):
    # every accumulator of every shape against the oracle (34 / 92 / 92 GMAC of its plain loops)
    sampled_linear(agq, oracle, 2048, K, N, 8, seed=2, n_out=synth.n_outlier_channels(K), rows=None)


@pytest.mark.parametrize("K,N", [(4096, 4096), (4096, 11008), (11008, 4096)])
def test_config3_llama7b_prefill_w4a4(agq, oracle, K, N):
    # the same kernels on the 4-bit grid: a row of every 32-token block, plus the checks that cover every row
    sampled_linear(agq, oracle, 2048, K, N, 4, seed=3, n_out=synth.n_outlier_channels(K), rows=tile_rows(2048))


# ------------------------------------------------------------------ Eq.3 path, pruning

@pytest.mark.parametrize("H,S,D,qmax,causal", [(2, 64, 16, 15, True), (3, 128, 64, 15, True), (2, 192, 128, 7, True),
                                                (1, 72, 32, 15, True), (2, 64, 128, 15, False), (1, 200, 48, 7, False)])
def test_log2_attn_small(agq, oracle, H, S, D, qmax, causal):
    p, v = synth.make_attention(H, S, D, seed=H + S + D)
    if not causal:      # make the upper triangle meaningful too
        p2, _ = synth.make_attention(H, S, D, seed=99)
        p = (0.5 * p.astype(np.float32) + 0.5 * p2.astype(np.float32).transpose(0, 2, 1)).astype(np.float16)
        p = np.minimum(p, np.float16(1.0))
    e_v = oracle.calibrate_act_exp(v.reshape(H * S, D), 8)
    vq = oracle.quantize_act(v.reshape(H * S, D), 8, e_v, 0).astype(np.int8).reshape(H, S, D)
    A, O = oracle.attn_v_log2(p, vq, e_v, qmax, causal)
    o, codes, score = agq.log2_quant_softmax(dev(p), dev(vq), e_v, qmax=qmax, causal=causal, want_codes=True)
    assert np.array_equal(host(o).view(np.uint16), O.view(np.uint16))       # exact integers, one rounding
    assert np.array_equal(host(codes), oracle.log2_codes_packed(p, qmax, causal))
    assert np.array_equal(host(score).astype(np.int64), oracle.start_token_score(p))


@pytest.mark.parametrize("H,S,D,qmax,causal", [(8, 264, 128, 15, True), (16, 136, 64, 7, True), (2, 328, 256, 15, True),
                                                (1, 8, 16, 15, True), (3, 200, 240, 7, False), (8, 392, 128, 15, False)])
def test_log2_attn_shapes_without_codes(agq, oracle, H, S, D, qmax, causal):
    """The variant that skips the code map, over: several row blocks with a ragged
    last one, head counts that do and do not spread evenly over the chip's eight
    partitions, head dims above 128 (two column blocks) and the smallest S."""
    p, v = synth.make_attention(H, S, D, seed=7 * H + S + D)
    e_v = oracle.calibrate_act_exp(v.reshape(H * S, D), 8)
    vq = oracle.quantize_act(v.reshape(H * S, D), 8, e_v, 0).astype(np.int8).reshape(H, S, D)
    _, O = oracle.attn_v_log2(p, vq, e_v, qmax, causal)
    o, _, score = agq.log2_quant_softmax(dev(p), dev(vq), e_v, qmax=qmax, causal=causal, want_codes=False)
    assert np.array_equal(host(o).view(np.uint16), O.view(np.uint16))
    assert np.array_equal(host(score).astype(np.int64), oracle.start_token_score(p))
    o2, codes, _ = agq.log2_quant_softmax(dev(p), dev(vq), e_v, qmax=qmax, causal=causal, want_codes=True,
                                          want_score=False)
    assert np.array_equal(host(o2).view(np.uint16), O.view(np.uint16))
    assert np.array_equal(host(codes), oracle.log2_codes_packed(p, qmax, causal))


def test_log2_codes_all_fp16_probabilities(agq, oracle):
    # every fp16 in [0,1] once, through the kernel's code output (non-causal rows)
    vals = np.arange(0x3C00 + 1, dtype=np.uint16).view(np.float16)
    S = 128
    n = (vals.size + S - 1) // S
    flat = np.concatenate([vals, np.zeros(n * S - vals.size, np.float16)])
    H = (n + S - 1) // S
    p = np.zeros((H, S, S), np.float16)
    p.reshape(-1)[: flat.size] = flat
    vq = np.zeros((H, S, 16), np.int8)
    for qmax in (15, 7):
        _, codes, _ = agq.log2_quant_softmax(dev(p), dev(vq), 0, qmax=qmax, causal=False, want_codes=True,
                                             want_score=False)
        assert np.array_equal(host(codes), oracle.log2_codes_packed(p, qmax, causal=False))


@pytest.mark.parametrize("S,keep,d", [(64, 32, 64), (100, 1, 8), (257, 200, 40), (2048, 1024, 5120), (7, 7, 16)])
def test_prune(agq, oracle, S, keep, d):
    rng = np.random.default_rng(S + keep)
    score = rng.integers(0, max(S // 3, 2), size=S).astype(np.int32)      # many ties
    x = rng.standard_normal((S, d)).astype(np.float16)
    idx, out = agq.prune_tokens(dev(score), keep, dev(x))
    want_idx, want_x = oracle.prune_tokens(score, keep, x)
    assert np.array_equal(host(idx), want_idx)
    assert np.array_equal(host(out).view(np.uint16), want_x.view(np.uint16))


@pytest.mark.parametrize("kind", ["equal", "signed", "extremes", "max_size", "keep_none"])
def test_prune_degenerate(agq, oracle, kind):
    """Score patterns that stress the threshold search: one value everywhere
    (index order alone decides), both signs, the int32 limits, the largest S the
    call takes, and n_keep = 0."""
    rng = np.random.default_rng(11)
    S, keep, d = 1000, 333, 16
    if kind == "equal":
        score = np.full(S, 5, np.int32)
    elif kind == "signed":
        score = rng.integers(-50, 50, size=S).astype(np.int32)
    elif kind == "extremes":
        score = rng.choice(np.array([-2**31, -1, 0, 1, 2**31 - 1], np.int64), size=S).astype(np.int32)
    elif kind == "max_size":
        S, keep = 8192, 4097
        score = rng.integers(-2**31, 2**31, size=S).astype(np.int32)
        score[::7] = score[0]
    else:
        keep = 0
        score = rng.integers(0, 9, size=S).astype(np.int32)
    x = rng.standard_normal((S, d)).astype(np.float16)
    idx, out = agq.prune_tokens(dev(score), keep, dev(x))
    want_idx, want_x = oracle.prune_tokens(score, keep, x)
    assert np.array_equal(host(idx), want_idx)
    assert np.array_equal(host(out).view(np.uint16), want_x.view(np.uint16))


def test_config4_attention_block_reduced(agq, oracle):
    """Config 4 at a size the oracle finishes: heads x head_dim as LLaMA-13B
    scaled down (H=4, D=128, S=256), top 50 % of tokens, then two W4A8
    projections on the survivors."""
    H, D, S = 4, 128, 256
    hid, ffn = H * D, 1408
    p, v = synth.make_attention(H, S, D, seed=4)
    e_v = oracle.calibrate_act_exp(v.reshape(H * S, D), 8)
    vq = oracle.quantize_act(v.reshape(H * S, D), 8, e_v, 0).astype(np.int8).reshape(H, S, D)
    gamma = oracle.progressive_ratio(0.5, 1)
    keep = oracle.n_keep(S, gamma)
    # oracle chain
    _, O = oracle.attn_v_log2(p, vq, e_v, 15, True)
    t = oracle.start_token_score(p)
    idx_w, xp = oracle.prune_tokens(t, keep, O)
    w1, s1 = synth.make_weight_q4(hid, hid, 41)
    w2, s2 = synth.make_weight_q4(ffn, hid, 42)
    e1 = oracle.calibrate_act_exp(xp, 8)
    _, y1 = oracle.linear_w4(xp, 8, e1, 0, w1, s1)
    # GPU chain through the C ABI
    o, _, score = agq.log2_quant_softmax(dev(p), dev(vq), e_v, qmax=15, causal=True)
    idx, xg = agq.prune_tokens(score, keep, o)
    assert np.array_equal(host(idx), idx_w)
    assert np.array_equal(host(xg).view(np.uint16), xp.view(np.uint16))
    eg = int(host(agq.calibrate_act_exp(xg, 8))[0])
    assert eg == e1
    acc1 = torch.empty((keep, hid), dtype=torch.int32, device="cuda")
    yg1 = agq.gemm_w4a8(xg, eg, agq.pack_w4(dev(w1)), dev(s1), hid, hid, acc_out=acc1)
    assert_f16_close(host(yg1), y1, "y1")
    # second projection: fed with the oracle's y1 on both sides so that a legal
    # 1-ulp difference in y1 cannot change a code of the next layer
    e2 = oracle.calibrate_act_exp(y1, 8)
    acc2_w, y2 = oracle.linear_w4(y1, 8, e2, 0, w2, s2)
    acc2 = torch.empty((keep, ffn), dtype=torch.int32, device="cuda")
    yg2 = agq.gemm_w4a8(dev(y1), e2, agq.pack_w4(dev(w2)), dev(s2), ffn, hid, acc_out=acc2)
    assert np.array_equal(host(acc2).astype(np.int64), acc2_w)
    assert_f16_close(host(yg2), y2, "y2")


def test_config4_attention_block_full(agq, oracle):
    """Config 4 at full size: 40 heads x 128, 2048 tokens, 4-bit log2 codes times
    int8 V, keep the top half of the tokens by start-token attention, then W4A8
    5120->5120 and 5120->13824 on the survivors.  The oracle does the attention
    product with an exact float64 matmul and the projections with its C loops
    on sampled rows."""
    H, D, S = synth.LLAMA13B_ATTN["H"], synth.LLAMA13B_ATTN["D"], synth.LLAMA13B_ATTN["S"]
    p, v = synth.make_attention(H, S, D, seed=4)
    e_v = oracle.calibrate_act_exp(v.reshape(H * S, D), 8)
    vq = oracle.quantize_act(v.reshape(H * S, D), 8, e_v, 0).astype(np.int8).reshape(H, S, D)
    keep = oracle.n_keep(S, oracle.progressive_ratio(0.5, 1))
    assert keep == 1024
    _, O = oracle.attn_v_log2(p, vq, e_v, 15, True)
    t = oracle.start_token_score(p)
    idx_w, xp = oracle.prune_tokens(t, keep, O)

    o, _, score = agq.log2_quant_softmax(dev(p), dev(vq), e_v, qmax=15, causal=True)
    assert np.array_equal(host(score).astype(np.int64), t)
    assert np.array_equal(host(o).view(np.uint16), O.view(np.uint16))
    idx, xg = agq.prune_tokens(score, keep, o)
    assert np.array_equal(host(idx), idx_w)
    assert np.array_equal(host(xg).view(np.uint16), xp.view(np.uint16))

    rows = [0, 1, 17, 511, 512, 1000, 1023] + list(range(300, 309))
    x_in = xp
    for k, (name, K, N) in enumerate(synth.LLAMA13B_TAIL):
        wq, sw = synth.make_weight_q4(N, K, 40 + k)
        e = oracle.calibrate_act_exp(x_in, 8)
        assert int(host(agq.calibrate_act_exp(dev(x_in), 8))[0]) == e
        acc = torch.empty((keep, N), dtype=torch.int32, device="cuda")
        y = agq.gemm_w4a8(dev(x_in), e, agq.pack_w4(dev(wq)), dev(sw), N, K, acc_out=acc)
        q = oracle.quantize_act(x_in, 8, e, 0).astype(np.int8)
        if k == 0:   # whole first projection through the C loops: its output feeds the next one
            want = oracle.gemm_int_c(q, wq, threads=oracle.c_max_threads())
            assert np.array_equal(host(acc), want)
            y_w = oracle.dequant_out(want, e, sw)
            assert_f16_close(host(y), y_w, name)
            x_in = y_w
        else:
            want = oracle.gemm_int_c(q[rows], wq, threads=oracle.c_max_threads())
            assert np.array_equal(host(acc)[rows], want)
            assert_f16_close(host(y)[rows], oracle.dequant_out(want, e, sw), name)


# ------------------------------------------------------------------ TRIP (Eq.5-8, Section 4.4)

def trip_case(M, K, N, seed, n_out, kmax, bits, oracle):
    x, wq, sw = make_case(M, K, N, seed, n_out)
    e = oracle.trip_base_exp(x, bits, kmax)
    return x, wq, sw, e


@pytest.mark.parametrize("M,K,bits,kmax,zp", [(1, 128, 8, 4, 0), (7, 384, 8, 4, 0), (64, 512, 8, 3, 0),
                                              (300, 1024, 4, 2, 0), (33, 256, 8, 4, 131), (16, 4096, 8, 4, 0)])
def test_trip_search_matches_oracle(agq, oracle, M, K, bits, kmax, zp):
    x = synth.make_activation(M, K, max(2, K // 100), seed=31 + M)
    e = oracle.trip_base_exp(x, bits, kmax)
    want = oracle.trip_search(x, bits, e, zp, kmax)
    got = host(agq.trip_search(dev(x), bits, e, kmax, zp=zp))
    assert got.dtype == np.int8 and np.array_equal(got, want)
    if zp == 0 and kmax == 4 and M >= 7:
        assert want.max() == kmax and (want > 0).sum() < K // 4     # the recipe's outlier channels


def test_trip_search_strided_infinite_and_empty(agq, oracle):
    rng = np.random.default_rng(32)
    big = (rng.standard_normal((40, 200)) * 3).astype(np.float16)
    big[3, 17] = np.inf
    big[9, 60] = -np.inf
    x = big[:, 8:136]                                    # a view: row pitch 200, 128 channels
    xd = dev(big)[:, 8:136]
    want = oracle.trip_search(np.ascontiguousarray(x), 8, -5, 0, 4)
    assert np.array_equal(host(agq.trip_search(xd, 8, -5, 4)), want)
    assert want[9] == 0 and want[52] == 0                 # the channels holding the infinities
    empty = torch.empty((0, 128), dtype=torch.float16, device="cuda")
    assert not host(agq.trip_search(empty, 8, 0, 4)).any()


def random_alpha(rng, K, counts):
    """counts[a-1] channels get factor a (a = 1..4), the rest 0."""
    alpha = np.zeros(K, dtype=np.int8)
    pick = rng.choice(K, size=sum(counts), replace=False)
    pos = 0
    for a, c in enumerate(counts, start=1):
        alpha[pick[pos:pos + c]] = a
        pos += c
    return alpha


def test_trip_pack_roundtrip_and_tables(agq, oracle):
    rng = np.random.default_rng(33)
    for N, K, counts in ((16, 128, (0, 0, 0, 0)), (40, 256, (3, 0, 0, 2)), (300, 384, (130, 1, 0, 5)),
                         (64, 2048, (0, 0, 129, 256))):
        wq = rng.integers(-8, 8, size=(N, K)).astype(np.int8)
        alpha = random_alpha(rng, K, counts)
        E = sum((c + 127) // 128 for c in counts)
        assert agq.trip_extra_chunks(alpha, K) == E
        packed, n_extra = agq.pack_w4_trip(dev(wq), alpha)
        assert n_extra == E and packed.numel() == agq.lib().agq_pack_w4_trip_bytes(N, K, E)
        assert np.array_equal(host(agq.unpack_w4_trip(packed, N, K, E)), wq)
        # the weight sums behind the nibbles carry the factors
        npad = (N + 255) // 256 * 256
        nib_bytes = npad * (K // 128 + E) * 64
        wsum = host(packed)[nib_bytes: nib_bytes + 4 * npad].view(np.int32)
        assert np.array_equal(wsum[:N], (wq.astype(np.int64) << alpha[None, :].astype(np.int64)).sum(axis=1))
        assert not wsum[N:].any()
    # invalid factor sets are refused on the host
    bad = np.zeros(128, dtype=np.int8)
    bad[3] = 5
    with pytest.raises(agq.AgqError):
        agq.trip_extra_chunks(bad, 128)
    many = np.ones(128 * 17, dtype=np.int8)              # 17 chunks of factor 1
    with pytest.raises(agq.AgqError):
        agq.trip_extra_chunks(many, 128 * 17)


def run_trip_linear(agq, oracle, x, wq, sw, bits, e, alpha, zp=0):
    N, K = wq.shape
    M = x.shape[0]
    packed, n_extra = agq.pack_w4_trip(dev(wq), alpha)
    acc = torch.empty((M, N), dtype=torch.int32, device="cuda")
    y = agq.gemm_trip(dev(x), bits, e, packed, n_extra, dev(sw), N, K, acc_out=acc, zp=zp)
    want_acc, want_y = oracle.linear_w4_trip(x, bits, e, zp, alpha, wq, sw)
    assert np.array_equal(host(acc).astype(np.int64), want_acc), (M, K, N, bits, zp)
    assert_f16_close(host(y), want_y, "trip linear %s" % ((M, K, N, bits, zp),))


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("M", [1, 3, 4, 7, 8, 13, 16])
def test_trip_linear_decode(agq, oracle, M, bits):
    K, N, kmax = 1024, 272, 4 if bits == 8 else 3
    x, wq, sw, e = trip_case(M, K, N, 40 + M, 10, kmax, bits, oracle)
    alpha = oracle.trip_search(x, bits, e, 0, kmax)
    assert (alpha > 0).any()
    run_trip_linear(agq, oracle, x, wq, sw, bits, e, alpha)


@pytest.mark.parametrize("M,K,N", [(2, 128, 16), (16, 11008, 48), (5, 4096, 4096), (16, 8192, 64), (9, 256, 1000)])
def test_trip_linear_decode_shapes(agq, oracle, M, K, N):
    rng = np.random.default_rng(41)
    x, wq, sw, e = trip_case(M, K, N, 50 + M, max(2, K // 100), 4, 8, oracle)
    # factors of every level, more than one chunk of one of them, unused slots in all
    alpha = random_alpha(rng, K, (min(130, K // 8), 3, 1, min(20, K // 16)))
    run_trip_linear(agq, oracle, x, wq, sw, 8, e, alpha)


@pytest.mark.parametrize("M,K,N,bits", [(17, 128, 16, 8), (100, 512, 200, 8), (256, 1024, 384, 4), (300, 4096, 130, 8)])
def test_trip_linear_tiled(agq, oracle, M, K, N, bits):
    rng = np.random.default_rng(42)
    kmax = 4 if bits == 8 else 3
    x, wq, sw, e = trip_case(M, K, N, 60 + M, max(2, K // 100), kmax, bits, oracle)
    alpha = oracle.trip_search(x, bits, e, 0, kmax)
    run_trip_linear(agq, oracle, x, wq, sw, bits, e, alpha)
    # hand-made factors: all levels, a level that fills more than one chunk, skipped levels
    run_trip_linear(agq, oracle, x, wq, sw, bits, e, random_alpha(rng, K, (K // 8 + 3, 0, 2, 7)))
    run_trip_linear(agq, oracle, x, wq, sw, bits, e, random_alpha(rng, K, (0, 0, 0, 1)))


@pytest.mark.parametrize("M,K,N,bits,zp", [(300, 4096, 300, 8, 0), (140, 8192, 700, 4, 9)])
def test_trip_tiled_split_k(agq, oracle, M, K, N, bits, zp):
    """TRIP blobs with few tiles and a long K: the K split keeps the extra steps and their shifts in the first slice.
    Against the oracle and, bit for bit, against the call with a workspace too small for a split."""
    rng = np.random.default_rng(43)
    kmax = 4 if bits == 8 else 3
    x, wq, sw, e = trip_case(M, K, N, 70 + M, K // 100, kmax, bits, oracle)
    e += 1 if zp else 0
    alpha = random_alpha(rng, K, (140, 3, 0, 20)[:kmax] + (0,) * (4 - kmax))
    packed, n_extra = agq.pack_w4_trip(dev(wq), alpha)
    assert n_extra >= 3
    full = agq.lib().agq_gemm_trip_workspace_bytes(M, N, K, n_extra)
    small = agq.lib().agq_gemm_trip_workspace_bytes(M, 0, K, n_extra)
    assert full > small == -(-M // 128) * 128 * (K + 128 * n_extra)
    res = []
    for nbytes in (full, small, full):
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda").fill_(0x5A)
        acc = torch.empty((M, N), dtype=torch.int32, device="cuda")
        y = agq.gemm_trip(dev(x), bits, e, packed, n_extra, dev(sw), N, K, acc_out=acc, zp=zp, workspace=ws)
        res.append((host(acc), host(y)))
    for a, yy in res[1:]:
        assert np.array_equal(a, res[0][0]) and np.array_equal(yy.view(np.int16), res[0][1].view(np.int16))
    rows = sorted({0, 1, 31, 32, 127, 128, M // 2, M - 1})
    want_acc, want_y = oracle.linear_w4_trip(x[rows], bits, e, zp, alpha, wq, sw)
    assert np.array_equal(res[0][0][rows].astype(np.int64), want_acc)
    assert_f16_close(res[0][1][rows], want_y, "trip split")


@pytest.mark.parametrize("M,bits,zp", [(1, 8, 0), (9, 8, 0), (16, 4, 0), (40, 8, 0), (300, 8, 131), (130, 4, 0)])
def test_trip_multi_projection(agq, oracle, M, bits, zp):
    """The factors belong to the activation: three projections packed with the same factors, one call."""
    K, Ns = 1024, [272, 64, 1000]
    x = synth.make_activation(M if M > 40 else 64, K, 10, seed=600 + M)
    e = oracle.trip_base_exp(x, bits, 4) + (1 if zp else 0)
    alpha = oracle.trip_search(x, bits, e, zp, 4)
    x = x[:M]
    projs, wants, n_extra = [], [], None
    for i, N in enumerate(Ns):
        wq, sw = synth.make_weight_q4(N, K, seed=610 + i)
        blob, n_extra = agq.pack_w4_trip(dev(wq), alpha)
        acc = torch.full((M, N), -5, dtype=torch.int32, device="cuda")
        projs.append((blob, dev(sw), N, None, acc))
        wants.append(oracle.linear_w4_trip(x, bits, e, zp, alpha, wq, sw))
    assert n_extra >= 1
    ys = agq.gemm_trip_multi(dev(x), bits, e, projs, n_extra, K, zp=zp)
    for (acc_w, y_w), (_, _, _, _, acc), y in zip(wants, projs, ys):
        assert np.array_equal(host(acc).astype(np.int64), acc_w)
        assert_f16_close(host(y), y_w, "trip multi")
    L = agq.lib()
    assert L.agq_gemm_w4a8_trip_multi(dev(x).data_ptr(), M, K, K, e, 0, None, 3, n_extra, None, 0, None) == agq.AGQ_EINVAL


@pytest.mark.parametrize("M", [4, 16, 200])
def test_trip_linear_no_factors_equals_plain(agq, oracle, M):
    """All factors zero: the TRIP layer is the plain layer (no extra chunks)."""
    K, N = 512, 144
    x, wq, sw = make_case(M, K, N, 70 + M)
    e = oracle.calibrate_act_exp(x, 8)
    alpha = np.zeros(K, dtype=np.int8)
    run_trip_linear(agq, oracle, x, wq, sw, 8, e, alpha)
    want_acc, _ = oracle.linear_w4(x, 8, e, 0, wq, sw)
    got_acc, _ = oracle.linear_w4_trip(x, 8, e, 0, alpha, wq, sw)
    assert np.array_equal(want_acc, got_acc)


@pytest.mark.parametrize("M,bits,zp", [(3, 8, 128), (16, 8, 77), (150, 8, 131), (12, 4, 9), (130, 4, 8)])
def test_trip_linear_unsigned_grid(agq, oracle, M, bits, zp):
    rng = np.random.default_rng(43)
    K, N = 640, 80
    x, wq, sw, e = trip_case(M, K, N, 80 + M, 6, 3, bits, oracle)
    run_trip_linear(agq, oracle, x, wq, sw, bits, e, random_alpha(rng, K, (9, 0, 4, 2)), zp=zp)


def test_trip_linear_extreme_values(agq, oracle):
    """Largest accumulators: every code and weight at its bound, sixteen extra chunks of factor 4."""
    M, K, N = 16, 32768 - 2048, 16
    x = np.full((M, K), 60000.0, dtype=np.float16)
    x[1::2] = -60000.0
    wq = np.full((N, K), -8, dtype=np.int8)
    wq[1::2] = 7
    sw = np.full(N, 2.0 ** -20, dtype=np.float16)
    alpha = np.zeros(K, dtype=np.int8)
    alpha[:2048] = 4
    run_trip_linear(agq, oracle, x, wq, sw, 8, 0, alpha)


def test_trip_argument_errors(agq):
    L = agq.lib()
    x = torch.zeros((4, 128), dtype=torch.float16, device="cuda")
    y = torch.zeros((4, 16), dtype=torch.float16, device="cuda")
    sw = torch.ones(16, dtype=torch.float16, device="cuda")
    blob = torch.zeros(L.agq_pack_w4_trip_bytes(16, 128, 1), dtype=torch.uint8, device="cuda")
    ok = lambda **kw: L.agq_gemm_w4a8_trip(kw.get("x", x.data_ptr()), 4, kw.get("K", 128), 128, kw.get("e", 0),
                                            kw.get("zp", 0), blob.data_ptr(), kw.get("n_extra", 1), sw.data_ptr(), 16,
                                            y.data_ptr(), kw.get("ldy", 16), None, None, 0, None)
    assert ok() == agq.AGQ_OK
    assert ok(n_extra=-1) == agq.AGQ_EINVAL and ok(n_extra=17) == agq.AGQ_EINVAL
    assert ok(K=100) == agq.AGQ_EINVAL and ok(K=65536) == agq.AGQ_EINVAL
    assert ok(zp=256) == agq.AGQ_EINVAL and ok(e=99) == agq.AGQ_EINVAL and ok(ldy=8) == agq.AGQ_EINVAL
    assert ok(x=None) == agq.AGQ_EINVAL
    assert L.agq_trip_search(x.data_ptr(), 4, 128, 128, 8, 0, 0, 5, blob.data_ptr(), None) == agq.AGQ_EINVAL
    assert L.agq_trip_search(x.data_ptr(), 4, 128, 64, 8, 0, 0, 4, blob.data_ptr(), None) == agq.AGQ_EINVAL
    assert L.agq_pack_w4_trip_bytes(16, 128, 17) == 0 and L.agq_pack_w4_trip_bytes(16, 100, 0) == 0
    torch.cuda.synchronize()


@pytest.mark.parametrize("K,N", [(4096, 4096), (4096, 11008), (11008, 4096)])
def test_trip_llama7b_full_size_sampled(agq, oracle, K, N):
    """The benchmark's TRIP configuration: factors from Eq.8 on the 2048-token activation
    with 1 % outlier channels (searched on the GPU, compared with the oracle on sampled
    channels and used from the GPU), the M = 2048 GEMM and the decode launches on its first
    rows; the oracle computes whole sampled rows with the folded weights."""
    M, bits, kmax = 2048, 8, 4
    x, wq, sw = make_case(M, K, N, seed=2, n_out=synth.n_outlier_channels(K))
    e = oracle.trip_base_exp(x, bits, kmax)
    xd = dev(x)
    alpha = host(agq.trip_search(xd, bits, e, kmax))
    cols = sorted(set(list(range(0, K, 97)) + np.flatnonzero(alpha > 0).tolist()))
    assert np.array_equal(alpha[cols], oracle.trip_search(x[:, cols], bits, e, 0, kmax))
    assert 0 < (alpha > 0).sum() <= 3 * synth.n_outlier_channels(K)
    packed, n_extra = agq.pack_w4_trip(dev(wq), alpha)
    folded = (wq.astype(np.int16) << alpha[None, :].astype(np.int16))          # |w 2^alpha| <= 128
    swd = dev(sw)

    def check(Mrun, rows):
        acc = torch.empty((Mrun, N), dtype=torch.int32, device="cuda")
        y = agq.gemm_trip(xd[:Mrun], bits, e, packed, n_extra, swd, N, K, acc_out=acc)
        acc_h, y_h = host(acc), host(y)
        q = oracle.trip_quantize(x[rows], bits, e, 0, alpha).astype(np.int64)
        want = q @ folded.T.astype(np.int64)
        assert np.array_equal(want, oracle.gemm_int_trip(q, 0, wq, alpha))
        assert np.array_equal(acc_h[rows].astype(np.int64), want)
        assert_f16_close(y_h[rows], oracle.dequant_out(want, e, sw), "trip y")

    check(M, [0, 1, 31, 32, 127, 128, 1023, 1024, 2047] + list(range(600, 612)))
    for Mrun in (1, 4, 16):
        check(Mrun, list(range(Mrun)))


# ------------------------------------------------------------------ attention from quantized Q and K

CODE_MARGIN = 1e-4      # the kernel evaluates -log2 p in fp32: codes are compared where the oracle's
                        # distance from a rounding boundary exceeds this (its error is ~1e-5); about
                        # 2 * CODE_MARGIN of all elements fall inside, which the tests assert


def unpack_codes(codes_bytes, S):
    b = np.asarray(codes_bytes)
    out = np.empty(b.shape[:-1] + (S,), dtype=np.int32)
    out[..., 0::2] = b & 0xF
    out[..., 1::2] = b >> 4
    return out


def run_qk_attention(agq, oracle, H, S, D, qmax, causal, seed, e_q=-5, e_k=-5, e_v=-4):
    qq, kq, vq = synth.make_qkv_int8(H, S, D, seed)
    o, codes, score = agq.qk_log2_softmax(dev(qq), dev(kq), dev(vq), e_q, e_k, e_v, qmax=qmax, causal=causal,
                                          want_codes=True, want_score=True)
    got_c = unpack_codes(host(codes), S)
    want_c, margin = oracle.qk_log2_codes(qq, kq, e_q, e_k, qmax, causal)
    sure = margin > CODE_MARGIN
    assert np.array_equal(got_c[sure], want_c[sure]), "codes differ away from every rounding boundary"
    # near a boundary either neighbour is valid; everywhere the code stays on the grid
    assert np.abs(got_c - want_c).max() <= 1 and got_c.min() >= 0 and got_c.max() <= qmax
    assert sure.mean() > 0.999
    if causal:
        assert (got_c[:, np.triu_indices(S, 1)[0], np.triu_indices(S, 1)[1]] == qmax).all()
    # everything behind the codes is exact: output and importance follow from the kernel's own codes
    _, want_o = oracle.attn_v_from_codes(got_c, vq, e_v, qmax, causal)
    assert np.array_equal(host(o).view(np.uint16), want_o.view(np.uint16))
    assert np.array_equal(host(score).astype(np.int64), oracle.start_token_score_codes(got_c, qmax))
    # and with its own codes the oracle gets the same output wherever no code was in doubt
    _, oracle_o = oracle.attn_v_from_codes(want_c, vq, e_v, qmax, causal)
    rows_sure = sure.all(axis=2)                              # [H, S]
    for h in range(H):
        r = np.flatnonzero(rows_sure[h])
        assert np.array_equal(host(o)[r, h * D:(h + 1) * D].view(np.uint16), oracle_o[r, h * D:(h + 1) * D].view(np.uint16))
    return float(sure.mean())


@pytest.mark.parametrize("H,S,D,qmax,causal", [(1, 128, 128, 15, True), (2, 256, 64, 15, True), (3, 384, 128, 7, True),
                                               (2, 256, 128, 15, False), (1, 512, 64, 7, False), (5, 640, 128, 15, True)])
def test_qk_attention_small(agq, oracle, H, S, D, qmax, causal):
    run_qk_attention(agq, oracle, H, S, D, qmax, causal, seed=90 + S)


def test_qk_attention_scale_and_argument_errors(agq, oracle):
    # sharper and flatter softmax through the exponents
    run_qk_attention(agq, oracle, 2, 256, 128, 15, True, seed=97, e_q=-3, e_k=-4)
    run_qk_attention(agq, oracle, 2, 256, 128, 15, True, seed=98, e_q=-8, e_k=-8)
    L = agq.lib()
    t = torch.zeros(128 * 128, dtype=torch.int8, device="cuda")
    o = torch.zeros(128 * 128, dtype=torch.float16, device="cuda")
    call = lambda **kw: L.agq_qk_log2_softmax(t.data_ptr(), t.data_ptr(), 1, kw.get("S", 128), kw.get("D", 128), 1,
                                               kw.get("qmax", 15), 0, 0, t.data_ptr(), 0, o.data_ptr(), None, None, None)
    assert call() == agq.AGQ_OK
    assert call(S=100) == agq.AGQ_EINVAL and call(S=64) == agq.AGQ_EINVAL and call(D=96) == agq.AGQ_EINVAL
    assert call(qmax=8) == agq.AGQ_EINVAL
    torch.cuda.synchronize()


def test_qk_attention_llama13b_full_size(agq, oracle):
    """The benchmark's configuration (H = 40, S = 2048, D = 128, causal); the oracle checks two
    whole heads, and the exact integer relations behind the codes are checked for every head."""
    H, S, D, qmax, e_q, e_k, e_v = 40, 2048, 128, 15, -5, -5, -4
    qq, kq, vq = synth.make_qkv_int8(H, S, D, seed=4)
    o, codes, score = agq.qk_log2_softmax(dev(qq), dev(kq), dev(vq), e_q, e_k, e_v, qmax=qmax, causal=True,
                                          want_codes=True, want_score=True)
    codes_h, o_h = host(codes), host(o)
    for h in (0, 39):
        got_c = unpack_codes(codes_h[h:h + 1], S)
        want_c, margin = oracle.qk_log2_codes(qq[h:h + 1], kq[h:h + 1], e_q, e_k, qmax, True)
        sure = margin > CODE_MARGIN
        assert np.array_equal(got_c[sure], want_c[sure]) and np.abs(got_c - want_c).max() <= 1 and sure.mean() > 0.999
        _, want_o = oracle.attn_v_from_codes(got_c, vq[h:h + 1], e_v, qmax, True)
        assert np.array_equal(o_h[:, h * D:(h + 1) * D].view(np.uint16), want_o.view(np.uint16))
    # importance: from the first column of every head's codes
    c0 = np.stack([unpack_codes(codes_h[h, :, :1], 2)[:, 0] for h in range(H)])
    assert np.array_equal(host(score).astype(np.int64), (np.int64(1) << (qmax - c0.astype(np.int64))).sum(axis=0))
    # every row's weights sum to about 2^qmax (the probabilities sum to one; rounding each to a
    # power of two moves the sum by at most a factor sqrt(2) either way)
    for h in (7, 23):
        c = unpack_codes(codes_h[h], S).astype(np.int64)
        w = np.where(np.tril(np.ones((S, S), dtype=bool)), np.int64(1) << (qmax - c), 0).sum(axis=1).astype(np.float64)
        live = c.min(axis=1) < qmax                       # rows whose weights are not all clipped at 2^0
        assert (w[live] > 2.0 ** qmax / 1.5).all() and (w[live] < 2.0 ** qmax * 1.5 + S).all()


def test_graph_replay_attention_and_trip(agq, oracle):
    """The attention calls and the TRIP decode launch enqueue kernels only: captured into one HIP graph
    after an eager warm-up, every replay must reproduce the eager results bit for bit."""
    H, S, D, qmax = 3, 256, 128, 15
    p, _ = synth.make_attention(H, S, D, seed=501)
    qq, kq, vq = synth.make_qkv_int8(H, S, D, seed=502)
    pd, qd, kd, vd = dev(p), dev(qq), dev(kq), dev(vq)
    M, K, N = 4, 1024, 144
    x, wq, sw = make_case(M, K, N, 503, 10)
    e = oracle.trip_base_exp(x, 8, 4)
    alpha = oracle.trip_search(x, 8, e, 0, 4)
    packed, n_extra = agq.pack_w4_trip(dev(wq), alpha)
    xd, swd = dev(x), dev(sw)
    L = agq.lib()
    st = lambda: torch.cuda.current_stream().cuda_stream
    o1 = torch.zeros((S, H * D), dtype=torch.float16, device="cuda")
    o2 = torch.zeros_like(o1)
    score1 = torch.zeros(S, dtype=torch.int32, device="cuda")
    score2 = torch.zeros(S, dtype=torch.int32, device="cuda")
    y = torch.zeros((M, N), dtype=torch.float16, device="cuda")

    def run_all():
        assert L.agq_log2_quant_softmax(pd.data_ptr(), H, S, D, 1, qmax, vd.data_ptr(), -4, o1.data_ptr(), None,
                                        score1.data_ptr(), st()) == 0
        score2.zero_()                                             # the call accumulates (a fill kernel, not a memset node)
        assert L.agq_qk_log2_softmax(qd.data_ptr(), kd.data_ptr(), H, S, D, 1, qmax, -5, -5, vd.data_ptr(), -4,
                                     o2.data_ptr(), None, score2.data_ptr(), st()) == 0
        assert L.agq_gemm_w4a8_trip(xd.data_ptr(), M, K, K, e, 0, packed.data_ptr(), n_extra, swd.data_ptr(), N,
                                    y.data_ptr(), N, None, None, 0, st()) == 0

    outs = (o1, o2, score1, score2, y)
    run_all()
    eager = [host(t).copy() for t in outs]
    assert_f16_close(eager[4], oracle.linear_w4_trip(x, 8, e, 0, alpha, wq, sw)[1], "trip eager")
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run_all()
    for rep in range(3):
        for t in outs:
            t.fill_(rep + 1)                                       # eager work between replays; proves the replay writes
        torch.cuda.synchronize()
        graph.replay()
        for t, want in zip(outs, eager):
            got = host(t)
            assert np.array_equal(got.view(np.uint8), want.view(np.uint8)), "replay differs from eager"


# ------------------------------------------------------------------ maximum sizes

@pytest.mark.parametrize("bits", [8, 4])
def test_gemm_longest_reduction(agq, oracle, bits):
    """K = 65536, the longest reduction the calls accept, with every operand at its extreme: the accumulator
    reaches 128 * 8 * K = 2^26 (8 * 8 * K for 4-bit codes), and 2^30 inside the kernels with their extra factors."""
    K, N = 65536, 32
    lo = -(1 << (bits - 1))
    wq = np.full((N, K), -8, np.int8)
    wq[1::2] = 7
    sw = np.full(N, 2.0 ** -14, np.float16)
    for M in (3, 40):
        x = np.full((M, K), float(lo), np.float16)
        run_linear(agq, oracle, x, wq, sw, bits, e=0)
    x, wq2, sw2 = make_case(5, K, N, seed=61, n_out=7)
    run_linear(agq, oracle, x, wq2, sw2, bits)
    assert agq.lib().agq_pack_w4_bytes(N, 2 * K) == 0


def test_log2_attn_longest_sequence(agq, oracle):
    """S = 32768, the longest sequence agq_log2_quant_softmax accepts (one head, 2 GiB of probabilities made on
    the GPU); the oracle checks sampled rows, among them the first, the last and both sides of tile borders."""
    S, D, qmax, e_v = 32768, 16, 15, -3
    g = torch.Generator(device="cuda")
    g.manual_seed(77)
    p = torch.empty((1, S, S), dtype=torch.float16, device="cuda")
    for r0 in range(0, S, 2048):
        u = torch.rand((2048, S), generator=g, device="cuda") ** 24          # a few large entries per row
        u[:, 0] += 0.05                                                       # attention to the first token
        rows = torch.arange(r0, r0 + 2048, device="cuda")[:, None]
        u = torch.where(torch.arange(S, device="cuda")[None, :] <= rows, u, torch.zeros_like(u))
        p[0, r0:r0 + 2048] = (u / u.sum(dim=1, keepdim=True)).to(torch.float16)
        del u
    vq = np.random.default_rng(78).integers(-127, 128, size=(1, S, D)).astype(np.int8)
    o, _, score = agq.log2_quant_softmax(p, dev(vq), e_v, qmax=qmax, causal=True)
    rows = np.array([0, 1, 63, 64, 127, 128, 129, 4095, 4096, 20000, 32639, 32640, 32767])
    p_rows = p[0, torch.from_numpy(rows).cuda()].cpu().numpy()
    A = oracle.attn_v_rows(p_rows, rows + 1, vq[0], qmax)
    want = np.ldexp(A.astype(np.float64), e_v - qmax).astype(np.float16)
    assert np.array_equal(host(o)[rows].view(np.uint16), want.view(np.uint16))
    col0 = p[:, :, 0].cpu().numpy()
    assert np.array_equal(host(score).astype(np.int64), oracle.start_token_score(col0[:, :, None]))


def test_qk_attention_longest_sequence(agq, oracle):
    """S = 32768 for agq_qk_log2_softmax (one head, D = 64): the oracle evaluates sampled rows, each as the
    non-causal attention of that query over the keys up to it."""
    H, S, D, qmax, e_q, e_k, e_v = 1, 32768, 64, 15, -5, -5, -4
    qq, kq, vq = synth.make_qkv_int8(H, S, D, seed=79)
    o, codes, score = agq.qk_log2_softmax(dev(qq), dev(kq), dev(vq), e_q, e_k, e_v, qmax=qmax, causal=True,
                                          want_codes=True, want_score=True)
    o_h, score_h = host(o), host(score)
    rows = [0, 1, 31, 32, 127, 128, 4095, 4096, 17000, 32639, 32640, 32767]
    for i in rows:
        got_c = unpack_codes(codes[0, i].cpu().numpy()[None, None], S)          # [1, 1, S]
        assert (got_c[0, 0, i + 1:] == qmax).all()
        want_c, margin = oracle.qk_log2_codes(qq[:, i:i + 1], kq[:, :i + 1], e_q, e_k, qmax, causal=False)
        sure = margin > CODE_MARGIN
        live = got_c[:, :, :i + 1]
        assert np.array_equal(live[sure], want_c[sure]) and np.abs(live - want_c).max() <= 1
        _, want_o = oracle.attn_v_from_codes(live, vq[:, :i + 1], e_v, qmax, causal=False)
        assert np.array_equal(o_h[i:i + 1].view(np.uint16), want_o.view(np.uint16)), i
        assert score_h[i] == 1 << (qmax - int(live[0, 0, 0]))
