"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol include/agq.h declares, sizes are right, and every argument error
is reported as a status before any HIP call is made."""
from __future__ import annotations

import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2312_05693_amd import build
    build.build(force=False)
    from paper_2312_05693_amd import binding
    return binding.lib()


def test_exports_every_declared_symbol(lib):
    from paper_2312_05693_amd import binding
    header = open(os.path.join(ROOT, "include", "agq.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(agq_[a-z0-9_]+)\s*\(", header))
    assert {"agq_quantize_act", "agq_pack_w4", "agq_gemm_w4a8", "agq_gemm_w4a4", "agq_log2_quant_softmax"} <= declared
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(binding.SIGNATURES)
    assert lib.agq_version() >= 1
    assert lib.agq_status_string(0) == b"ok"
    assert lib.agq_status_string(-1) == b"invalid argument"


def test_sizes(lib):
    # nibbles (rows padded to 256) plus one int32 weight sum per padded row
    assert lib.agq_pack_w4_bytes(768, 768) == 768 * 768 // 2 + 768 * 4
    assert lib.agq_pack_w4_bytes(4096, 4096) == 8388608 + 4096 * 4
    assert lib.agq_pack_w4_bytes(11008, 4096) == 22544384 + 11008 * 4
    assert lib.agq_pack_w4_bytes(4096, 11008) == 22544384 + 4096 * 4
    assert lib.agq_pack_w4_bytes(13824, 5120) == 35389440 + 13824 * 4
    assert lib.agq_pack_w4_bytes(100, 128) == 256 * 128 // 2 + 256 * 4
    assert lib.agq_pack_w4_bytes(16, 100) == 0                        # K must be a multiple of 128
    assert lib.agq_pack_w4_bytes(0, 128) == 0
    assert lib.agq_gemm_workspace_bytes(16, 4096, 4096) == 0
    assert lib.agq_gemm_workspace_bytes(2048, 4096, 4096) == 2048 * 4096
    # few tiles and a long K: room for the int32 partial tiles of a K split behind the codes (whole 64 KiB
    # tiles); N = 0 asks for the codes alone
    codes = 128 * 4096
    assert lib.agq_gemm_workspace_bytes(128, 0, 4096) == codes
    extra = lib.agq_gemm_workspace_bytes(128, 4096, 4096) - codes
    assert extra > 0 and extra % (128 * 128 * 4) == 0 and extra <= 256 * 128 * 128 * 4
    assert lib.agq_gemm_workspace_bytes(100, 11008, 4096) > lib.agq_gemm_workspace_bytes(100, 0, 4096)
    assert lib.agq_gemm_workspace_bytes(128, 768, 768) == 128 * 768           # short K: no split


def test_argument_errors_need_no_gpu(lib):
    EINVAL, ESIZE = -1, -2
    p = ctypes.c_void_p(4096)       # plausible, aligned, never dereferenced: every call below fails validation
    odd = ctypes.c_void_p(4100)
    g = lib.agq_gemm_w4a8
    ok_args = dict(x=p, kind=0, M=4, K=256, ldx=256, e=0, zp=0, w=p, sw=p, N=64, y=p, ldy=64, acc=None, ws=None, wsb=0, st=None)

    def call(fn=g, **kw):
        a = dict(ok_args, **kw)
        return fn(a["x"], a["kind"], a["M"], a["K"], a["ldx"], a["e"], a["zp"], a["w"], a["sw"], a["N"], a["y"],
                  a["ldy"], a["acc"], a["ws"], a["wsb"], a["st"])

    assert call(x=None) == EINVAL
    assert call(w=None) == EINVAL
    assert call(sw=None) == EINVAL
    assert call(y=None) == EINVAL
    assert call(x=odd) == EINVAL
    assert call(K=200) == EINVAL and call(K=0) == EINVAL and call(K=131072) == EINVAL
    assert call(N=0) == EINVAL and call(M=-1) == EINVAL
    assert call(ldx=128) == EINVAL and call(ldx=260) == EINVAL and call(ldy=32) == EINVAL
    assert call(e=41) == EINVAL and call(e=-41) == EINVAL
    assert call(zp=256) == EINVAL and call(zp=-1) == EINVAL   # outside Eq.2's unsigned 8-bit grid
    assert call(fn=lib.agq_gemm_w4a4, zp=16) == EINVAL
    assert call(kind=7) == EINVAL
    assert call(kind=1, ldx=264) == EINVAL           # int8 codes need ldx % 16 == 0
    assert call(fn=lib.agq_gemm_w4a4, kind=1, ldx=272) == EINVAL
    assert call(M=64, ws=None) == EINVAL             # tiled kernel needs the workspace
    assert call(M=64, ws=p, wsb=100) == ESIZE
    assert call(M=1 << 30, N=1 << 30, ldy=1 << 30, ws=p, wsb=1 << 62) == EINVAL   # more tiles than a grid holds
    assert call(M=0, x=None, y=None) == 0            # empty batch is a no-op

    # the call on the library's fixed workspace: same checks, and a size beyond the array is an error of its own
    s = lib.agq_gemm_w4a8_static

    def scall(**kw):
        a = dict(ok_args, **kw)
        return s(a["x"], a["kind"], a["M"], a["K"], a["ldx"], a["e"], a["zp"], a["w"], a["sw"], a["N"], a["y"],
                 a["ldy"], a["acc"], a["st"])

    assert scall(x=None) == EINVAL and scall(w=None) == EINVAL and scall(y=None) == EINVAL and scall(x=odd) == EINVAL
    assert scall(K=200) == EINVAL and scall(N=0) == EINVAL and scall(e=41) == EINVAL and scall(zp=256) == EINVAL
    assert scall(M=0, x=None, y=None) == 0
    assert scall(M=2049, K=16384, ldx=16384) == ESIZE      # 2176 x 16384 codes: more than the 32 MiB array
    assert scall(M=4096, K=16384, ldx=16384) == ESIZE

    from paper_2312_05693_amd.binding import AgqProj
    m = lib.agq_gemm_w4a8_multi
    good = (AgqProj * 2)(AgqProj(4096, 4096, 64, 4096, 64, None), AgqProj(4096, 4096, 32, 4096, 32, None))
    gp = ctypes.cast(good, ctypes.c_void_p)
    assert m(p, 0, 4, 256, 256, 0, 0, gp, 0, None, 0, None) == EINVAL          # count
    assert m(p, 0, 4, 256, 256, 0, 0, gp, 5, None, 0, None) == EINVAL
    assert m(p, 0, 4, 256, 256, 0, 0, None, 2, None, 0, None) == EINVAL        # no descriptors
    assert m(None, 0, 4, 256, 256, 0, 0, gp, 2, None, 0, None) == EINVAL
    bad = (AgqProj * 2)(AgqProj(4096, 4096, 64, 4096, 64, None), AgqProj(4096, None, 32, 4096, 32, None))
    assert m(p, 0, 4, 256, 256, 0, 0, ctypes.cast(bad, ctypes.c_void_p), 2, None, 0, None) == EINVAL
    bad = (AgqProj * 1)(AgqProj(4096, 4096, 64, 4096, 32, None))               # ldy < N
    assert m(p, 0, 4, 256, 256, 0, 0, ctypes.cast(bad, ctypes.c_void_p), 1, None, 0, None) == EINVAL
    assert m(p, 0, 0, 256, 256, 0, 0, gp, 2, None, 0, None) == 0               # no tokens

    q = lib.agq_quantize_act
    assert q(p, 4, 64, 64, 5, 0, 0, p, None) == EINVAL          # bits
    assert q(p, 4, 60, 64, 8, 0, 0, p, None) == EINVAL          # K % 8
    assert q(p, 4, 64, 32, 8, 0, 0, p, None) == EINVAL          # ldx < K
    assert q(p, 4, 64, 64, 8, 0, 256, p, None) == EINVAL        # zp outside the grid
    assert q(p, 4, 64, 64, 4, 0, 16, p, None) == EINVAL
    assert q(None, 4, 64, 64, 8, 0, 0, p, None) == EINVAL
    assert q(p, 0, 64, 64, 8, 0, 0, p, None) == 0               # no rows
    assert lib.agq_calibrate_act_exp(p, 4, 64, 64, 8, None, None) == EINVAL
    assert lib.agq_calibrate_act_exp(p, 4, 64, 64, 3, p, None) == EINVAL
    assert lib.agq_pack_w4(p, 16, 100, p, None, None) == EINVAL
    assert lib.agq_pack_w4(None, 16, 128, p, None, None) == EINVAL
    assert lib.agq_unpack_w4(p, 16, 128, None, None) == EINVAL
    a = lib.agq_log2_quant_softmax
    assert a(p, 2, 64, 64, 1, 9, p, 0, p, None, None, None) == EINVAL     # qmax
    assert a(p, 2, 60, 64, 1, 15, p, 0, p, None, None, None) == EINVAL    # S % 8
    assert a(p, 2, 64, 72, 1, 15, p, 0, p, None, None, None) == EINVAL    # D % 16
    assert a(p, 200, 64, 64, 1, 15, p, 0, p, None, p, None) == EINVAL     # score needs H <= 127
    assert a(None, 2, 64, 64, 1, 15, p, 0, p, None, None, None) == EINVAL
    pr = lib.agq_prune_tokens
    assert pr(p, 64, 65, p, 64, p, p, None) == EINVAL
    assert pr(p, 64, 8, p, 60, p, p, None) == EINVAL
    assert pr(p, 8193, 8, p, 64, p, p, None) == EINVAL
    assert pr(p, 64, 0, p, 64, None, None, None) == 0


def test_binding_refuses_missing_library(monkeypatch):
    from paper_2312_05693_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", "/nonexistent/libagq.so")
    with pytest.raises(RuntimeError):
        binding.lib()


def test_trip_and_fused_attention_host_checks(lib):
    """Sizes, factor validation and argument errors of the TRIP and attention-from-Q-and-K entry points
    (all decided on the host)."""
    import numpy as np
    EINVAL = -1
    K = 1024
    alpha = np.zeros(K, dtype=np.int8)
    assert lib.agq_trip_extra_chunks(alpha.ctypes.data, K) == 0
    alpha[[3, 500]] = 4
    alpha[7] = 1
    assert lib.agq_trip_extra_chunks(alpha.ctypes.data, K) == 2            # one chunk per factor in use
    alpha[:129] = 2
    assert lib.agq_trip_extra_chunks(alpha.ctypes.data, K) == 3            # 129 channels of factor 2 need two chunks
    alpha[0] = 5
    assert lib.agq_trip_extra_chunks(alpha.ctypes.data, K) == EINVAL
    alpha[0] = -1
    assert lib.agq_trip_extra_chunks(alpha.ctypes.data, K) == EINVAL
    assert lib.agq_trip_extra_chunks(None, K) == EINVAL
    assert lib.agq_trip_extra_chunks(alpha.ctypes.data, 100) == EINVAL
    # blob: nibbles of K/128 + E chunks per 16-row tile (rows padded to 256), weight sums, 32 + 128 E table
    # entries, the factors
    npad = 256
    assert lib.agq_pack_w4_trip_bytes(100, K, 2) == (npad // 16) * (K // 128 + 2) * 1024 + npad * 4 + 128 + 2 * 512 + K
    assert lib.agq_pack_w4_trip_bytes(100, K, 0) == lib.agq_pack_w4_bytes(100, K) + 128 + K
    assert lib.agq_pack_w4_trip_bytes(100, K, 17) == 0 and lib.agq_pack_w4_trip_bytes(100, 65536, 1) == 0
    assert lib.agq_gemm_trip_workspace_bytes(16, 64, K, 2) == 0
    assert lib.agq_gemm_trip_workspace_bytes(130, 0, K, 2) == 256 * (K + 256)          # the codes alone
    split_room = lib.agq_gemm_trip_workspace_bytes(130, 64, K, 2) - 256 * (K + 256)  # + partial tiles of a K split
    assert split_room > 0 and split_room % (128 * 128 * 4) == 0
    p = ctypes.c_void_p(4096)
    odd = ctypes.c_void_p(4100)
    trip = lambda **kw: lib.agq_gemm_w4a8_trip(kw.get("x", p), kw.get("M", 4), kw.get("K", K), kw.get("ldx", K),
                                               kw.get("e", 0), kw.get("zp", 0), kw.get("w", p), kw.get("E", 1), p, 64, p,
                                               kw.get("ldy", 64), None, kw.get("ws", None), 0, None)
    for bad in (dict(M=-1), dict(K=1000), dict(K=65536), dict(ldx=K - 8), dict(ldx=K + 4), dict(e=50), dict(zp=-1),
                dict(zp=256), dict(E=-1), dict(E=17), dict(ldy=32), dict(x=None), dict(x=odd), dict(w=odd),
                dict(M=200)):                                                # M = 200 needs a workspace
        assert trip(**bad) == EINVAL, bad
    assert trip(M=0) == 0
    assert lib.agq_trip_search(p, 4, K, K, 8, 0, 0, 5, p, None) == EINVAL
    assert lib.agq_trip_search(p, 4, K, K, 8, 0, 0, 4, None, None) == EINVAL
    assert lib.agq_trip_search(p, 4, K, K, 3, 0, 0, 4, p, None) == EINVAL
    qk = lambda **kw: lib.agq_qk_log2_softmax(kw.get("q", p), p, kw.get("H", 2), kw.get("S", 256), kw.get("D", 128), 1,
                                              kw.get("qmax", 15), kw.get("e_q", 0), 0, p, 0, kw.get("o", p), None, None, None)
    for bad in (dict(H=0), dict(S=64), dict(S=200), dict(S=65536), dict(D=32), dict(D=256), dict(qmax=4), dict(e_q=99),
                dict(q=None), dict(q=odd), dict(o=None)):
        assert qk(**bad) == EINVAL, bad


def _fake_block(binding, **kw):
    p = 4096
    blk = binding.AgqBlock(d=512, H=4, F=1408, qmax=15, bits_attn_out=4, rms_eps=1e-5, g_attn_f16=p, g_mlp_f16=p)
    for n in binding.BLOCK_PROJ:
        setattr(blk, "w_" + n, p)
        setattr(blk, "s_" + n, p)
    for n in binding.BLOCK_SITES:
        setattr(blk, "trip_" + n, -1)
    for k, v in kw.items():
        setattr(blk, k, v)
    return blk


def test_block_layout_and_host_checks(lib):
    from paper_2312_05693_amd import binding
    EINVAL, ESIZE = -1, -2
    L = binding.AgqBlockLayout()
    lay = lambda blk, S, keep: lib.agq_block_layout_of(ctypes.byref(blk), S, keep, ctypes.byref(L))
    blk = _fake_block(binding)
    assert lay(blk, 200, 150) == 0
    assert L.S_pad == 256 and L.h1 == 0 and L.q == 200 * 512 * 2 and L.total % 256 == 0
    offs = [getattr(L, n) for n in binding.BLOCK_TENSORS] + [L.gemm_ws, L.total]
    assert offs == sorted(offs) and all(o % 256 == 0 for o in offs)
    assert L.o_kept - L.idx == 768                       # 150 int32 indices, padded to 256 bytes
    assert L.gate - L.h2 == 150 * 512 * 2 and L.up - L.gate == 150 * 1408 * 2
    assert lay(blk, 200, 200) == 0 and L.o_kept == L.o   # nothing pruned: no gathered copy
    for bad in (dict(d=500), dict(H=3), dict(H=16), dict(F=1400), dict(qmax=8), dict(bits_attn_out=6),
                dict(rms_eps=-1.0), dict(H=0), dict(d=0)):
        assert lay(_fake_block(binding, **bad), 200, 150) == EINVAL, bad
    assert lay(blk, 0, 0) == EINVAL and lay(blk, 200, 0) == EINVAL and lay(blk, 200, 201) == EINVAL
    assert lay(blk, 8193, 100) == EINVAL and lay(blk, 8193, 8193) == 0 and lay(blk, 32768, 32768) == 0
    assert lay(blk, 32769, 32769) == EINVAL

    p, odd = ctypes.c_void_p(4096), ctypes.c_void_p(4100)
    ok = dict(blk=blk, x=p, pos=p, cos=p, sin=p, P=256, S=200, keep=150, out=p, pos_out=p, ws=p, wsb=1 << 40, st=None)

    def call(fn=lib.agq_block_forward, **kw):
        a = dict(ok, **kw)
        return fn(ctypes.byref(a["blk"]), a["x"], a["pos"], a["cos"], a["sin"], a["P"], a["S"], a["keep"], a["out"],
                  a["pos_out"], a["ws"], a["wsb"], a["st"])

    for name in ("x", "pos", "cos", "sin", "out", "ws"):
        assert call(**{name: None}) == EINVAL, name
    assert call(x=odd) == EINVAL and call(ws=ctypes.c_void_p(4096 + 16)) == EINVAL
    assert call(P=0) == EINVAL and call(S=0) == EINVAL and call(keep=201) == EINVAL
    assert call(wsb=1000) == ESIZE
    assert call(blk=_fake_block(binding, e_q=41)) == EINVAL
    assert call(blk=_fake_block(binding, w_down=None)) == EINVAL
    assert call(blk=_fake_block(binding, s_gate=4100)) == EINVAL
    assert call(fn=lib.agq_block_calibrate, wsb=1000) == ESIZE
    # TRIP sites: the count of extra chunks is checked, the workspace grows with it, calibration wants plain blobs
    assert call(blk=_fake_block(binding, trip_mlp_in=17)) == EINVAL and call(blk=_fake_block(binding, trip_attn_in=-2)) == EINVAL
    assert call(fn=lib.agq_block_calibrate, blk=_fake_block(binding, trip_attn_out=0)) == EINVAL
    L2 = binding.AgqBlockLayout()
    assert lib.agq_block_layout_of(ctypes.byref(_fake_block(binding, trip_mlp_act=3)), 200, 150, ctypes.byref(L2)) == 0
    assert lay(blk, 200, 150) == 0 and L2.total - L2.gemm_ws >= 256 * (1408 + 3 * 128) > 256 * 1408
    assert lib.agq_block_forward(None, p, p, p, p, 256, 200, 150, p, p, p, 1 << 40, None) == EINVAL


def test_stack_host_checks(lib):
    from paper_2312_05693_amd import binding
    n = 3
    arr = (binding.AgqBlock * n)(*[_fake_block(binding) for _ in range(n)])
    keep = lambda *v: ctypes.cast((ctypes.c_int64 * n)(*v), ctypes.c_void_p)
    size = lambda S, k: lib.agq_stack_workspace_bytes(ctypes.cast(arr, ctypes.c_void_p), n, S, k)
    L = binding.AgqBlockLayout()
    assert lib.agq_block_layout_of(ctypes.byref(arr[0]), 200, 200, ctypes.byref(L)) == 0
    full = size(200, keep(200, 200, 200))
    assert full == L.total + 2 * 200 * 512 * 2 + 2 * 1024          # two token buffers, two position buffers, one block
    # the largest block decides (not always the first: fewer tokens can mean more room for split-K partial tiles)
    totals = []
    for S_in, k in ((200, 200), (200, 150), (150, 100)):
        assert lib.agq_block_layout_of(ctypes.byref(arr[0]), S_in, k, ctypes.byref(L)) == 0
        totals.append(L.total)
    assert size(200, keep(200, 150, 100)) == max(totals) + 2 * 200 * 512 * 2 + 2 * 1024
    assert size(200, keep(150, 160, 100)) == 0 and size(200, keep(201, 100, 100)) == 0 and size(0, keep(1, 1, 1)) == 0
    p = ctypes.c_void_p(4096)
    call = lambda k, ws=p, wsb=1 << 40, x=p: lib.agq_stack_forward(ctypes.cast(arr, ctypes.c_void_p), n, k, x, p, p, p, 256,
                                                                  200, p, p, ws, wsb, None)
    assert call(keep(200, 150, 160)) == -1 and call(keep(200, 150, 100), wsb=1000) == -2
    assert call(keep(200, 150, 100), ws=None) == -1 and call(keep(200, 150, 100), x=None) == -1
    bad = (binding.AgqBlock * n)(_fake_block(binding), _fake_block(binding, e_k=99), _fake_block(binding))
    assert lib.agq_stack_forward(ctypes.cast(bad, ctypes.c_void_p), n, keep(200, 150, 100), p, p, p, p, 256, 200, p, p, p,
                                 1 << 40, None) == -1               # found before anything is launched


def test_cascade_keep_matches_the_oracle(lib, oracle):
    from oracle import agq_block_oracle
    from paper_2312_05693_amd import binding
    for S, beta, m in [(2048, 0.75, 2), (2048, 0.5, 1), (2048, 0.3, 4), (777, 0.6, 5), (4096, 0.1, 8), (5, 0.9, 3),
                       (0, 0.5, 2), (2048, 0.0, 3)]:
        assert binding.cascade_keep(S, beta, m) == agq_block_oracle.cascade_keep(S, beta, m)
    out = (ctypes.c_int64 * 4)()
    assert lib.agq_cascade_keep(100, 1.0, 2, ctypes.cast(out, ctypes.c_void_p)) == -1
    assert lib.agq_cascade_keep(100, -0.1, 2, ctypes.cast(out, ctypes.c_void_p)) == -1
    assert lib.agq_cascade_keep(100, 0.5, 0, ctypes.cast(out, ctypes.c_void_p)) == -1
    assert lib.agq_cascade_keep(100, float("nan"), 2, ctypes.cast(out, ctypes.c_void_p)) == -1
    assert lib.agq_cascade_keep(100, 0.5, 2, None) == -1


def test_chain_argument_errors_need_no_gpu(lib):
    """agq_gemm_chain_*: every argument error is found on the host (the stage array is host memory)."""
    from paper_2312_05693_amd.binding import AgqChainStage, AgqProj
    EINVAL, ESIZE = -1, -2
    p = 4096

    def chain(*stages):
        arr = (AgqChainStage * len(stages))()
        for i, (x, ldx, src, bits, e, K, projs) in enumerate(stages):
            arr[i].x_f16, arr[i].ldx, arr[i].src_proj, arr[i].bits, arr[i].e, arr[i].K, arr[i].count = x, ldx, src, bits, e, K, len(projs)
            for j, (N, ldy) in enumerate(projs):
                arr[i].projs[j] = AgqProj(p, p, N, p, ldy, None)
        return arr, len(stages)

    def size(arr_n, M=2):
        return lib.agq_gemm_chain_workspace_bytes(ctypes.cast(arr_n[0], ctypes.c_void_p), arr_n[1], M)

    def prep(arr_n, M=2, ws=256 * 4096, nbytes=1 << 40):
        return lib.agq_gemm_chain_prepare(ctypes.cast(arr_n[0], ctypes.c_void_p), arr_n[1], M, ws, nbytes, None)

    good = chain((p, 256, 0, 8, 0, 256, [(128, 128), (64, 64)]), (None, 0, 0, 8, -1, 128, [(32, 32)]))
    need = size(good)
    assert need > 0 and need % 8 == 0
    # the records: two parities x M rows x half the widest stage x 8 bytes, behind header, progress words and table
    assert size(good, 4) - size(good, 2) == 2 * 2 * (192 // 2) * 8
    assert prep(good, ws=None) == EINVAL and prep(good, ws=4100) == EINVAL        # workspace missing / misaligned
    assert prep(good, nbytes=need - 1) == ESIZE
    for M in (0, 5, -1):
        assert size(good, M) == 0 and prep(good, M) == EINVAL
    bad = [
        chain((None, 0, 0, 8, 0, 256, [(128, 128)])),                                  # first stage without input
        chain((p, 256, 0, 8, 0, 256, [(128, 128)]), (None, 0, 0, 8, 0, 256, [(32, 32)])),   # K != width of the source
        chain((p, 256, 0, 8, 0, 256, [(128, 128)]), (None, 0, 1, 8, 0, 128, [(32, 32)])),   # no such projection
        chain((p, 256, 0, 8, 0, 200, [(128, 128)])),                                   # K % 128
        chain((p, 256, 0, 8, 0, 16512, [(128, 128)])),                                 # K beyond the limit
        chain((p, 128, 0, 8, 0, 256, [(128, 128)])),                                   # ldx < K
        chain((p + 4, 256, 0, 8, 0, 256, [(128, 128)])),                               # misaligned input
        chain((p, 256, 0, 5, 0, 256, [(128, 128)])),                                   # bits
        chain((p, 256, 0, 8, 41, 256, [(128, 128)])),                                  # exponent
        chain((p, 256, 0, 8, 0, 256, [(120, 120)])),                                   # N % 16
        chain((p, 256, 0, 8, 0, 256, [(128, 64)])),                                    # ldy < N
        chain((p, 256, 0, 8, 0, 256, [])),                                             # no projection
    ]
    for c in bad:
        assert size(c) == 0 and prep(c) == EINVAL
    assert lib.agq_gemm_chain_run(None, None) == EINVAL and lib.agq_gemm_chain_run(4100, None) == EINVAL
    assert lib.agq_gemm_chain_status(None, None) == EINVAL
    assert lib.agq_status_string(-4) == b"a wait inside the kernel timed out"
