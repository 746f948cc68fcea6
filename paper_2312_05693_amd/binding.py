"""ctypes binding of libagq.so with the names of include/agq.h.

Argument marshalling only: every step of the path runs in the HIP kernels.
PyTorch is used for device memory and the current stream, nothing else.  There
is no CPU fallback: if the library has not been built, loading raises."""
from __future__ import annotations

import ctypes
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libagq.so")

AGQ_OK, AGQ_EINVAL, AGQ_ESIZE, AGQ_EHIP, AGQ_ETIMEOUT = 0, -1, -2, -3, -4
AGQ_X_F16, AGQ_X_Q, AGQ_X_F16_DOT = 0, 1, 2

_i64, _int, _vp, _sz = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t
_GEMM_ARGS = [_vp, _int, _i64, _i64, _i64, _int, _int, _vp, _vp, _i64, _vp, _i64, _vp, _vp, _sz, _vp]
_TRIP_GEMM_ARGS = [_vp, _i64, _i64, _i64, _int, _int, _vp, _int, _vp, _i64, _vp, _i64, _vp, _vp, _sz, _vp]
SIGNATURES = {
    "agq_status_string": (ctypes.c_char_p, [_int]),
    "agq_version": (_int, []),
    "agq_calibrate_act_exp": (_int, [_vp, _i64, _i64, _i64, _int, _vp, _vp]),
    "agq_quantize_act": (_int, [_vp, _i64, _i64, _i64, _int, _int, _int, _vp, _vp]),
    "agq_pack_w4_bytes": (_sz, [_i64, _i64]),
    "agq_pack_w4": (_int, [_vp, _i64, _i64, _vp, _vp, _vp]),
    "agq_unpack_w4": (_int, [_vp, _i64, _i64, _vp, _vp]),
    "agq_gemm_workspace_bytes": (_sz, [_i64, _i64, _i64]),
    "agq_gemm_w4a8": (_int, _GEMM_ARGS),
    "agq_gemm_w4a4": (_int, _GEMM_ARGS),
    "agq_gemm_w4a8_static": (_int, _GEMM_ARGS[:13] + [_vp]),
    "agq_gemm_w4a8_multi": (_int, [_vp, _int, _i64, _i64, _i64, _int, _int, _vp, _int, _vp, _sz, _vp]),
    "agq_gemm_w4a4_multi": (_int, [_vp, _int, _i64, _i64, _i64, _int, _int, _vp, _int, _vp, _sz, _vp]),
    "agq_gemm_chain_workspace_bytes": (_sz, [_vp, _int, _i64]),
    "agq_gemm_chain_prepare": (_int, [_vp, _int, _i64, _vp, _sz, _vp]),
    "agq_gemm_chain_run": (_int, [_vp, _vp]),
    "agq_gemm_chain_status": (_int, [_vp, _vp]),
    "agq_trip_search": (_int, [_vp, _i64, _i64, _i64, _int, _int, _int, _int, _vp, _vp]),
    "agq_trip_extra_chunks": (_int, [_vp, _i64]),
    "agq_pack_w4_trip_bytes": (_sz, [_i64, _i64, _int]),
    "agq_pack_w4_trip": (_int, [_vp, _i64, _i64, _vp, _vp, _vp, _vp]),
    "agq_unpack_w4_trip": (_int, [_vp, _i64, _i64, _int, _vp, _vp]),
    "agq_gemm_trip_workspace_bytes": (_sz, [_i64, _i64, _i64, _int]),
    "agq_gemm_w4a8_trip": (_int, _TRIP_GEMM_ARGS),
    "agq_gemm_w4a4_trip": (_int, _TRIP_GEMM_ARGS),
    "agq_gemm_w4a8_trip_multi": (_int, [_vp, _i64, _i64, _i64, _int, _int, _vp, _int, _int, _vp, _sz, _vp]),
    "agq_gemm_w4a4_trip_multi": (_int, [_vp, _i64, _i64, _i64, _int, _int, _vp, _int, _int, _vp, _sz, _vp]),
    "agq_log2_quant_softmax": (_int, [_vp, _i64, _i64, _i64, _int, _int, _vp, _int, _vp, _vp, _vp, _vp]),
    "agq_qk_log2_softmax": (_int, [_vp, _vp, _i64, _i64, _i64, _int, _int, _int, _int, _vp, _int, _vp, _vp, _vp, _vp]),
    "agq_prune_tokens": (_int, [_vp, _i64, _i64, _vp, _i64, _vp, _vp, _vp]),
    "agq_rmsnorm": (_int, [_vp, _vp, _vp, _vp, _i64, _i64, ctypes.c_double, _vp, _vp, _vp]),
    "agq_rope_quantize": (_int, [_vp, _vp, _vp, _i64, _i64, _i64, _vp, _vp, _vp, _i64, _int, _int, _int, _i64, _vp, _vp,
                                 _vp, _vp]),
    "agq_swiglu": (_int, [_vp, _vp, _vp, _i64, _vp]),
    "agq_residual_add": (_int, [_vp, _vp, _vp, _i64, _vp]),
    "agq_block_layout_of": (_int, [_vp, _i64, _i64, _vp]),
    "agq_block_forward": (_int, [_vp, _vp, _vp, _vp, _vp, _i64, _i64, _i64, _vp, _vp, _vp, _sz, _vp]),
    "agq_block_calibrate": (_int, [_vp, _vp, _vp, _vp, _vp, _i64, _i64, _i64, _vp, _vp, _vp, _sz, _vp]),
    "agq_cascade_keep": (_int, [_i64, ctypes.c_double, _int, _vp]),
    "agq_stack_workspace_bytes": (_sz, [_vp, _int, _i64, _vp]),
    "agq_stack_forward": (_int, [_vp, _int, _vp, _vp, _vp, _vp, _vp, _i64, _i64, _vp, _vp, _vp, _sz, _vp]),
}

AGQ_MAX_PROJ = 4


class AgqProj(ctypes.Structure):
    """struct agq_proj of include/agq.h"""
    _fields_ = [("w_packed", _vp), ("w_scale_f16", _vp), ("N", _i64), ("y_f16", _vp), ("ldy", _i64),
                ("acc_out", _vp)]


AGQ_CHAIN_MAX_M = 4


class AgqChainStage(ctypes.Structure):
    """struct agq_chain_stage of include/agq.h"""
    _fields_ = [("x_f16", _vp), ("ldx", _i64), ("src_proj", _int), ("bits", _int), ("e", _int), ("K", _i64),
                ("count", _int), ("projs", AgqProj * AGQ_MAX_PROJ)]


BLOCK_PROJ = ("q", "k", "v", "o", "gate", "up", "down")
BLOCK_EXPS = ("e_attn_in", "e_q", "e_k", "e_v", "e_attn_out", "e_mlp_in", "e_mlp_act")
BLOCK_SITES = ("attn_in", "attn_out", "mlp_in", "mlp_act")
BLOCK_TENSORS = ("h1", "q", "k", "v", "q_q", "k_q", "v_q", "o", "score", "idx", "o_kept", "attn_out", "x1", "h2",
                 "gate", "up", "act", "down", "q_rot", "k_rot")


class AgqBlock(ctypes.Structure):
    """struct agq_block of include/agq.h"""
    _fields_ = ([("d", _i64), ("H", _i64), ("F", _i64), ("qmax", _int), ("bits_attn_out", _int),
                 ("rms_eps", ctypes.c_double), ("g_attn_f16", _vp), ("g_mlp_f16", _vp)]
                + [("w_" + n, _vp) for n in BLOCK_PROJ] + [("s_" + n, _vp) for n in BLOCK_PROJ]
                + [(n, _int) for n in BLOCK_EXPS] + [("trip_" + n, _int) for n in BLOCK_SITES])


class AgqBlockLayout(ctypes.Structure):
    """struct agq_block_layout of include/agq.h"""
    _fields_ = [("S_pad", _i64)] + [(n, _sz) for n in BLOCK_TENSORS] + [("gemm_ws", _sz), ("total", _sz)]


_lib = None


class AgqError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: %s (%d)" % (where, lib().agq_status_string(status).decode(), status))


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libagq.so is missing: run paper_2312_05693_amd/build.py (no CPU fallback exists)")
        handle = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(handle, name)
            fn.restype, fn.argtypes = res, args
        _lib = handle
    return _lib


def _ptr(t):
    return None if t is None else t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _ok(status: int, where: str):
    if status != AGQ_OK:
        raise AgqError(status, where)


def version() -> int:
    return lib().agq_version()


def calibrate_act_exp(x: torch.Tensor, bits: int, e_dev: torch.Tensor | None = None) -> torch.Tensor:
    """Device int32 tensor holding e (read it with .item() after the call)."""
    M, K = x.shape
    if e_dev is None:
        e_dev = torch.empty(1, dtype=torch.int32, device=x.device)
    _ok(lib().agq_calibrate_act_exp(_ptr(x), M, K, x.stride(0), bits, _ptr(e_dev), _stream()), "agq_calibrate_act_exp")
    return e_dev


def quantize_act(x: torch.Tensor, bits: int, e: int, zp: int = 0, out: torch.Tensor | None = None) -> torch.Tensor:
    M, K = x.shape
    if out is None:
        cols = K if bits == 8 else K // 2
        out = torch.empty((M, cols), dtype=torch.uint8 if (zp or bits == 4) else torch.int8, device=x.device)
    _ok(lib().agq_quantize_act(_ptr(x), M, K, x.stride(0), bits, e, zp, _ptr(out), _stream()), "agq_quantize_act")
    return out


def pack_w4_bytes(N: int, K: int) -> int:
    return lib().agq_pack_w4_bytes(N, K)


def pack_w4(wq: torch.Tensor, packed: torch.Tensor | None = None, bad_count: torch.Tensor | None = None):
    N, K = wq.shape
    if packed is None:
        packed = torch.empty(pack_w4_bytes(N, K), dtype=torch.uint8, device=wq.device)
    _ok(lib().agq_pack_w4(_ptr(wq), N, K, _ptr(packed), _ptr(bad_count), _stream()), "agq_pack_w4")
    return packed


def unpack_w4(packed: torch.Tensor, N: int, K: int) -> torch.Tensor:
    out = torch.empty((N, K), dtype=torch.int8, device=packed.device)
    _ok(lib().agq_unpack_w4(_ptr(packed), N, K, _ptr(out), _stream()), "agq_unpack_w4")
    return out


def gemm_workspace_bytes(M: int, N: int, K: int) -> int:
    return lib().agq_gemm_workspace_bytes(M, N, K)


def _gemm(fn_name, x, x_kind, M, K, ldx, e, zp, w_packed, w_scale, N, y, acc_out, workspace):
    if y is None:
        y = torch.empty((M, N), dtype=torch.float16, device=w_packed.device)
    need = gemm_workspace_bytes(M, N, K)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=w_packed.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    fn = getattr(lib(), fn_name)
    _ok(fn(_ptr(x), x_kind, M, K, ldx, e, zp, _ptr(w_packed), _ptr(w_scale), N, _ptr(y), y.stride(0) if M else N,
           _ptr(acc_out), _ptr(workspace), ws_bytes, _stream()), fn_name)
    return y


def gemm_w4a8(x, e, w_packed, w_scale, N, K, x_kind=AGQ_X_F16, y=None, acc_out=None, workspace=None, zp=0):
    """x: fp16 [M,K] (AGQ_X_F16) or int8 codes [M,K] (AGQ_X_Q)."""
    M = x.shape[0]
    return _gemm("agq_gemm_w4a8", x, x_kind, M, K, x.stride(0) if M else K, e, zp, w_packed, w_scale, N, y, acc_out,
                 workspace)


def gemm_w4a8_static(x, e, w_packed, w_scale, N, K, y, x_kind=AGQ_X_F16, acc_out=None, zp=0):
    """agq_gemm_w4a8 on the library's fixed workspace; y (and acc_out) are the caller's: nothing is allocated."""
    M = x.shape[0]
    _ok(lib().agq_gemm_w4a8_static(_ptr(x), x_kind, M, K, x.stride(0) if M else K, e, zp, _ptr(w_packed), _ptr(w_scale),
                                   N, _ptr(y), y.stride(0) if M else N, _ptr(acc_out), _stream()), "agq_gemm_w4a8_static")
    return y


def gemm_w4a4(x, e, w_packed, w_scale, N, K, x_kind=AGQ_X_F16, y=None, acc_out=None, workspace=None, zp=0):
    """x: fp16 [M,K] (AGQ_X_F16) or nibble codes [M,K/2] bytes (AGQ_X_Q)."""
    M = x.shape[0]
    ldx = (x.stride(0) if M else K) * (2 if x_kind == AGQ_X_Q else 1)
    return _gemm("agq_gemm_w4a4", x, x_kind, M, K, ldx, e, zp, w_packed, w_scale, N, y, acc_out, workspace)


def _gemm_multi(fn_name, x, x_kind, M, K, ldx, e, zp, projs, workspace):
    """projs: list of (w_packed, w_scale, N, y or None, acc_out or None); returns the list of y."""
    dev = projs[0][0].device
    ys, arr = [], (AgqProj * len(projs))()
    for i, (packed, scale, N, y, acc) in enumerate(projs):
        if y is None:
            y = torch.empty((M, N), dtype=torch.float16, device=dev)
        ys.append(y)
        arr[i] = AgqProj(_ptr(packed), _ptr(scale), N, _ptr(y), y.stride(0) if M else N, _ptr(acc))
    need = gemm_workspace_bytes(M, sum(p[2] for p in projs), K)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    fn = getattr(lib(), fn_name)
    _ok(fn(_ptr(x), x_kind, M, K, ldx, e, zp, ctypes.cast(arr, _vp), len(projs), _ptr(workspace), ws_bytes,
           _stream()), fn_name)
    return ys


def gemm_w4a8_multi(x, e, projs, K, x_kind=AGQ_X_F16, workspace=None, zp=0):
    """Several projections of one activation: projs = [(w_packed, w_scale, N, y|None, acc_out|None), ...]."""
    M = x.shape[0]
    return _gemm_multi("agq_gemm_w4a8_multi", x, x_kind, M, K, x.stride(0) if M else K, e, zp, projs, workspace)


def gemm_w4a4_multi(x, e, projs, K, x_kind=AGQ_X_F16, workspace=None, zp=0):
    M = x.shape[0]
    ldx = (x.stride(0) if M else K) * (2 if x_kind == AGQ_X_Q else 1)
    return _gemm_multi("agq_gemm_w4a4_multi", x, x_kind, M, K, ldx, e, zp, projs, workspace)


class ChainPlan:
    """A prepared chain: the stage array, its workspace, and the tensors the baked pointers refer to."""

    def __init__(self, arr, n, M, workspace, keepalive, ys):
        self.arr, self.n, self.M, self.workspace, self.keepalive, self.ys = arr, n, M, workspace, keepalive, ys


def gemm_chain_stages(stages, M):
    """stages: list of dicts with x (fp16 [M,K] tensor, or None: the output of projection `src_proj` of the stage
    before), bits, e, K and projs = [(w_packed, w_scale, N, y|None, acc_out|None), ...].  Returns the ctypes array,
    the per-stage lists of outputs and everything that must stay alive."""
    arr = (AgqChainStage * len(stages))()
    keep, ys = [], []
    for i, st in enumerate(stages):
        x = st.get("x")
        c = arr[i]
        c.x_f16, c.ldx = _ptr(x), (x.stride(0) if x is not None else 0)
        c.src_proj, c.bits, c.e, c.K, c.count = int(st.get("src_proj", 0)), int(st["bits"]), int(st["e"]), int(st["K"]), len(st["projs"])
        outs = []
        for p, (packed, scale, N, y, acc) in enumerate(st["projs"]):
            if y is None:
                y = torch.zeros((M, N), dtype=torch.float16, device=packed.device)
            outs.append(y)
            c.projs[p] = AgqProj(_ptr(packed), _ptr(scale), N, _ptr(y), y.stride(0), _ptr(acc))
            keep += [packed, scale, y, acc]
        keep.append(x)
        ys.append(outs)
    return arr, ys, keep


def gemm_chain_prepare(stages, M, workspace=None) -> ChainPlan:
    """agq_gemm_chain_prepare: checks the chain, writes its table into a workspace (allocated here unless given) and
    waits for the current stream."""
    arr, ys, keep = gemm_chain_stages(stages, M)
    n = len(stages)
    need = lib().agq_gemm_chain_workspace_bytes(ctypes.cast(arr, _vp), n, M)
    if need == 0:
        raise AgqError(AGQ_EINVAL, "agq_gemm_chain_workspace_bytes")
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=keep[0].device)
    _ok(lib().agq_gemm_chain_prepare(ctypes.cast(arr, _vp), n, M, _ptr(workspace), workspace.numel(), _stream()),
        "agq_gemm_chain_prepare")
    return ChainPlan(arr, n, M, workspace, keep, ys)


def gemm_chain_run(plan: ChainPlan):
    """agq_gemm_chain_run: one kernel launch on the current stream; returns the per-stage lists of outputs."""
    _ok(lib().agq_gemm_chain_run(_ptr(plan.workspace), _stream()), "agq_gemm_chain_run")
    return plan.ys


def gemm_chain_status(plan: ChainPlan) -> int:
    """agq_gemm_chain_status: waits for the current stream; AGQ_OK or AGQ_ETIMEOUT."""
    return lib().agq_gemm_chain_status(_ptr(plan.workspace), _stream())


def trip_search(x: torch.Tensor, bits: int, e: int, kmax: int, zp: int = 0, alpha: torch.Tensor | None = None):
    """Eq.8: device int8 [K] of per-channel factors."""
    M, K = x.shape
    if alpha is None:
        alpha = torch.empty(K, dtype=torch.int8, device=x.device)
    _ok(lib().agq_trip_search(_ptr(x), M, K, x.stride(0) if M else K, bits, e, zp, kmax, _ptr(alpha), _stream()),
        "agq_trip_search")
    return alpha


def _host_alpha(alpha):
    """The factors as a contiguous host int8 array (kept alive by the caller for the call)."""
    import numpy as np
    if isinstance(alpha, torch.Tensor):
        alpha = alpha.cpu().numpy()
    return np.ascontiguousarray(alpha, dtype=np.int8)


def trip_extra_chunks(alpha, K: int) -> int:
    a = _host_alpha(alpha)
    n = lib().agq_trip_extra_chunks(a.ctypes.data, K)
    if n < 0:
        raise AgqError(n, "agq_trip_extra_chunks")
    return n


def pack_w4_trip(wq: torch.Tensor, alpha, packed: torch.Tensor | None = None, bad_count: torch.Tensor | None = None):
    """Returns (blob, n_extra)."""
    N, K = wq.shape
    a = _host_alpha(alpha)
    n_extra = trip_extra_chunks(a, K)
    if packed is None:
        packed = torch.empty(lib().agq_pack_w4_trip_bytes(N, K, n_extra), dtype=torch.uint8, device=wq.device)
    _ok(lib().agq_pack_w4_trip(_ptr(wq), N, K, a.ctypes.data, _ptr(packed), _ptr(bad_count), _stream()),
        "agq_pack_w4_trip")
    return packed, n_extra


def unpack_w4_trip(packed: torch.Tensor, N: int, K: int, n_extra: int) -> torch.Tensor:
    out = torch.zeros((N, K), dtype=torch.int8, device=packed.device)
    _ok(lib().agq_unpack_w4_trip(_ptr(packed), N, K, n_extra, _ptr(out), _stream()), "agq_unpack_w4_trip")
    return out


def gemm_trip(x, bits, e, w_packed, n_extra, w_scale, N, K, y=None, acc_out=None, workspace=None, zp=0):
    """The TRIP linear layer (Section 4.4) with b = bits; x is fp16 [M, K]."""
    M = x.shape[0]
    if y is None:
        y = torch.empty((M, N), dtype=torch.float16, device=x.device)
    need = lib().agq_gemm_trip_workspace_bytes(M, N, K, n_extra)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    fn = lib().agq_gemm_w4a8_trip if bits == 8 else lib().agq_gemm_w4a4_trip
    _ok(fn(_ptr(x), M, K, x.stride(0) if M else K, e, zp, _ptr(w_packed), n_extra, _ptr(w_scale), N, _ptr(y),
           y.stride(0) if M else N, _ptr(acc_out), _ptr(workspace), workspace.numel() if workspace is not None else 0,
           _stream()), "agq_gemm_w4a%d_trip" % bits)
    return y


def gemm_trip_multi(x, bits, e, projs, n_extra, K, workspace=None, zp=0):
    """The TRIP layer for several projections of one activation: projs = [(blob, w_scale, N, y|None, acc_out|None), ...],
    every blob packed with the same factors.  Returns the list of y."""
    M = x.shape[0]
    ys, arr = [], (AgqProj * len(projs))()
    for i, (packed, scale, N, y, acc) in enumerate(projs):
        if y is None:
            y = torch.empty((M, N), dtype=torch.float16, device=x.device)
        ys.append(y)
        arr[i] = AgqProj(_ptr(packed), _ptr(scale), N, _ptr(y), y.stride(0) if M else N, _ptr(acc))
    need = lib().agq_gemm_trip_workspace_bytes(M, sum(p[2] for p in projs), K, n_extra)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    fn = lib().agq_gemm_w4a8_trip_multi if bits == 8 else lib().agq_gemm_w4a4_trip_multi
    _ok(fn(_ptr(x), M, K, x.stride(0) if M else K, e, zp, ctypes.cast(arr, _vp), len(projs), n_extra, _ptr(workspace),
           workspace.numel() if workspace is not None else 0, _stream()), "agq_gemm_w4a%d_trip_multi" % bits)
    return ys


def log2_quant_softmax(p, v_q, e_v, qmax=15, causal=True, want_codes=False, want_score=True):
    """p fp16 [H,S,S], v_q int8 [H,S,D] -> (o fp16 [S,H*D], codes or None, score or None)."""
    H, S, _ = p.shape
    D = v_q.shape[2]
    o = torch.empty((S, H * D), dtype=torch.float16, device=p.device)
    codes = torch.empty((H, S, S // 2), dtype=torch.uint8, device=p.device) if want_codes else None
    score = torch.empty(S, dtype=torch.int32, device=p.device) if want_score else None
    _ok(lib().agq_log2_quant_softmax(_ptr(p), H, S, D, int(causal), qmax, _ptr(v_q), e_v, _ptr(o), _ptr(codes),
                                     _ptr(score), _stream()), "agq_log2_quant_softmax")
    return o, codes, score


def qk_log2_softmax(qq, kq, vq, e_q, e_k, e_v, qmax=15, causal=True, want_codes=False, want_score=True):
    """Attention from quantized Q, K, V (int8 [H,S,D]).  Returns (o, codes or None, score or None);
    the score buffer is zeroed here because the call accumulates into it."""
    H, S, D = qq.shape
    o = torch.empty((S, H * D), dtype=torch.float16, device=qq.device)
    codes = torch.empty((H, S, S // 2), dtype=torch.uint8, device=qq.device) if want_codes else None
    score = torch.zeros(S, dtype=torch.int32, device=qq.device) if want_score else None
    _ok(lib().agq_qk_log2_softmax(_ptr(qq), _ptr(kq), H, S, D, int(causal), qmax, e_q, e_k, _ptr(vq), e_v, _ptr(o),
                                  _ptr(codes), _ptr(score), _stream()), "agq_qk_log2_softmax")
    return o, codes, score


def prune_tokens(score, n_keep, x):
    S, d = x.shape
    idx = torch.empty(n_keep, dtype=torch.int32, device=x.device)
    out = torch.empty((n_keep, d), dtype=torch.float16, device=x.device)
    _ok(lib().agq_prune_tokens(_ptr(score), S, n_keep, _ptr(x), d, _ptr(idx), _ptr(out), _stream()), "agq_prune_tokens")
    return idx, out


def rmsnorm(x, g, eps, res=None, idx=None):
    """y = RMSNorm(x; g), or with res: (t, y) with t = res[idx] + x and y = RMSNorm(t; g)."""
    rows, d = x.shape
    y = torch.empty_like(x)
    t = torch.empty_like(x) if res is not None else None
    _ok(lib().agq_rmsnorm(_ptr(x), _ptr(res), _ptr(idx), _ptr(g), rows, d, eps, _ptr(t), _ptr(y), _stream()),
        "agq_rmsnorm")
    return y if res is None else (t, y)


def rope_quantize(q, k, v, H, pos, rope_cos, rope_sin, e_q, e_k, e_v, S_pad=None):
    """fp16 [S, H*D] each -> int8 [H, S_pad, D] each (q and k rotated, all three on Eq.2's grid)."""
    S, d = q.shape
    D = d // H
    S_pad = -(-S // 128) * 128 if S_pad is None else S_pad
    outs = [torch.empty((H, S_pad, D), dtype=torch.int8, device=q.device) for _ in range(3)]
    _ok(lib().agq_rope_quantize(_ptr(q), _ptr(k), _ptr(v), S, H, D, _ptr(pos), _ptr(rope_cos), _ptr(rope_sin),
                                rope_cos.shape[0], e_q, e_k, e_v, S_pad, _ptr(outs[0]), _ptr(outs[1]), _ptr(outs[2]),
                                _stream()), "agq_rope_quantize")
    return outs


def swiglu(gate, up):
    out = torch.empty_like(gate)
    _ok(lib().agq_swiglu(_ptr(gate), _ptr(up), _ptr(out), gate.numel(), _stream()), "agq_swiglu")
    return out


def residual_add(a, b):
    out = torch.empty_like(a)
    _ok(lib().agq_residual_add(_ptr(a), _ptr(b), _ptr(out), a.numel(), _stream()), "agq_residual_add")
    return out


def make_block(d, H, F, weights: dict, qmax=15, bits_attn_out=4, rms_eps=1e-5, exps: dict | None = None,
               trip: dict | None = None) -> AgqBlock:
    """weights: device tensors g_attn, g_mlp (fp16 [d]) and, for every projection in BLOCK_PROJ, the agq_pack_w4
    blob `w_<name>` and the fp16 scales `s_<name>`.  trip: for the sites of BLOCK_SITES whose projections are
    agq_pack_w4_trip blobs, the number of extra chunks of their factors.  The struct keeps the tensors alive."""
    blk = AgqBlock(d=d, H=H, F=F, qmax=qmax, bits_attn_out=bits_attn_out, rms_eps=rms_eps,
                   g_attn_f16=_ptr(weights["g_attn"]), g_mlp_f16=_ptr(weights["g_mlp"]))
    for n in BLOCK_PROJ:
        setattr(blk, "w_" + n, _ptr(weights["w_" + n]))
        setattr(blk, "s_" + n, _ptr(weights["s_" + n]))
    for n in BLOCK_EXPS:
        setattr(blk, n, 0 if exps is None else int(exps[n]))
    for n in BLOCK_SITES:
        setattr(blk, "trip_" + n, -1 if trip is None or trip.get(n) is None else int(trip[n]))
    blk._keepalive = dict(weights)
    return blk


def block_exps(blk: AgqBlock) -> dict:
    return {n: int(getattr(blk, n)) for n in BLOCK_EXPS}


def block_layout(blk: AgqBlock, S: int, n_keep: int) -> AgqBlockLayout:
    L = AgqBlockLayout()
    _ok(lib().agq_block_layout_of(ctypes.byref(blk), S, n_keep, ctypes.byref(L)), "agq_block_layout_of")
    return L


def block_forward(blk: AgqBlock, x, pos, rope_cos, rope_sin, n_keep=None, workspace=None, calibrate=False, out=None):
    """One block (Section 4.2's pipeline with pruning after attention).  x fp16 [S,d], pos int32 [S], rope tables
    float32 [P, D/2].  calibrate=True derives the exponents from this input and stores them in blk.
    out: optional (x_out, pos_out) to write into.  Returns (x_out [n_keep,d], pos_out [n_keep], workspace, layout)."""
    S, d = x.shape
    n_keep = S if n_keep is None else n_keep
    L = block_layout(blk, S, n_keep)
    if workspace is None:
        workspace = torch.empty(L.total, dtype=torch.uint8, device=x.device)
    if out is None:
        out = (torch.empty((n_keep, d), dtype=torch.float16, device=x.device),
               torch.empty(n_keep, dtype=torch.int32, device=x.device))
    x_out, pos_out = out
    fn = lib().agq_block_calibrate if calibrate else lib().agq_block_forward
    _ok(fn(ctypes.byref(blk), _ptr(x), _ptr(pos), _ptr(rope_cos), _ptr(rope_sin), rope_cos.shape[0], S, n_keep,
           _ptr(x_out), _ptr(pos_out), _ptr(workspace), workspace.numel(), _stream()),
        "agq_block_calibrate" if calibrate else "agq_block_forward")
    return x_out, pos_out, workspace, L


def block_tensor(blk: AgqBlock, L: AgqBlockLayout, workspace, name: str, S: int, n_keep: int):
    """View of one intermediate tensor of the last call inside its workspace."""
    d, H, F, sp = blk.d, blk.H, blk.F, L.S_pad
    shapes = dict(h1=(S, d), q=(S, d), k=(S, d), v=(S, d), q_rot=(S, d), k_rot=(S, d), o=(sp, d),
                  o_kept=(n_keep, d), attn_out=(n_keep, d), x1=(n_keep, d), h2=(n_keep, d), down=(n_keep, d),
                  gate=(n_keep, F), up=(n_keep, F), act=(n_keep, F))
    off = getattr(L, name)
    if name in ("q_q", "k_q", "v_q"):
        return workspace[off:off + sp * d].view(torch.int8).view(H, sp, d // H)
    if name in ("score", "idx"):
        n = sp if name == "score" else n_keep
        return workspace[off:off + 4 * n].view(torch.int32)
    r, c = shapes[name]
    return workspace[off:off + 2 * r * c].view(torch.float16).view(r, c)


def stack_forward(blocks, keep, x, pos, rope_cos, rope_sin, workspace=None, out=None):
    """A stack of blocks with cascade pruning: block l keeps keep[l] of the tokens it receives.
    Returns (x_out [keep[-1], d], pos_out, workspace)."""
    n = len(blocks)
    arr = (AgqBlock * n)(*blocks)
    kp = (ctypes.c_int64 * n)(*[int(k) for k in keep])
    S, d = x.shape
    need = lib().agq_stack_workspace_bytes(ctypes.cast(arr, _vp), n, S, ctypes.cast(kp, _vp))
    if need == 0:
        raise AgqError(AGQ_EINVAL, "agq_stack_workspace_bytes")
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    if out is None:
        out = (torch.empty((int(keep[-1]), d), dtype=torch.float16, device=x.device),
               torch.empty(int(keep[-1]), dtype=torch.int32, device=x.device))
    _ok(lib().agq_stack_forward(ctypes.cast(arr, _vp), n, ctypes.cast(kp, _vp), _ptr(x), _ptr(pos), _ptr(rope_cos),
                                _ptr(rope_sin), rope_cos.shape[0], S, _ptr(out[0]), _ptr(out[1]), _ptr(workspace),
                                workspace.numel(), _stream()), "agq_stack_forward")
    return out[0], out[1], workspace


def cascade_keep(S: int, beta: float, m: int) -> list:
    out = (ctypes.c_int64 * m)()
    _ok(lib().agq_cascade_keep(S, beta, m, ctypes.cast(out, _vp)), "agq_cascade_keep")
    return list(out)
