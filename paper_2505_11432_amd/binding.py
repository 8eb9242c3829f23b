"""ctypes binding of libmoe_hip.so: same names as the C ABI (include/moe.h), argument marshalling only.

Every function takes torch tensors that already live on the GPU (torch is used for device memory
and streams, nothing else), passes their device pointers and the current stream to the library and
raises MoEError on a non-zero status.  There is no CPU fallback: if the library is missing the
import of this module fails.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import c_char_p, c_int, c_size_t, c_void_p

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmoe_hip.so")

F32, BF16, F8E4M3 = 0, 1, 2
Q_ROW, Q_COLGROUP128 = 0, 1
MAX_EXPERTS, MAX_TOPK = 256, 16

EXPORTS = (
    "moe_abi_version", "moe_last_hip_error", "moe_status_string", "moe_workspace_bytes",
    "moe_router_fwd", "moe_router_bwd", "moe_route", "moe_route_bwd", "moe_dispatch", "moe_combine",
    "moe_gate_grad", "moe_expert_ffn_fwd", "moe_expert_ffn_bwd", "moe_quant_fp8", "moe_dequant_fp8",
    "moe_expert_ffn_bwd_fp8", "moe_tgroup_tokens", "moe_quant_fp8_tgroup", "moe_route_range",
    "moe_route_capacity_workspace_bytes", "moe_route_capacity", "moe_balance_loss", "moe_balance_loss_bwd",
    "moe_row_map", "moe_expert_ffn_fused_workspace_bytes", "moe_expert_ffn_fused_fwd", "moe_expert_ffn_fused_bwd",
    "moe_route_noalloc", "moe_init", "moe_transpose",
)


class FfnBwdFp8Args(ctypes.Structure):
    """Mirror of moe_ffn_bwd_fp8_args (include/moe.h), field for field."""
    _fields_ = (
        [(n, c_void_p) for n in ("d_yp", "h_save", "xp_deq", "a_deq", "offsets", "w1t", "w1t_scale", "w2t", "w2t_scale")]
        + [(n, c_int) for n in ("M", "d", "E", "f")]
        + [(n, c_void_p) for n in ("d_xp", "d_w1", "d_w2")]
        + [("grad_dt", c_int), ("accumulate", c_int)]
        + [(n, c_void_p) for n in ("dy_codes", "dy_scale", "dh", "dh_codes", "dh_scale", "pad_offsets")]
        + [("ldt", ctypes.c_long)]
        + [(n, c_void_p) for n in ("dy_t", "dy_e8m0", "dh_t", "dh_e8m0", "a_t", "a_e8m0", "x_t", "x_e8m0", "splitk_ws")]
        + [(n, c_void_p) for n in ("xp_codes", "xp_scale", "a_codes", "a_scale")]
    )


SPLITK_WS_BYTES = 256 * 256 * 256 * 4


class MoEError(RuntimeError):
    def __init__(self, fn: str, status: int):
        msg = _lib.moe_status_string(status).decode()
        extra = f" (hipError {_lib.moe_last_hip_error()})" if status == -4 else ""
        super().__init__(f"{fn} failed: {status} {msg}{extra}")
        self.status = status


def _load() -> ctypes.CDLL:
    from . import build as _build
    if not _build.is_current():
        # missing, or built from other sources than the ones in the tree: never load a stale library
        import sys
        sys.stderr.write(f"{LIB_PATH} is missing or older than its sources: building it\n")
        _build.build(verbose=False)
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built; run `python -m paper_2505_11432_amd.build` "
                          "(there is no fallback path)")
    lib = ctypes.CDLL(LIB_PATH)
    P, I, Z = c_void_p, c_int, c_size_t
    sig = {
        "moe_abi_version": (I, []),
        "moe_init": (I, []),
        "moe_last_hip_error": (I, []),
        "moe_status_string": (c_char_p, [I]),
        "moe_workspace_bytes": (Z, [I, I, I, I, I, I]),
        "moe_router_fwd": (I, [P, P, P, I, I, I, I, P, P]),
        "moe_router_bwd": (I, [P, P, P, I, I, I, I, P, P, P, Z, P]),
        "moe_route": (I, [P, I, I, I, I, P, P, P, P, P, P, P, Z, P]),
        "moe_route_noalloc": (I, [P, I, I, I, I, P, P, P, P, P, P, P]),
        "moe_route_range": (I, [P, I, I, I, I, I, I, P, P, P, P, P, P, P, Z, P]),
        "moe_route_capacity_workspace_bytes": (Z, [I, I, I]),
        "moe_route_capacity": (I, [P, I, I, I, I, I, I, P, P, P, P, P, P, P, P, Z, P]),
        "moe_balance_loss": (I, [P, P, I, I, I, I, ctypes.c_float, P, P, P, P, Z, P]),
        "moe_balance_loss_bwd": (I, [P, P, I, I, I, ctypes.c_float, P, P]),
        "moe_route_bwd": (I, [P, P, P, P, I, I, I, I, P, P]),
        "moe_dispatch": (I, [P, P, I, P, P, I, I, I, P, P, P]),
        "moe_combine": (I, [P, P, I, P, P, I, I, I, P, I, P]),
        "moe_gate_grad": (I, [P, I, P, P, I, P, I, I, I, P, P]),
        "moe_expert_ffn_fwd": (I, [P, P, I, P, P, P, P, P, I, I, I, I, I, P, P, P, I, P, P, P, Z, P]),
        "moe_expert_ffn_bwd": (I, [P, P, P, P, P, P, P, I, I, I, I, I, P, P, P, I, I, P, Z, P]),
        "moe_quant_fp8": (I, [P, I, I, I, I, P, P, P]),
        "moe_dequant_fp8": (I, [P, P, I, I, I, P, I, P]),
        "moe_expert_ffn_bwd_fp8": (I, [ctypes.POINTER(FfnBwdFp8Args), P]),
        "moe_tgroup_tokens": (Z, [I, I]),
        "moe_transpose": (I, [P, I, I, I, I, P, P]),
        "moe_row_map": (I, [P, P, P, I, I, I, P, P, P]),
        "moe_expert_ffn_fused_workspace_bytes": (Z, [I, I, I, I]),
        "moe_expert_ffn_fused_fwd": (I, [P, P, P, P, P, P, I, I, I, I, I, P, P, P, Z, P]),
        "moe_expert_ffn_fused_bwd": (I, [P, P, P, P, P, P, P, P, P, I, I, I, I, I, P, P, P, I, I, P, P, Z, P]),
        "moe_quant_fp8_tgroup": (I, [P, I, I, I, P, I, P, P, ctypes.c_long, P, P]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    return lib


_lib = _load()


def dtype_code(t: torch.dtype) -> int:
    if t == torch.float32:
        return F32
    if t == torch.bfloat16:
        return BF16
    if t in (torch.uint8, torch.float8_e4m3fn):
        return F8E4M3
    raise TypeError(f"unsupported dtype {t}")


def _p(t):
    """Device pointer of a tensor (None -> NULL)."""
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "tensors must be contiguous and on the GPU"
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _check(fn: str, status: int):
    if status != 0:
        raise MoEError(fn, status)


def moe_abi_version() -> int:
    return _lib.moe_abi_version()


def moe_init():
    _check("moe_init", _lib.moe_init())


def moe_workspace_bytes(T, d, E, k, f, act) -> int:
    return _lib.moe_workspace_bytes(T, d, E, k, f, act)


def moe_router_fwd(x, w_r, bias, logits):
    T, d = x.shape
    E = w_r.shape[0]
    _check("moe_router_fwd", _lib.moe_router_fwd(_p(x), _p(w_r), _p(bias), dtype_code(x.dtype), T, d, E,
                                                 _p(logits), _stream()))


def moe_router_bwd(x, w_r, d_logits, d_w_r, dx, workspace):
    T, d = x.shape
    E = w_r.shape[0]
    _check("moe_router_bwd", _lib.moe_router_bwd(_p(x), _p(w_r), _p(d_logits), dtype_code(x.dtype), T, d, E,
                                                 _p(d_w_r), _p(dx), _p(workspace),
                                                 workspace.numel() * workspace.element_size(), _stream()))


def moe_route(logits, k, renorm, topk_idx, topk_w, counts, offsets, perm, inv_perm, workspace):
    T, E = logits.shape
    _check("moe_route", _lib.moe_route(_p(logits), T, E, k, renorm, _p(topk_idx), _p(topk_w), _p(counts),
                                       _p(offsets), _p(perm), _p(inv_perm), _p(workspace),
                                       workspace.numel() * workspace.element_size(), _stream()))


def moe_route_noalloc(logits, k, renorm, topk_idx, topk_w, counts, offsets, perm, inv_perm):
    T, E = logits.shape
    _check("moe_route_noalloc", _lib.moe_route_noalloc(_p(logits), T, E, k, renorm, _p(topk_idx), _p(topk_w), _p(counts),
                                                       _p(offsets), _p(perm), _p(inv_perm), _stream()))


def moe_route_bwd(logits, topk_idx, topk_w, d_topk_w, E, renorm, d_logits):
    T, k = topk_idx.shape
    _check("moe_route_bwd", _lib.moe_route_bwd(_p(logits), _p(topk_idx), _p(topk_w), _p(d_topk_w), T, E, k,
                                               renorm, _p(d_logits), _stream()))


def moe_dispatch(x, x_scale, inv_perm, row_mul, k, xp, xp_scale):
    T, d = x.shape
    _check("moe_dispatch", _lib.moe_dispatch(_p(x), _p(x_scale), dtype_code(x.dtype), _p(inv_perm), _p(row_mul),
                                             T, k, d, _p(xp), _p(xp_scale), _stream()))


def moe_combine(yp, yp_scale, inv_perm, topk_w, k, y):
    T, d = y.shape
    _check("moe_combine", _lib.moe_combine(_p(yp), _p(yp_scale), dtype_code(yp.dtype), _p(inv_perm), _p(topk_w),
                                           T, k, d, _p(y), dtype_code(y.dtype), _stream()))


def moe_gate_grad(dy, yp, yp_scale, inv_perm, k, d_topk_w):
    T, d = dy.shape
    _check("moe_gate_grad", _lib.moe_gate_grad(_p(dy), dtype_code(dy.dtype), _p(yp), _p(yp_scale),
                                               dtype_code(yp.dtype), _p(inv_perm), T, k, d, _p(d_topk_w),
                                               _stream()))


def moe_expert_ffn_fwd(xp, xp_scale, offsets, w1, w1_scale, w2, w2_scale, h_save, yp, yp_scale, workspace,
                       a_codes_out=None, a_scale_out=None):
    M, d = xp.shape
    E, two_f, _ = w1.shape
    _check("moe_expert_ffn_fwd", _lib.moe_expert_ffn_fwd(
        _p(xp), _p(xp_scale), dtype_code(xp.dtype), _p(offsets), _p(w1), _p(w1_scale), _p(w2), _p(w2_scale),
        dtype_code(w1.dtype), M, d, E, two_f // 2, _p(h_save), _p(yp), _p(yp_scale), dtype_code(yp.dtype),
        _p(a_codes_out), _p(a_scale_out), _p(workspace), workspace.numel() * workspace.element_size(), _stream()))


def moe_expert_ffn_bwd(xp, h_save, d_yp, a_override, offsets, w1, w2, d_xp, d_w1, d_w2, accumulate, workspace):
    M, d = xp.shape
    E, two_f, _ = w1.shape
    _check("moe_expert_ffn_bwd", _lib.moe_expert_ffn_bwd(
        _p(xp), _p(h_save), _p(d_yp), _p(a_override), _p(offsets), _p(w1), _p(w2), dtype_code(xp.dtype), M, d, E,
        two_f // 2, _p(d_xp), _p(d_w1), _p(d_w2), dtype_code(d_w1.dtype), int(accumulate), _p(workspace),
        workspace.numel() * workspace.element_size(), _stream()))


def moe_quant_fp8(src, mode, codes, scales):
    rows, cols = src.shape
    _check("moe_quant_fp8", _lib.moe_quant_fp8(_p(src), dtype_code(src.dtype), rows, cols, mode, _p(codes),
                                               _p(scales), _stream()))


def moe_dequant_fp8(codes, scales, mode, dst):
    rows, cols = codes.shape
    _check("moe_dequant_fp8", _lib.moe_dequant_fp8(_p(codes), _p(scales), rows, cols, mode, _p(dst),
                                                   dtype_code(dst.dtype), _stream()))


def moe_transpose(src, dst):
    """src [batch, rows, cols] -> dst [batch, cols, rows]."""
    batch, rows, cols = src.shape
    assert tuple(dst.shape) == (batch, cols, rows) and dst.dtype == src.dtype
    _check("moe_transpose", _lib.moe_transpose(_p(src), dtype_code(src.dtype), batch, rows, cols, _p(dst), _stream()))


def moe_tgroup_tokens(rows: int, E: int) -> int:
    return _lib.moe_tgroup_tokens(rows, E)


def moe_quant_fp8_tgroup(src, offsets, pad_offsets, codes_t, e8m0):
    """src [rows, cols]; codes_t [cols, ldt] uint8; e8m0 [ldt/128, cols] uint8; pad_offsets [E+1] int32."""
    rows, cols = src.shape
    E = offsets.numel() - 1
    ldt = codes_t.shape[1]
    _check("moe_quant_fp8_tgroup", _lib.moe_quant_fp8_tgroup(_p(src), dtype_code(src.dtype), rows, cols, _p(offsets), E,
                                                             _p(pad_offsets), _p(codes_t), ldt, _p(e8m0), _stream()))


def moe_expert_ffn_bwd_fp8(d_yp, h_save, xp_deq, a_deq, offsets, w1t, w1t_scale, w2t, w2t_scale, d_xp, d_w1, d_w2,
                           accumulate, inter):
    """`inter` maps the names of the intermediate buffers of moe_ffn_bwd_fp8_args to tensors; xp_deq / a_deq may
    instead be (codes, scales) pairs of the forward's e4m3 operands."""
    M, d = d_yp.shape
    codes = {}
    if isinstance(xp_deq, tuple):
        codes["xp_codes"], codes["xp_scale"] = xp_deq
        xp_deq = None
    if isinstance(a_deq, tuple):
        codes["a_codes"], codes["a_scale"] = a_deq
        a_deq = None
    f = h_save.shape[1] // 2
    a = FfnBwdFp8Args()
    for name, t in (("d_yp", d_yp), ("h_save", h_save), ("xp_deq", xp_deq), ("a_deq", a_deq), ("offsets", offsets),
                    ("w1t", w1t), ("w1t_scale", w1t_scale), ("w2t", w2t), ("w2t_scale", w2t_scale), ("d_xp", d_xp),
                    ("d_w1", d_w1), ("d_w2", d_w2)):
        setattr(a, name, _p(t))
    for name in ("dy_codes", "dy_scale", "dh", "dh_codes", "dh_scale", "pad_offsets", "dy_t", "dy_e8m0", "dh_t",
                 "dh_e8m0", "a_t", "a_e8m0", "x_t", "x_e8m0"):
        setattr(a, name, _p(inter[name]))
    a.splitk_ws = _p(inter.get("splitk_ws"))
    for name, t in codes.items():
        setattr(a, name, _p(t))
    a.M, a.d, a.E, a.f = M, d, offsets.numel() - 1, f
    a.grad_dt = dtype_code(d_w1.dtype)
    a.accumulate = int(accumulate)
    a.ldt = inter["dy_t"].shape[1]
    _check("moe_expert_ffn_bwd_fp8", _lib.moe_expert_ffn_bwd_fp8(ctypes.byref(a), _stream()))


def moe_route_range(logits, k, renorm, e_lo, e_hi, topk_idx, topk_w, counts, offsets, perm, inv_perm, workspace):
    T, E = logits.shape
    _check("moe_route_range", _lib.moe_route_range(_p(logits), T, E, k, renorm, e_lo, e_hi, _p(topk_idx), _p(topk_w),
                                                   _p(counts), _p(offsets), _p(perm), _p(inv_perm), _p(workspace),
                                                   workspace.numel(), _stream()))


def moe_route_capacity_workspace_bytes(T, E, k) -> int:
    return _lib.moe_route_capacity_workspace_bytes(T, E, k)


def moe_route_capacity(logits, k, renorm, n_groups, capacity, topk_idx, topk_w, score, counts, offsets, perm, inv_perm,
                       workspace):
    T, E = logits.shape
    _check("moe_route_capacity", _lib.moe_route_capacity(
        _p(logits), T, E, k, renorm, n_groups, capacity, _p(topk_idx), _p(topk_w), _p(score), _p(counts), _p(offsets),
        _p(perm), _p(inv_perm), _p(workspace), workspace.numel() * workspace.element_size(), _stream()))


def moe_balance_loss(logits, counts, k, n_groups, alpha, loss, group_f, group_p, workspace):
    T, E = logits.shape
    _check("moe_balance_loss", _lib.moe_balance_loss(_p(logits), _p(counts), T, E, k, n_groups, alpha, _p(loss), _p(group_f),
                                                     _p(group_p), _p(workspace),
                                                     workspace.numel() * workspace.element_size(), _stream()))


def moe_balance_loss_bwd(logits, group_f, n_groups, alpha, d_logits):
    T, E = logits.shape
    _check("moe_balance_loss_bwd", _lib.moe_balance_loss_bwd(_p(logits), _p(group_f), T, E, n_groups, alpha, _p(d_logits),
                                                             _stream()))


def moe_row_map(perm, topk_w, offsets, row_token, row_w):
    T, k = topk_w.shape
    E = offsets.numel() - 1
    _check("moe_row_map", _lib.moe_row_map(_p(perm), _p(topk_w), _p(offsets), E, T, k, _p(row_token), _p(row_w), _stream()))


def moe_expert_ffn_fused_workspace_bytes(T, k, d, f) -> int:
    return _lib.moe_expert_ffn_fused_workspace_bytes(T, k, d, f)


def moe_expert_ffn_fused_fwd(x, row_token, row_w, offsets, w1, w2, k, h_save, ypw, workspace):
    T, d = x.shape
    E, two_f, _ = w1.shape
    _check("moe_expert_ffn_fused_fwd", _lib.moe_expert_ffn_fused_fwd(
        _p(x), _p(row_token), _p(row_w), _p(offsets), _p(w1), _p(w2), T, k, d, E, two_f // 2, _p(h_save), _p(ypw),
        _p(workspace), workspace.numel() * workspace.element_size(), _stream()))


def moe_expert_ffn_fused_bwd(x, dy, h_save, inv_perm, topk_w, row_w, offsets, w1, w2, k, d_xp, d_w1, d_w2, accumulate,
                             d_topk_w, workspace):
    T, d = x.shape
    E, two_f, _ = w1.shape
    _check("moe_expert_ffn_fused_bwd", _lib.moe_expert_ffn_fused_bwd(
        _p(x), _p(dy), _p(h_save), _p(inv_perm), _p(topk_w), _p(row_w), _p(offsets), _p(w1), _p(w2), T, k, d, E, two_f // 2,
        _p(d_xp), _p(d_w1), _p(d_w2), dtype_code(d_w1.dtype), int(accumulate), _p(d_topk_w), _p(workspace),
        workspace.numel() * workspace.element_size(), _stream()))
