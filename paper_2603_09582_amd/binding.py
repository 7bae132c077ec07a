"""Thin ctypes binding of libbinattn.so (include/binattn.h).

Argument marshalling only: tensors are torch CUDA tensors used for device
memory and streams; every step of the path runs in the library's HIP kernels.
There is no fallback: if the shared library is missing, loading fails loudly.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbinattn.so")

BIAS_BF16, BIAS_F32 = 1, 2
FLAG_NO_MU, FLAG_NO_BIAS, FLAG_LUT, FLAG_WIDE8 = 1, 2, 4, 8
LOGITS_POPCOUNT, LOGITS_MFMA_I8, LOGITS_MFMA_FP4 = 0, 1, 2
LOGITS_ROWSUM = 0x100

EXPORTS = ["binattn_version", "binattn_strerror", "binattn_pack_qk", "binattn_workspace_bytes",
           "binattn_prepare_kv", "binattn_attend", "binattn_forward", "binattn_attend_axial",
           "binattn_forward_axial", "binattn_attend_relpos", "binattn_forward_relpos", "binattn_forward_fused",
           "binattn_forward_fused_relpos", "binattn_forward_static", "binattn_probe_valu", "binattn_attention", "binattn_attention_relpos",
           "binattn_logits_debug", "binattn_quant_v_debug"]

_lib = None


class BinAttnError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = lib().binattn_strerror(code).decode()
        super().__init__(f"{where} failed with {code}: {msg}")


def lib():
    """Load libbinattn.so (built in-tree by paper_2603_09582_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} not found: build it with `python -m paper_2603_09582_amd.build` "
            "(there is no non-HIP fallback)")
    L = C.CDLL(LIB_PATH)
    vp, i64p = C.c_void_p, C.POINTER(C.c_int64)
    L.binattn_version.restype = C.c_int
    L.binattn_strerror.restype = C.c_char_p
    L.binattn_strerror.argtypes = [C.c_int]
    L.binattn_workspace_bytes.restype = C.c_size_t
    L.binattn_workspace_bytes.argtypes = [C.c_int] * 4
    L.binattn_pack_qk.restype = C.c_int
    L.binattn_pack_qk.argtypes = [vp, vp, C.c_int, C.c_int, C.c_int, C.c_int, i64p, i64p,
                                  vp, vp, vp, vp, vp]
    L.binattn_forward.restype = C.c_int
    L.binattn_forward.argtypes = [vp, vp, vp, vp, vp, i64p, vp, C.c_int, i64p, C.c_float,
                                  C.c_int, C.c_int, C.c_int, C.c_int, vp, i64p, vp, C.c_size_t,
                                  C.c_uint, vp]
    L.binattn_forward_static.restype = C.c_int
    L.binattn_forward_static.argtypes = [vp, vp, vp, vp, vp, i64p, vp, C.c_int, i64p, C.c_float,
                                         C.c_int, C.c_int, C.c_int, C.c_int, vp, i64p, C.c_uint, vp]
    L.binattn_probe_valu.restype = C.c_int
    L.binattn_probe_valu.argtypes = [C.c_int, C.c_int, C.c_int, vp, vp]
    L.binattn_prepare_kv.restype = C.c_int
    L.binattn_prepare_kv.argtypes = [vp, vp, i64p, C.c_int, C.c_int, C.c_int, C.c_int, vp,
                                     C.c_size_t, vp]
    L.binattn_attend.restype = C.c_int
    L.binattn_attend.argtypes = [vp, vp, vp, vp, C.c_int, i64p, C.c_float, C.c_int, C.c_int, C.c_int,
                                 C.c_int, vp, i64p, vp, C.c_size_t, C.c_uint, vp]
    L.binattn_attend_axial.restype = C.c_int
    L.binattn_attend_axial.argtypes = [vp, vp, vp, vp, vp, C.c_int, C.c_int, C.c_float, C.c_int, C.c_int,
                                       C.c_int, C.c_int, vp, i64p, vp, C.c_size_t, C.c_uint, vp]
    L.binattn_forward_axial.restype = C.c_int
    L.binattn_forward_axial.argtypes = [vp, vp, vp, vp, vp, i64p, vp, vp, C.c_int, C.c_int, C.c_float,
                                        C.c_int, C.c_int, C.c_int, C.c_int, vp, i64p, vp, C.c_size_t,
                                        C.c_uint, vp]
    L.binattn_attend_relpos.restype = C.c_int
    L.binattn_attend_relpos.argtypes = [vp, vp, vp, vp, C.c_int, C.c_int, C.c_float, C.c_int, C.c_int,
                                        C.c_int, C.c_int, vp, i64p, vp, C.c_size_t, C.c_uint, vp]
    L.binattn_forward_relpos.restype = C.c_int
    L.binattn_forward_relpos.argtypes = [vp, vp, vp, vp, vp, i64p, vp, C.c_int, C.c_int, C.c_float,
                                         C.c_int, C.c_int, C.c_int, C.c_int, vp, i64p, vp, C.c_size_t,
                                         C.c_uint, vp]
    L.binattn_forward_fused.restype = C.c_int
    L.binattn_forward_fused.argtypes = [vp, vp, vp, i64p, i64p, i64p, vp, C.c_int, i64p, C.c_float, C.c_int,
                                        C.c_int, C.c_int, C.c_int, vp, i64p, vp, vp, C.c_uint, vp]
    L.binattn_attention.restype = C.c_int
    L.binattn_attention.argtypes = [vp, vp, vp, i64p, i64p, i64p, vp, C.c_int, i64p, C.c_float, C.c_int,
                                    C.c_int, C.c_int, C.c_int, vp, i64p, vp, vp, vp, C.c_size_t, C.c_uint, vp]
    L.binattn_forward_fused_relpos.restype = C.c_int
    L.binattn_forward_fused_relpos.argtypes = [vp, vp, vp, i64p, i64p, i64p, vp, C.c_int, C.c_int, C.c_float,
                                               C.c_int, C.c_int, C.c_int, C.c_int, vp, i64p, vp, vp, C.c_uint, vp]
    L.binattn_attention_relpos.restype = C.c_int
    L.binattn_attention_relpos.argtypes = [vp, vp, vp, i64p, i64p, i64p, vp, C.c_int, C.c_int, C.c_float,
                                           C.c_int, C.c_int, C.c_int, C.c_int, vp, i64p, vp, vp, vp, C.c_size_t,
                                           C.c_uint, vp]
    L.binattn_logits_debug.restype = C.c_int
    L.binattn_logits_debug.argtypes = [vp, vp, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                       vp, C.c_int, vp, C.c_size_t, vp]
    L.binattn_quant_v_debug.restype = C.c_int
    L.binattn_quant_v_debug.argtypes = [vp, i64p, C.c_int, C.c_int, C.c_int, C.c_int, vp, vp, vp,
                                        C.c_size_t, vp]
    _lib = L
    return L


def _strides3(t: torch.Tensor):
    assert t.dim() == 4 and t.stride(3) == 1, "innermost stride must be 1"
    return (C.c_int64 * 3)(t.stride(0), t.stride(1), t.stride(2))


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _check(rc: int, where: str):
    if rc != 0:
        raise BinAttnError(rc, where)


def workspace_bytes(B: int, H: int, N: int, d: int) -> int:
    return int(lib().binattn_workspace_bytes(B, H, N, d))


def alloc_workspace(B: int, H: int, N: int, d: int, device="cuda") -> torch.Tensor:
    n = workspace_bytes(B, H, N, d)
    if n == 0:
        raise BinAttnError(-2, "binattn_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def pack_qk(q: torch.Tensor, k: torch.Tensor, q_bits=None, k_bits=None, mu_q=None, mu_k=None):
    """binattn_pack_qk: bf16 [B,H,N,d] -> (q_bits, k_bits int32 [B,H,N,W], mu_q, mu_k f32 [B,H])."""
    assert q.dtype == torch.bfloat16 and k.dtype == torch.bfloat16 and q.is_cuda and k.is_cuda
    B, H, N, d = q.shape
    W = (d + 31) // 32
    dev = q.device
    if q_bits is None:
        q_bits = torch.empty(B, H, N, W, dtype=torch.int32, device=dev)
    if k_bits is None:
        k_bits = torch.empty(B, H, N, W, dtype=torch.int32, device=dev)
    if mu_q is None:
        mu_q = torch.empty(B, H, dtype=torch.float32, device=dev)
    if mu_k is None:
        mu_k = torch.empty(B, H, dtype=torch.float32, device=dev)
    rc = lib().binattn_pack_qk(q.data_ptr(), k.data_ptr(), B, H, N, d, _strides3(q), _strides3(k),
                               q_bits.data_ptr(), k_bits.data_ptr(), mu_q.data_ptr(),
                               mu_k.data_ptr(), _stream())
    _check(rc, "binattn_pack_qk")
    return q_bits, k_bits, mu_q, mu_k


def _bias_args(bias):
    if bias is None:
        return None, BIAS_BF16, None
    assert bias.stride(-1) == 1
    bdt = {torch.bfloat16: BIAS_BF16, torch.float32: BIAS_F32}[bias.dtype]
    if bias.dim() == 3:
        bst = (C.c_int64 * 3)(0, bias.stride(0), bias.stride(1))
    else:
        bst = (C.c_int64 * 3)(bias.stride(0), bias.stride(1), bias.stride(2))
    return bias.data_ptr(), bdt, bst


def prepare_kv(k_bits: torch.Tensor, v: torch.Tensor, workspace: torch.Tensor) -> None:
    """binattn_prepare_kv: V quantisation and key-side operand layout into `workspace`."""
    assert v.dtype == torch.bfloat16 and v.is_cuda
    B, H, N, d = v.shape
    rc = lib().binattn_prepare_kv(k_bits.data_ptr(), v.data_ptr(), _strides3(v), B, H, N, d,
                                  workspace.data_ptr(), workspace.numel(), _stream())
    _check(rc, "binattn_prepare_kv")


def attend(q_bits: torch.Tensor, mu_q: Optional[torch.Tensor], mu_k: Optional[torch.Tensor],
           bias: Optional[torch.Tensor], scale: float, d: int, workspace: torch.Tensor,
           out: Optional[torch.Tensor] = None, flags: int = 0) -> torch.Tensor:
    """binattn_attend: the fused attention loop over a prepared workspace."""
    B, H, N, _ = q_bits.shape
    if out is None:
        out = torch.empty(B, H, N, d, dtype=torch.bfloat16, device=q_bits.device)
    bptr, bdt, bst = _bias_args(bias)
    rc = lib().binattn_attend(
        q_bits.data_ptr(), None if mu_q is None else mu_q.data_ptr(),
        None if mu_k is None else mu_k.data_ptr(), bptr, bdt, bst, float(scale), B, H, N, d,
        out.data_ptr(), _strides3(out), workspace.data_ptr(), workspace.numel(), int(flags),
        _stream())
    _check(rc, "binattn_attend")
    return out


def _axial_tables(bias_y: torch.Tensor, bias_x: torch.Tensor, H: int):
    assert bias_y.dtype == torch.float32 and bias_x.dtype == torch.float32
    assert bias_y.is_contiguous() and bias_x.is_contiguous() and bias_y.shape[0] == H == bias_x.shape[0]
    Gy, Gx = (bias_y.shape[1] + 1) // 2, (bias_x.shape[1] + 1) // 2
    return Gy, Gx


def attend_axial(q_bits: torch.Tensor, mu_q: Optional[torch.Tensor], mu_k: Optional[torch.Tensor],
                 bias_y: torch.Tensor, bias_x: torch.Tensor, scale: float, d: int,
                 workspace: torch.Tensor, out: Optional[torch.Tensor] = None, flags: int = 0) -> torch.Tensor:
    """binattn_attend_axial: bias_y fp32 [H, 2Gy-1], bias_x fp32 [H, 2Gx-1]; N = Gy * Gx."""
    B, H, N, _ = q_bits.shape
    Gy, Gx = _axial_tables(bias_y, bias_x, H)
    if out is None:
        out = torch.empty(B, H, N, d, dtype=torch.bfloat16, device=q_bits.device)
    rc = lib().binattn_attend_axial(
        q_bits.data_ptr(), None if mu_q is None else mu_q.data_ptr(),
        None if mu_k is None else mu_k.data_ptr(), bias_y.data_ptr(), bias_x.data_ptr(), Gy, Gx,
        float(scale), B, H, N, d, out.data_ptr(), _strides3(out), workspace.data_ptr(),
        workspace.numel(), int(flags), _stream())
    _check(rc, "binattn_attend_axial")
    return out


def forward_axial(q_bits: torch.Tensor, k_bits: torch.Tensor, mu_q: Optional[torch.Tensor],
                  mu_k: Optional[torch.Tensor], v: torch.Tensor, bias_y: torch.Tensor,
                  bias_x: torch.Tensor, scale: float, out: Optional[torch.Tensor] = None,
                  workspace: Optional[torch.Tensor] = None, flags: int = 0) -> torch.Tensor:
    """binattn_forward_axial = prepare_kv + attend_axial."""
    B, H, N, d = v.shape
    Gy, Gx = _axial_tables(bias_y, bias_x, H)
    if out is None:
        out = torch.empty(B, H, N, d, dtype=torch.bfloat16, device=v.device)
    if workspace is None:
        workspace = alloc_workspace(B, H, N, d, v.device)
    rc = lib().binattn_forward_axial(
        q_bits.data_ptr(), k_bits.data_ptr(), None if mu_q is None else mu_q.data_ptr(),
        None if mu_k is None else mu_k.data_ptr(), v.data_ptr(), _strides3(v), bias_y.data_ptr(),
        bias_x.data_ptr(), Gy, Gx, float(scale), B, H, N, d, out.data_ptr(), _strides3(out),
        workspace.data_ptr(), workspace.numel(), int(flags), _stream())
    _check(rc, "binattn_forward_axial")
    return out


def _relpos_table(table: torch.Tensor, H: int):
    assert table.dtype == torch.float32 and table.is_contiguous() and table.dim() == 3 and table.shape[0] == H
    return (table.shape[1] + 1) // 2, (table.shape[2] + 1) // 2


def attend_relpos(q_bits: torch.Tensor, mu_q: Optional[torch.Tensor], mu_k: Optional[torch.Tensor],
                  table: torch.Tensor, scale: float, d: int, workspace: torch.Tensor,
                  out: Optional[torch.Tensor] = None, flags: int = 0) -> torch.Tensor:
    """binattn_attend_relpos: table fp32 [H, 2Gy-1, 2Gx-1]; N = Gy * Gx."""
    B, H, N, _ = q_bits.shape
    Gy, Gx = _relpos_table(table, H)
    if out is None:
        out = torch.empty(B, H, N, d, dtype=torch.bfloat16, device=q_bits.device)
    rc = lib().binattn_attend_relpos(
        q_bits.data_ptr(), None if mu_q is None else mu_q.data_ptr(),
        None if mu_k is None else mu_k.data_ptr(), table.data_ptr(), Gy, Gx, float(scale), B, H, N, d,
        out.data_ptr(), _strides3(out), workspace.data_ptr(), workspace.numel(), int(flags), _stream())
    _check(rc, "binattn_attend_relpos")
    return out


def forward_relpos(q_bits: torch.Tensor, k_bits: torch.Tensor, mu_q: Optional[torch.Tensor],
                   mu_k: Optional[torch.Tensor], v: torch.Tensor, table: torch.Tensor, scale: float,
                   out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                   flags: int = 0) -> torch.Tensor:
    """binattn_forward_relpos = prepare_kv + attend_relpos."""
    B, H, N, d = v.shape
    Gy, Gx = _relpos_table(table, H)
    if out is None:
        out = torch.empty(B, H, N, d, dtype=torch.bfloat16, device=v.device)
    if workspace is None:
        workspace = alloc_workspace(B, H, N, d, v.device)
    rc = lib().binattn_forward_relpos(
        q_bits.data_ptr(), k_bits.data_ptr(), None if mu_q is None else mu_q.data_ptr(),
        None if mu_k is None else mu_k.data_ptr(), v.data_ptr(), _strides3(v), table.data_ptr(), Gy, Gx,
        float(scale), B, H, N, d, out.data_ptr(), _strides3(out), workspace.data_ptr(),
        workspace.numel(), int(flags), _stream())
    _check(rc, "binattn_forward_relpos")
    return out


def forward(q_bits: torch.Tensor, k_bits: torch.Tensor, mu_q: Optional[torch.Tensor],
            mu_k: Optional[torch.Tensor], v: torch.Tensor, bias: Optional[torch.Tensor],
            scale: float, out: Optional[torch.Tensor] = None,
            workspace: Optional[torch.Tensor] = None, flags: int = 0) -> torch.Tensor:
    """binattn_forward.  bias: None, [H,N,N] (shared over the batch) or [B,H,N,N], bf16 or f32."""
    assert v.dtype == torch.bfloat16 and v.is_cuda
    B, H, N, d = v.shape
    if out is None:
        out = torch.empty(B, H, N, d, dtype=torch.bfloat16, device=v.device)
    if workspace is None:
        workspace = alloc_workspace(B, H, N, d, v.device)
    bptr, bdt, bst = _bias_args(bias)
    rc = lib().binattn_forward(
        q_bits.data_ptr(), k_bits.data_ptr(),
        None if mu_q is None else mu_q.data_ptr(), None if mu_k is None else mu_k.data_ptr(),
        v.data_ptr(), _strides3(v), bptr, bdt, bst, float(scale), B, H, N, d,
        out.data_ptr(), _strides3(out), workspace.data_ptr(), workspace.numel(), int(flags),
        _stream())
    _check(rc, "binattn_forward")
    return out


STATIC_SCRATCH_BYTES = 64 << 20


def forward_static(q_bits: torch.Tensor, k_bits: torch.Tensor, mu_q: Optional[torch.Tensor],
                   mu_k: Optional[torch.Tensor], v: torch.Tensor, bias: Optional[torch.Tensor],
                   scale: float, out: torch.Tensor, flags: int = 0) -> torch.Tensor:
    """binattn_forward_static: binattn_forward on the library's own static scratch.  `out` is
    the caller's (this wrapper allocates nothing either)."""
    B, H, N, d = v.shape
    bptr, bdt, bst = _bias_args(bias)
    rc = lib().binattn_forward_static(
        q_bits.data_ptr(), k_bits.data_ptr(),
        None if mu_q is None else mu_q.data_ptr(), None if mu_k is None else mu_k.data_ptr(),
        v.data_ptr(), _strides3(v), bptr, bdt, bst, float(scale), B, H, N, d,
        out.data_ptr(), _strides3(out), int(flags), _stream())
    _check(rc, "binattn_forward_static")
    return out


def forward_fused(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, bias: Optional[torch.Tensor],
                  scale: float, out: Optional[torch.Tensor] = None, mu_q: Optional[torch.Tensor] = None,
                  mu_k: Optional[torch.Tensor] = None, flags: int = 0) -> torch.Tensor:
    """binattn_forward_fused: the whole forward pass in one launch (N <= 256)."""
    assert q.dtype == k.dtype == v.dtype == torch.bfloat16 and q.is_cuda
    B, H, N, d = q.shape
    if out is None:
        out = torch.empty(B, H, N, d, dtype=torch.bfloat16, device=q.device)
    bptr, bdt, bst = _bias_args(bias)
    rc = lib().binattn_forward_fused(
        q.data_ptr(), k.data_ptr(), v.data_ptr(), _strides3(q), _strides3(k), _strides3(v), bptr, bdt,
        bst, float(scale), B, H, N, d, out.data_ptr(), _strides3(out),
        None if mu_q is None else mu_q.data_ptr(), None if mu_k is None else mu_k.data_ptr(),
        int(flags), _stream())
    _check(rc, "binattn_forward_fused")
    return out


def attention(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, bias: Optional[torch.Tensor], scale: float,
              out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
              mu_q: Optional[torch.Tensor] = None, mu_k: Optional[torch.Tensor] = None, flags: int = 0) -> torch.Tensor:
    """binattn_attention: the whole forward pass from the bf16 tensors, any N."""
    assert q.dtype == k.dtype == v.dtype == torch.bfloat16 and q.is_cuda
    B, H, N, d = q.shape
    if out is None:
        out = torch.empty(B, H, N, d, dtype=torch.bfloat16, device=q.device)
    if workspace is None and N > 256:
        workspace = alloc_workspace(B, H, N, d, q.device)
    bptr, bdt, bst = _bias_args(bias)
    rc = lib().binattn_attention(
        q.data_ptr(), k.data_ptr(), v.data_ptr(), _strides3(q), _strides3(k), _strides3(v), bptr, bdt,
        bst, float(scale), B, H, N, d, out.data_ptr(), _strides3(out),
        None if mu_q is None else mu_q.data_ptr(), None if mu_k is None else mu_k.data_ptr(),
        None if workspace is None else workspace.data_ptr(), 0 if workspace is None else workspace.numel(),
        int(flags), _stream())
    _check(rc, "binattn_attention")
    return out


def attention_relpos(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, table: torch.Tensor, scale: float,
                     out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                     mu_q: Optional[torch.Tensor] = None, mu_k: Optional[torch.Tensor] = None, flags: int = 0) -> torch.Tensor:
    """binattn_attention_relpos: the forward pass from the bf16 tensors with the head's relative-position table, any N."""
    assert q.dtype == k.dtype == v.dtype == torch.bfloat16 and q.is_cuda
    B, H, N, d = q.shape
    Gy, Gx = _relpos_table(table, H)
    if out is None:
        out = torch.empty(B, H, N, d, dtype=torch.bfloat16, device=q.device)
    if workspace is None:
        workspace = alloc_workspace(B, H, N, d, q.device)
    rc = lib().binattn_attention_relpos(
        q.data_ptr(), k.data_ptr(), v.data_ptr(), _strides3(q), _strides3(k), _strides3(v), table.data_ptr(),
        Gy, Gx, float(scale), B, H, N, d, out.data_ptr(), _strides3(out),
        None if mu_q is None else mu_q.data_ptr(), None if mu_k is None else mu_k.data_ptr(),
        workspace.data_ptr(), workspace.numel(), int(flags), _stream())
    _check(rc, "binattn_attention_relpos")
    return out


def forward_fused_relpos(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, table: torch.Tensor, scale: float,
                         out: Optional[torch.Tensor] = None, mu_q: Optional[torch.Tensor] = None,
                         mu_k: Optional[torch.Tensor] = None, flags: int = 0) -> torch.Tensor:
    """binattn_forward_fused_relpos: one launch, bias from the head's relative-position table (N <= 256)."""
    assert q.dtype == k.dtype == v.dtype == torch.bfloat16 and q.is_cuda
    B, H, N, d = q.shape
    Gy, Gx = _relpos_table(table, H)
    if out is None:
        out = torch.empty(B, H, N, d, dtype=torch.bfloat16, device=q.device)
    rc = lib().binattn_forward_fused_relpos(
        q.data_ptr(), k.data_ptr(), v.data_ptr(), _strides3(q), _strides3(k), _strides3(v), table.data_ptr(),
        Gy, Gx, float(scale), B, H, N, d, out.data_ptr(), _strides3(out),
        None if mu_q is None else mu_q.data_ptr(), None if mu_k is None else mu_k.data_ptr(),
        int(flags), _stream())
    _check(rc, "binattn_forward_fused_relpos")
    return out


def logits_debug(q_bits: torch.Tensor, k_bits: torch.Tensor, d: int, row_begin: int, row_end: int,
                 variant: int, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    B, H, N, _ = q_bits.shape
    shape = (B, H, row_end - row_begin) if variant & LOGITS_ROWSUM else (B, H, row_end - row_begin, N)
    out = torch.empty(shape, dtype=torch.int32, device=q_bits.device)
    if workspace is None and (variant & ~LOGITS_ROWSUM) == LOGITS_MFMA_FP4:
        workspace = alloc_workspace(B, H, N, d, q_bits.device)
    rc = lib().binattn_logits_debug(
        q_bits.data_ptr(), k_bits.data_ptr(), B, H, N, d, row_begin, row_end, out.data_ptr(),
        variant, None if workspace is None else workspace.data_ptr(),
        0 if workspace is None else workspace.numel(), _stream())
    _check(rc, "binattn_logits_debug")
    return out


PROBE_OPS = {"fma": 0, "exp2": 1, "add": 2, "max3": 3, "cvt_pk_u8": 4, "cvt_f32_i32": 5, "or": 6, "mul": 7,
             "lshl": 8, "and": 9, "xor": 10, "min3_i32": 11, "lshl_add": 12, "mov": 13, "add_u32": 14, "perm": 15}
PROBE_PARTNERS = ("fma", "cvt_pk_u8", "exp2", "or")
PROBE_SOFTMAX = 64
PROBE_CHAINS = 8


def probe_valu(op: int, iters: int, blocks: int, out: torch.Tensor) -> None:
    """binattn_probe_valu: the issue-rate probe (a measurement aid, see include/binattn.h)."""
    assert out.dtype == torch.float32 and out.numel() >= blocks * 256
    _check(lib().binattn_probe_valu(op, iters, blocks, out.data_ptr(), _stream()), "binattn_probe_valu")


def quant_v_debug(v: torch.Tensor, workspace: Optional[torch.Tensor] = None):
    B, H, N, d = v.shape
    vq = torch.empty(B, H, N, d, dtype=torch.int8, device=v.device)
    delta = torch.empty(B, H, d, dtype=torch.float32, device=v.device)
    if workspace is None:
        workspace = alloc_workspace(B, H, N, d, v.device)
    rc = lib().binattn_quant_v_debug(v.data_ptr(), _strides3(v), B, H, N, d, vq.data_ptr(),
                                     delta.data_ptr(), workspace.data_ptr(), workspace.numel(),
                                     _stream())
    _check(rc, "binattn_quant_v_debug")
    return vq, delta


def binary_attention(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor,
                     bias: Optional[torch.Tensor], scale: float, flags: int = 0,
                     workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """The whole hot path: pack_qk followed by forward."""
    q_bits, k_bits, mu_q, mu_k = pack_qk(q, k)
    return forward(q_bits, k_bits, mu_q, mu_k, v, bias, scale, workspace=workspace, flags=flags)
