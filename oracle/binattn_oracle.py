"""ctypes access to the CPU oracle (oracle/binattn_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg, never by the product package.  This file only
marshals numpy arrays; every arithmetic step lives in the C file.

bf16 tensors travel as uint16 bit patterns (numpy has no bf16).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "binattn_oracle.c")
_LIB = os.path.join(_HERE, "libbinattn_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, no fast-math, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-fPIC",
               "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    lib = C.CDLL(_LIB)
    p = C.c_void_p
    i64 = C.c_int64
    lib.ba_oracle_num_threads.restype = C.c_int
    lib.ba_oracle_sign_pm1.argtypes = [p, i64, p]
    lib.ba_oracle_sign_pack.argtypes = [p, i64, C.c_int, p]
    lib.ba_oracle_abs_mean.argtypes = [p, i64]
    lib.ba_oracle_abs_mean.restype = C.c_double
    lib.ba_oracle_logits_literal.argtypes = [p, p, i64, C.c_int, p, i64, p]
    lib.ba_oracle_logits_hamming.argtypes = [p, p, i64, C.c_int, p, i64, p]
    lib.ba_oracle_quant_v.argtypes = [p, i64, C.c_int, p, p]
    lib.ba_oracle_attention_rows.argtypes = [
        p, p, p, i64, C.c_int, p, C.c_int, i64, C.c_double, C.c_double, C.c_double,
        p, p, p, i64, p, p, p, p, p, p, p]
    lib.ba_oracle_algorithm1_rows.argtypes = [
        p, p, p, i64, C.c_int, p, C.c_int, i64, C.c_double, C.c_double, C.c_double,
        p, p, i64, C.c_int, p, i64, p]
    for f in ("ba_oracle_sign_pm1", "ba_oracle_sign_pack", "ba_oracle_logits_literal",
              "ba_oracle_logits_hamming", "ba_oracle_quant_v", "ba_oracle_attention_rows",
              "ba_oracle_algorithm1_rows"):
        getattr(lib, f).restype = None
    _lib = lib
    return lib


def num_threads() -> int:
    return int(_load().ba_oracle_num_threads())


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _u16(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, "bf16 data must be passed as uint16 bit patterns"
    return a


def _rows(rows, N) -> np.ndarray:
    if rows is None:
        return np.arange(N, dtype=np.int64)
    r = np.ascontiguousarray(np.asarray(rows, dtype=np.int64))
    assert r.ndim == 1 and (r.size == 0 or (r.min() >= 0 and r.max() < N))
    return r


def sign_pm1(x: np.ndarray) -> np.ndarray:
    x = _u16(x)
    s = np.empty(x.shape, dtype=np.int8)
    _load().ba_oracle_sign_pm1(_ptr(x), x.size, _ptr(s))
    return s


def sign_pack(x: np.ndarray) -> np.ndarray:
    """x: [..., d] bf16 bits -> uint32 [..., ceil(d/32)]."""
    x = _u16(x)
    d = x.shape[-1]
    W = (d + 31) // 32
    out = np.empty(x.shape[:-1] + (W,), dtype=np.uint32)
    _load().ba_oracle_sign_pack(_ptr(x), x.size // d, d, _ptr(out))
    return out


def abs_mean(x: np.ndarray) -> float:
    x = _u16(x)
    return float(_load().ba_oracle_abs_mean(_ptr(x), x.size))


def logits_literal(q: np.ndarray, k: np.ndarray, rows=None) -> np.ndarray:
    """q, k: [N, d] bf16 bits of one head -> int32 [n_rows, N]."""
    q, k = _u16(q), _u16(k)
    N, d = q.shape
    r = _rows(rows, N)
    out = np.empty((r.size, N), dtype=np.int32)
    _load().ba_oracle_logits_literal(_ptr(q), _ptr(k), N, d, _ptr(r), r.size, _ptr(out))
    return out


def logits_hamming(qw: np.ndarray, kw: np.ndarray, d: int, rows=None) -> np.ndarray:
    qw = np.ascontiguousarray(qw, dtype=np.uint32)
    kw = np.ascontiguousarray(kw, dtype=np.uint32)
    N = qw.shape[0]
    r = _rows(rows, N)
    out = np.empty((r.size, N), dtype=np.int32)
    _load().ba_oracle_logits_hamming(_ptr(qw), _ptr(kw), N, d, _ptr(r), r.size, _ptr(out))
    return out


def quant_v(v: np.ndarray):
    """v: [N, d] bf16 bits -> (codes int8 [N, d], delta float32 [d])."""
    v = _u16(v)
    N, d = v.shape
    vq = np.empty((N, d), dtype=np.int8)
    delta = np.empty((d,), dtype=np.float32)
    _load().ba_oracle_quant_v(_ptr(v), N, d, _ptr(vq), _ptr(delta))
    return vq, delta


def _bias_args(bias, N):
    if bias is None:
        return None, 0, 0
    b = np.ascontiguousarray(bias)
    assert b.shape == (N, N)
    if b.dtype == np.uint16:
        return b, 1, N
    if b.dtype == np.float32:
        return b, 2, N
    raise TypeError("bias must be uint16 (bf16 bits) or float32")


def attention_rows(q, k, v, bias, scale: float, mu_q: float, mu_k: float, vq, delta,
                   rows=None, want: Sequence[str] = ("O2", "O1")) -> dict:
    """One head by the definition (true row max).  Returns a dict with the
    arrays named in `want` out of O2, O1, P_hat, P_code, l, m, S."""
    q, k, v = _u16(q), _u16(k), _u16(v)
    N, d = q.shape
    r = _rows(rows, N)
    b, bdt, bstride = _bias_args(bias, N)
    vq = np.ascontiguousarray(vq, dtype=np.int8)
    delta = np.ascontiguousarray(delta, dtype=np.float32)
    shapes = {"O2": ((r.size, d), np.float64), "O1": ((r.size, d), np.float64),
              "P_hat": ((r.size, N), np.float64), "P_code": ((r.size, N), np.uint8),
              "l": ((r.size,), np.float64), "m": ((r.size,), np.float64),
              "S": ((r.size, N), np.float64)}
    out = {name: np.empty(*shapes[name]) for name in want}
    g = lambda name: _ptr(out.get(name))
    _load().ba_oracle_attention_rows(
        _ptr(q), _ptr(k), _ptr(v), N, d, _ptr(b), bdt, bstride, scale, mu_q, mu_k,
        _ptr(vq), _ptr(delta), _ptr(r), r.size,
        g("O2"), g("O1"), g("P_hat"), g("P_code"), g("l"), g("m"), g("S"))
    return out


def algorithm1_rows(q, k, v, bias, scale, mu_q, mu_k, vq, delta, Bv: int, quantise: bool,
                    rows=None) -> np.ndarray:
    """One head by Alg. 1 with key/value block size Bv -> float64 [n_rows, d]."""
    q, k, v = _u16(q), _u16(k), _u16(v)
    N, d = q.shape
    r = _rows(rows, N)
    b, bdt, bstride = _bias_args(bias, N)
    vq = np.ascontiguousarray(vq, dtype=np.int8)
    delta = np.ascontiguousarray(delta, dtype=np.float32)
    O = np.empty((r.size, d), dtype=np.float64)
    _load().ba_oracle_algorithm1_rows(
        _ptr(q), _ptr(k), _ptr(v), N, d, _ptr(b), bdt, bstride, scale, mu_q, mu_k,
        _ptr(vq), _ptr(delta), int(Bv), int(bool(quantise)), _ptr(r), r.size, _ptr(O))
    return O


def forward(q, k, v, bias, scale: float, use_mu: bool = True, rows=None,
            heads: Optional[Sequence[tuple]] = None, want: Sequence[str] = ("O2", "O1")) -> dict:
    """Whole-layer driver: q, k, v uint16 [B, H, N, d]; bias None, uint16 or
    float32 [H, N, N] (shared over the batch) or [B, H, N, N].
    Runs the per-head steps in the paper's order (phi on Q and K, psi on V, then
    the attention rows).  Returns arrays stacked as [B, H, n_rows, ...] plus
    mu_q, mu_k [B, H], vq [B, H, N, d], delta [B, H, d].  `heads` restricts the
    (b, h) pairs computed (others are left zero)."""
    q, k, v = _u16(q), _u16(k), _u16(v)
    B, H, N, d = q.shape
    r = _rows(rows, N)
    res = {"mu_q": np.ones((B, H)), "mu_k": np.ones((B, H)),
           "vq": np.zeros((B, H, N, d), np.int8), "delta": np.zeros((B, H, d), np.float32)}
    per = {"O2": (d,), "O1": (d,), "P_hat": (N,), "P_code": (N,), "S": (N,), "l": (), "m": ()}
    for name in want:
        dt = np.uint8 if name == "P_code" else np.float64
        res[name] = np.zeros((B, H, r.size) + per[name], dtype=dt)
    todo = heads if heads is not None else [(b, h) for b in range(B) for h in range(H)]
    for (b, h) in todo:
        if use_mu:
            res["mu_q"][b, h] = abs_mean(q[b, h])
            res["mu_k"][b, h] = abs_mean(k[b, h])
        vq, delta = quant_v(v[b, h])
        res["vq"][b, h], res["delta"][b, h] = vq, delta
        bb = None
        if bias is not None:
            bb = bias[h] if bias.ndim == 3 else bias[b, h]
        o = attention_rows(q[b, h], k[b, h], v[b, h], bb, scale, res["mu_q"][b, h],
                           res["mu_k"][b, h], vq, delta, rows=r, want=want)
        for name in want:
            res[name][b, h] = o[name]
    return res
