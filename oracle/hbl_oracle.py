"""ctypes wrapper over the CPU oracle (oracle/hbl_oracle.c).

TEST INFRASTRUCTURE ONLY: used by tests/, by ``__graft_entry__.smoke()`` and by
the ``cpu_baseline`` leg of ``bench.py``.  It never touches the GPU library and
the GPU library never touches it.  Arrays are numpy; bf16 tensors are uint16
bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hbl_oracle.c")
_LIB = os.path.join(_HERE, "libhbl_oracle.so")

F32, BF16 = 0, 1
EPS = 1e-5

# -O2 keeps gcc from any value-changing transformation; -ffp-contract=off forbids
# fused multiply-add so that every fp32 operation of the oracle rounds once.
CFLAGS = ["-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared", "-std=c11",
          "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (a few seconds).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.run(["gcc", *CFLAGS, _SRC, "-o", tmp, "-lm"], check=True)
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        i64, f32, ci, vp = ctypes.c_int64, ctypes.c_float, ctypes.c_int, ctypes.c_void_p
        _lib.hblo_num_threads.restype = ci
        _lib.hblo_ternarize_weights_absmean.argtypes = [vp, i64, i64, f32, vp, vp]
        _lib.hblo_hadamard_dense.argtypes = [ci, vp]
        _lib.hblo_fwht_rows.argtypes = [vp, i64, i64]
        _lib.hblo_rmsnorm.argtypes = [vp, ci, i64, i64, vp, f32, vp]
        _lib.hblo_hadamard_backward.argtypes = [vp, ci, i64, i64, vp, ci]
        _lib.hblo_fwht_quant.argtypes = [vp, ci, i64, i64, ci, f32, ci, vp, vp, vp]
        _lib.hblo_gemm_i32.argtypes = [vp, i64, i64, vp, i64, vp]
        _lib.hblo_dequant_bf16.argtypes = [vp, i64, i64, vp, vp, i64, vp]
        _lib.hblo_kv_quant_absmax.argtypes = [vp, ci, i64, i64, ci, f32, vp, vp, vp]
        _lib.hblo_kv_dequant.argtypes = [vp, vp, i64, i64, ci, vp, ci]
        _lib.hblo_bitlinear_forward.argtypes = [vp, ci, i64, i64, vp, i64, vp, i64, ci, f32, ci, vp, vp, vp, vp]
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _check(rc: int, what: str):
    if rc != 0:
        raise ValueError(f"oracle {what} rejected its arguments (status {rc})")


def num_threads() -> int:
    return int(lib().hblo_num_threads())


def _x_dtype(x: np.ndarray) -> int:
    if x.dtype == np.float32:
        return F32
    if x.dtype == np.uint16:
        return BF16
    raise TypeError("x must be float32 or uint16 (bf16 bit patterns)")


def ternarize_weights_absmean(W: np.ndarray, eps: float = EPS) -> Tuple[np.ndarray, np.float32]:
    """Eq. 1: returns (codes int8 [N,K] in {-1,0,1}, alpha fp32)."""
    W = np.ascontiguousarray(W, dtype=np.float32)
    N, K = W.shape
    codes = np.empty((N, K), dtype=np.int8)
    alpha = np.zeros(1, dtype=np.float32)
    _check(lib().hblo_ternarize_weights_absmean(_p(W), N, K, eps, _p(codes), _p(alpha)), "ternarize")
    return codes, alpha[0]


def hadamard_dense(m: int) -> np.ndarray:
    """Eq. 4: dense H_m (2^m x 2^m, fp64) built by the recursion."""
    n = 1 << m
    H = np.zeros((n, n), dtype=np.float64)
    _check(lib().hblo_hadamard_dense(m, _p(H)), "hadamard_dense")
    return H


def fwht_rows(x: np.ndarray) -> np.ndarray:
    """Eq. 3: Hadamard(x) for every row of a [T,n] fp32 array (returns a new array)."""
    out = np.array(x, dtype=np.float32, order="C", copy=True)
    T, n = out.shape
    _check(lib().hblo_fwht_rows(_p(out), T, n), "fwht_rows")
    return out


def rmsnorm(x: np.ndarray, gain: np.ndarray, ln_eps: float) -> np.ndarray:
    """LN of Eq. 7 as RMS normalisation: x [T,K] fp32 / bf16 bits, gain [K] fp32 -> fp32 [T,K]."""
    x = np.ascontiguousarray(x)
    gain = np.ascontiguousarray(gain, dtype=np.float32)
    T, K = x.shape
    assert gain.shape == (K,)
    out = np.empty((T, K), dtype=np.float32)
    _check(lib().hblo_rmsnorm(_p(x), _x_dtype(x), T, K, _p(gain), ln_eps, _p(out)), "rmsnorm")
    return out


def hadamard_backward(g: np.ndarray, out_bf16: bool = False) -> np.ndarray:
    """Eq. 8: gradient w.r.t. X from the gradient w.r.t. Hadamard(X), row by row ([T,n] fp32 or bf16 bits).
    Returns fp32, or bf16 bit patterns (uint16) if ``out_bf16``."""
    g = np.ascontiguousarray(g)
    T, n = g.shape
    out = np.empty((T, n), dtype=np.uint16 if out_bf16 else np.float32)
    _check(lib().hblo_hadamard_backward(_p(g), _x_dtype(g), T, n, _p(out), BF16 if out_bf16 else F32),
           "hadamard_backward")
    return out


def fwht_quant(x: np.ndarray, bits: int, hadamard: bool = True, eps: float = EPS, want_xr: bool = False):
    """Hadamard (optional) + Eq. 5/6.  Returns (codes int8 [T,K], s_dequant fp32 [T][, x_r fp32 [T,K]])."""
    x = np.ascontiguousarray(x)
    T, K = x.shape
    codes = np.empty((T, K), dtype=np.int8)
    sdeq = np.empty(T, dtype=np.float32)
    xr = np.empty((T, K), dtype=np.float32) if want_xr else None
    _check(lib().hblo_fwht_quant(_p(x), _x_dtype(x), T, K, bits, eps, int(hadamard), _p(codes), _p(sdeq), _p(xr)),
           "fwht_quant")
    return (codes, sdeq, xr) if want_xr else (codes, sdeq)


def gemm_i32(q: np.ndarray, c: np.ndarray) -> np.ndarray:
    """acc[t,o] = sum_k q[t,k]*c[o,k] in int32 (exact)."""
    q = np.ascontiguousarray(q, dtype=np.int8)
    c = np.ascontiguousarray(c, dtype=np.int8)
    T, K = q.shape
    N, K2 = c.shape
    if K != K2:
        raise ValueError("inner sizes differ")
    acc = np.empty((T, N), dtype=np.int32)
    _check(lib().hblo_gemm_i32(_p(q), T, K, _p(c), N, _p(acc)), "gemm_i32")
    return acc


def dequant_bf16(acc: np.ndarray, sdeq: np.ndarray, w_scales: np.ndarray) -> np.ndarray:
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    sdeq = np.ascontiguousarray(sdeq, dtype=np.float32)
    w_scales = np.ascontiguousarray(np.atleast_1d(w_scales), dtype=np.float32)
    T, N = acc.shape
    y = np.empty((T, N), dtype=np.uint16)
    _check(lib().hblo_dequant_bf16(_p(acc), T, N, _p(sdeq), _p(w_scales), w_scales.size, _p(y)), "dequant_bf16")
    return y


def bitlinear_forward(x: np.ndarray, wcodes: np.ndarray, w_scales, bits: int, hadamard: bool,
                      eps: float = EPS, want_intermediates: bool = False):
    """Eq. 7.  Returns y (uint16 bf16 bits [T,N]) or (y, codes, s_dequant, acc)."""
    x = np.ascontiguousarray(x)
    wcodes = np.ascontiguousarray(wcodes, dtype=np.int8)
    w_scales = np.ascontiguousarray(np.atleast_1d(w_scales), dtype=np.float32)
    T, K = x.shape
    N, K2 = wcodes.shape
    if K != K2:
        raise ValueError("inner sizes differ")
    y = np.empty((T, N), dtype=np.uint16)
    codes = sdeq = acc = None
    if want_intermediates:
        codes = np.empty((T, K), dtype=np.int8)
        sdeq = np.empty(T, dtype=np.float32)
        acc = np.empty((T, N), dtype=np.int32)
    _check(lib().hblo_bitlinear_forward(_p(x), _x_dtype(x), T, K, _p(wcodes), N, _p(w_scales), w_scales.size,
                                        bits, eps, int(hadamard), _p(y), _p(codes), _p(sdeq), _p(acc)),
           "bitlinear_forward")
    return (y, codes, sdeq, acc) if want_intermediates else y


def hbitlinear_forward(x, wcodes, w_scales, bits, eps: float = EPS, **kw):
    return bitlinear_forward(x, wcodes, w_scales, bits, True, eps, **kw)


def plain_bitlinear_forward(x, wcodes, w_scales, bits, eps: float = EPS, **kw):
    return bitlinear_forward(x, wcodes, w_scales, bits, False, eps, **kw)


def kv_quant_absmax(x: np.ndarray, bits: int, eps: float = EPS):
    """Low-bit head states (Section 3.1, Main Results): x [rows, d] fp32 or bf16 bits -> (unsigned codes [rows, d] uint8,
    packed [rows, d*bits/8] uint8, scales [rows] fp32)."""
    x = np.ascontiguousarray(x)
    rows, d = x.shape
    codes = np.empty((rows, d), np.uint8)
    packed = np.empty((rows, d * bits // 8), np.uint8)
    scales = np.empty(rows, np.float32)
    _check(lib().hblo_kv_quant_absmax(_p(x), _x_dtype(x), rows, d, bits, eps, _p(codes), _p(packed), _p(scales)),
           "kv_quant_absmax")
    return codes, packed, scales


def kv_dequant(codes: np.ndarray, scales: np.ndarray, bits: int, out_bf16: bool = False) -> np.ndarray:
    """(u - 2^(bits-1)) * scale per row, fp32 or bf16 bit patterns."""
    codes = np.ascontiguousarray(codes, np.uint8)
    scales = np.ascontiguousarray(scales, np.float32)
    rows, d = codes.shape
    out = np.empty((rows, d), np.uint16 if out_bf16 else np.float32)
    _check(lib().hblo_kv_dequant(_p(codes), _p(scales), rows, d, bits, _p(out), 1 if out_bf16 else 0), "kv_dequant")
    return out
