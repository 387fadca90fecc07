"""Thin ctypes binding over libhbitlinear.so (include/hbitlinear.h).

Argument marshalling only: every step of the path runs in the library's HIP
kernels.  PyTorch provides device memory (``tensor.data_ptr()``) and the
current stream; nothing here computes.  If the shared library is missing the
import of any function fails loudly - there is no CPU fallback.

bf16 activations / outputs are ``torch.bfloat16`` tensors; fp32 activations
``torch.float32``.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libhbitlinear.so")

OK = 0
E_NULL, E_SHAPE, E_BITS, E_DTYPE, E_WORKSPACE, E_HIP, E_ALIGN, E_SCRATCH = -1, -2, -3, -4, -5, -6, -7, -8
F32, BF16 = 0, 1
CODES_INT8, CODES_UINT4_PLUS8, CODES_BF6 = 0, 8, 6
EPS = 1e-5

EXPORTS = [
    "hbl_strerror", "hbl_last_hip_error", "hbl_ternarize_workspace_bytes", "hbl_ternarize_weights_absmean",
    "hbl_packed_bytes", "hbl_pack_ternary_2bit", "hbl_unpack_ternary_2bit", "hbl_workspace_bytes",
    "hbl_hbitlinear_forward", "hbl_plain_bitlinear_forward", "hbl_fwht_quant", "hbl_gemm_i32",
    "hbl_gemm_dequant_bf16", "hbl_grouped_workspace_bytes", "hbl_bitlinear_forward_grouped", "hbl_fwht",
    "hbl_ln_bitlinear_forward", "hbl_ln_fwht_quant", "hbl_gemm_i32_bf6",
    "hbl_kv_packed_bytes", "hbl_kv_quant_absmax", "hbl_kv_dequant", "hbl_trace_begin", "hbl_trace_end",
    "hbl_code_bytes", "hbl_bitlinear_forward_small",
]
# exports for the test suite only (csrc/hbl_test_exports.h)
TEST_EXPORTS = ["hbl_test_grouped_plan", "hbl_test_gemm_i32_tile"]
TILE_SQUARE, TILE_SMALL, TILE_WIDE, TILE_SPLIT_K = 0, 1, 2, 3

_lib = None


class Problem(ctypes.Structure):
    """``hbl_problem`` of include/hbitlinear.h."""
    _fields_ = [("x", ctypes.c_void_p), ("x_dtype", ctypes.c_int), ("bits", ctypes.c_int),
                ("hadamard", ctypes.c_int), ("reserved", ctypes.c_int), ("T", ctypes.c_int64),
                ("K", ctypes.c_int64), ("N", ctypes.c_int64), ("Wq_packed", ctypes.c_void_p),
                ("w_scales", ctypes.c_void_p), ("n_scale_groups", ctypes.c_int64), ("y", ctypes.c_void_p),
                ("ln_gain", ctypes.c_void_p), ("ln_eps", ctypes.c_float)]


class HblError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        msg = lib().hbl_strerror(status).decode()
        if status == E_HIP:
            msg += f" (hipError {lib().hbl_last_hip_error()})"
        super().__init__(f"{what}: {msg} [status {status}]")


def lib():
    """Load the C-ABI library (built by ``__graft_entry__.build()`` / ``paper_2504_18415_amd.build``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2504_18415_amd.build` "
                "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        i64, ci, f32, vp, sz = ctypes.c_int64, ctypes.c_int, ctypes.c_float, ctypes.c_void_p, ctypes.c_size_t
        L.hbl_strerror.restype = ctypes.c_char_p
        L.hbl_strerror.argtypes = [ci]
        L.hbl_last_hip_error.restype = ci
        L.hbl_ternarize_workspace_bytes.restype = sz
        L.hbl_ternarize_workspace_bytes.argtypes = [i64, i64]
        L.hbl_ternarize_weights_absmean.argtypes = [vp, i64, i64, f32, vp, vp, vp, sz, vp]
        L.hbl_packed_bytes.restype = sz
        L.hbl_packed_bytes.argtypes = [i64, i64]
        L.hbl_pack_ternary_2bit.argtypes = [vp, i64, i64, vp, vp]
        L.hbl_unpack_ternary_2bit.argtypes = [vp, i64, i64, vp, vp]
        L.hbl_workspace_bytes.restype = sz
        L.hbl_workspace_bytes.argtypes = [i64, i64, i64, ci]
        fwd = [vp, ci, i64, i64, vp, i64, vp, i64, ci, f32, vp, vp, sz, vp]
        L.hbl_hbitlinear_forward.argtypes = fwd
        L.hbl_plain_bitlinear_forward.argtypes = fwd
        L.hbl_fwht_quant.argtypes = [vp, ci, i64, i64, ci, f32, ci, ci, vp, vp, vp, vp]
        L.hbl_gemm_i32.argtypes = [vp, i64, i64, vp, i64, vp, vp]
        L.hbl_gemm_dequant_bf16.argtypes = [vp, ci, vp, vp, i64, i64, vp, i64, vp, i64, vp, vp]
        L.hbl_fwht.argtypes = [vp, ci, i64, i64, vp, ci, vp]
        L.hbl_kv_packed_bytes.argtypes = [i64, i64, ci]
        L.hbl_kv_packed_bytes.restype = ctypes.c_size_t
        L.hbl_kv_quant_absmax.argtypes = [vp, ci, i64, i64, ci, ctypes.c_float, vp, vp, vp]
        L.hbl_kv_dequant.argtypes = [vp, vp, i64, i64, ci, vp, ci, vp]
        ip = ctypes.POINTER(ci)
        L.hbl_test_grouped_plan.argtypes = [ctypes.POINTER(Problem), ci, ip, ip, ip, ip]
        L.hbl_test_gemm_i32_tile.argtypes = [vp, ci, i64, i64, vp, i64, vp, ci, vp, sz, vp]
        L.hbl_gemm_i32_bf6.argtypes = [vp, i64, i64, vp, i64, vp, vp, sz, vp]
        L.hbl_bitlinear_forward_small.argtypes = [vp, ci, i64, i64, vp, i64, vp, i64, ci, f32, ci, vp, vp]
        L.hbl_code_bytes.restype = sz
        L.hbl_code_bytes.argtypes = [i64, i64, ci]
        L.hbl_trace_begin.argtypes = [ci]
        L.hbl_trace_end.argtypes = [ctypes.POINTER(f32), ctypes.POINTER(ctypes.c_char_p), ci, ip]
        L.hbl_ln_bitlinear_forward.argtypes = [vp, ci, i64, i64, vp, f32, ci, vp, i64, vp, i64, ci, f32, vp, vp, sz, vp]
        L.hbl_ln_fwht_quant.argtypes = [vp, ci, i64, i64, vp, f32, ci, f32, ci, ci, vp, vp, vp, vp]
        L.hbl_grouped_workspace_bytes.restype = sz
        L.hbl_grouped_workspace_bytes.argtypes = [ctypes.POINTER(Problem), ci]
        L.hbl_bitlinear_forward_grouped.argtypes = [ctypes.POINTER(Problem), ci, f32, vp, sz, vp]
        _lib = L
    return _lib


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else t.data_ptr()


def _check(status: int, what: str):
    if status != OK:
        raise HblError(status, what)


def _x_dtype(x: torch.Tensor) -> int:
    if x.dtype == torch.bfloat16:
        return BF16
    if x.dtype == torch.float32:
        return F32
    raise TypeError("activations must be torch.bfloat16 or torch.float32")


def _dev_check(*ts):
    for t in ts:
        if t is not None and (not t.is_cuda or not t.is_contiguous()):
            raise ValueError("tensors must be contiguous device tensors")


def _check_projection(T, K, N, Wq_packed, w_scales, y, workspace=None):
    """Sizes and dtypes the kernels rely on and cannot see through raw pointers: a short packed buffer or
    output would make them read or write out of bounds on the device."""
    if N <= 0 or K <= 0:
        raise ValueError(f"N and K must be positive (N={N}, K={K})")
    if Wq_packed.dtype != torch.uint8 or Wq_packed.numel() < packed_bytes(N, K):
        raise ValueError(f"Wq_packed must be uint8 with at least packed_bytes({N}, {K}) = {packed_bytes(N, K)} "
                         f"elements (got {Wq_packed.dtype}, {Wq_packed.numel()})")
    if w_scales.dtype != torch.float32 or w_scales.numel() < 1:
        raise ValueError("w_scales must be a non-empty float32 tensor")
    if y is not None and (y.dtype != torch.bfloat16 or tuple(y.shape) != (T, N)):
        raise ValueError(f"y must be bfloat16 [{T}, {N}] (got {y.dtype} {tuple(y.shape)})")
    if workspace is not None and workspace.dtype != torch.uint8:
        raise ValueError("workspace must be a uint8 tensor")


def ternarize_weights_absmean(W: torch.Tensor, eps: float = EPS) -> Tuple[torch.Tensor, torch.Tensor]:
    """Eq. 1.  W [N,K] fp32 (device) -> (codes int8 [N,K], alpha fp32 [1]) on the device."""
    _dev_check(W)
    N, K = W.shape
    codes = torch.empty((N, K), dtype=torch.int8, device=W.device)
    alpha = torch.empty(1, dtype=torch.float32, device=W.device)
    ws = torch.empty(max(int(lib().hbl_ternarize_workspace_bytes(N, K)), 8), dtype=torch.uint8, device=W.device)
    _check(lib().hbl_ternarize_weights_absmean(_ptr(W), N, K, eps, _ptr(codes), _ptr(alpha), _ptr(ws), ws.numel(),
                                               _stream()), "ternarize_weights_absmean")
    return codes, alpha


def packed_bytes(N: int, K: int) -> int:
    return int(lib().hbl_packed_bytes(N, K))


def pack_ternary_2bit(codes: torch.Tensor) -> torch.Tensor:
    """codes int8 [N,K] in {-1,0,1} -> opaque packed uint8 [N*K/4 + 4*N] (2 bits per weight + row sums)."""
    _dev_check(codes)
    N, K = codes.shape
    packed = torch.empty(packed_bytes(N, K), dtype=torch.uint8, device=codes.device)
    _check(lib().hbl_pack_ternary_2bit(_ptr(codes), N, K, _ptr(packed), _stream()), "pack_ternary_2bit")
    return packed


def unpack_ternary_2bit(packed: torch.Tensor, N: int, K: int) -> torch.Tensor:
    _dev_check(packed)
    codes = torch.empty((N, K), dtype=torch.int8, device=packed.device)
    _check(lib().hbl_unpack_ternary_2bit(_ptr(packed), N, K, _ptr(codes), _stream()), "unpack_ternary_2bit")
    return codes


def workspace_bytes(T: int, K: int, N: int, bits: int) -> int:
    return int(lib().hbl_workspace_bytes(T, K, N, bits))


def alloc_workspace(T: int, K: int, N: int, bits: int, device="cuda") -> torch.Tensor:
    return torch.empty(workspace_bytes(T, K, N, bits), dtype=torch.uint8, device=device)


def _forward(fn, name, x, Wq_packed, N, w_scales, bits, eps, y, workspace):
    _dev_check(x, Wq_packed, w_scales, y, workspace)
    T, K = x.shape
    _check_projection(T, K, N, Wq_packed, w_scales, y, workspace)
    if y is None:
        y = torch.empty((T, N), dtype=torch.bfloat16, device=x.device)
    if workspace is None:
        workspace = alloc_workspace(T, K, N, bits, x.device)
    _check(fn(_ptr(x), _x_dtype(x), T, K, _ptr(Wq_packed), N, _ptr(w_scales), w_scales.numel(), bits, eps,
              _ptr(y), _ptr(workspace), workspace.numel(), _stream()), name)
    return y


def hbitlinear_forward(x: torch.Tensor, Wq_packed: torch.Tensor, N: int, w_scales: torch.Tensor, bits: int = 4,
                       eps: float = EPS, y: Optional[torch.Tensor] = None,
                       workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Eq. 7 with the Hadamard transform: x [T,K] -> y bf16 [T,N]."""
    return _forward(lib().hbl_hbitlinear_forward, "hbitlinear_forward", x, Wq_packed, N, w_scales, bits, eps, y,
                    workspace)


def plain_bitlinear_forward(x: torch.Tensor, Wq_packed: torch.Tensor, N: int, w_scales: torch.Tensor, bits: int = 4,
                            eps: float = EPS, y: Optional[torch.Tensor] = None,
                            workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Eq. 7 without the transform (W_qkv, W_up/gate)."""
    return _forward(lib().hbl_plain_bitlinear_forward, "plain_bitlinear_forward", x, Wq_packed, N, w_scales, bits,
                    eps, y, workspace)


def code_bytes(T: int, K: int, code_form: int) -> int:
    return int(lib().hbl_code_bytes(T, K, code_form))


def bitlinear_forward_small(x: torch.Tensor, Wq_packed: torch.Tensor, N: int, w_scales: torch.Tensor, y: torch.Tensor,
                            bits: int = 4, hadamard: bool = True, eps: float = EPS) -> torch.Tensor:
    """The forward call that allocates nothing (T <= 64; intermediates in the library's static device scratch).
    ``y`` bf16 [T,N] is the caller's; calls that may overlap on one GPU race."""
    _dev_check(x, Wq_packed, w_scales, y)
    T, K = x.shape
    _check_projection(T, K, N, Wq_packed, w_scales, y)
    _check(lib().hbl_bitlinear_forward_small(_ptr(x), _x_dtype(x), T, K, _ptr(Wq_packed), N, _ptr(w_scales),
                                             w_scales.numel(), bits, eps, int(bool(hadamard)), _ptr(y), _stream()),
           "bitlinear_forward_small")
    return y


def _alloc_codes(T: int, K: int, code_form: int, device) -> torch.Tensor:
    """Byte forms: int8 [T, K].  Record form: the flat record image (0.75 byte per code, whole 128-token panels)."""
    if code_form == CODES_BF6:
        return torch.empty(code_bytes(T, K, CODES_BF6), dtype=torch.int8, device=device)
    return torch.empty((T, K), dtype=torch.int8, device=device)


def fwht_quant(x: torch.Tensor, bits: int, hadamard: bool = True, eps: float = EPS, code_offset: int = 0):
    """Eq. 3-6 only -> (codes, s_dequant fp32 [T], code_sum int32 [T]); codes int8 [T,K] stored as
    code+code_offset, or for ``CODES_BF6`` the flat record image of ``code_bytes(T, K, CODES_BF6)`` bytes."""
    _dev_check(x)
    T, K = x.shape
    codes = _alloc_codes(T, K, code_offset, x.device)
    sd = torch.empty(T, dtype=torch.float32, device=x.device)
    cs = torch.empty(T, dtype=torch.int32, device=x.device)
    _check(lib().hbl_fwht_quant(_ptr(x), _x_dtype(x), T, K, bits, eps, int(hadamard), code_offset, _ptr(codes),
                                _ptr(sd), _ptr(cs), _stream()), "fwht_quant")
    return codes, sd, cs


def gemm_i32(codes: torch.Tensor, Wq_packed: torch.Tensor, N: int) -> torch.Tensor:
    """acc int32 [T,N] = codes [T,K] . c^T (exact)."""
    _dev_check(codes, Wq_packed)
    T, K = codes.shape
    _check_projection(T, K, N, Wq_packed, torch.empty(1), None)
    acc = torch.empty((T, N), dtype=torch.int32, device=codes.device)
    _check(lib().hbl_gemm_i32(_ptr(codes), T, K, _ptr(Wq_packed), N, _ptr(acc), _stream()), "gemm_i32")
    return acc


def _check_records(records: torch.Tensor, T: int, K: int):
    if records.element_size() != 1 or records.numel() < code_bytes(T, K, CODES_BF6) or code_bytes(T, K, CODES_BF6) == 0:
        raise ValueError(f"code records for [{T}, {K}] need {code_bytes(T, K, CODES_BF6)} bytes (got {records.numel()})")


def gemm_i32_bf6(records: torch.Tensor, Wq_packed: torch.Tensor, N: int, T: int, K: int,
                 workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """acc int32 [T,N] from the record image of [T,K] codes on the fp6 x fp4 kernel, in the forward call's own
    launch configuration for the shape (exact integers read out of its fp32 accumulators)."""
    _dev_check(records, Wq_packed, workspace)
    _check_records(records, T, K)
    _check_projection(T, K, N, Wq_packed, torch.empty(1), None, workspace)
    acc = torch.empty((T, N), dtype=torch.int32, device=records.device)
    if workspace is None:
        workspace = alloc_workspace(T, K, N, 4, records.device)
    _check(lib().hbl_gemm_i32_bf6(_ptr(records), T, K, _ptr(Wq_packed), N, _ptr(acc), _ptr(workspace),
                                  workspace.numel(), _stream()), "gemm_i32_bf6")
    return acc


def gemm_i32_tile_for_tests(codes: torch.Tensor, code_form: int, Wq_packed: torch.Tensor, N: int, tile: int,
                            T: Optional[int] = None, K: Optional[int] = None) -> torch.Tensor:
    """Test-suite export: the integer contraction through one named workgroup tile (TILE_*) of the int8
    (``CODES_INT8``, codes [T,K]) or fp6 x fp4 (``CODES_BF6``, record image; pass T and K) prefill kernel."""
    _dev_check(codes, Wq_packed)
    if code_form == CODES_BF6:
        _check_records(codes, T, K)
    else:
        T, K = codes.shape
    _check_projection(T, K, N, Wq_packed, torch.empty(1), None)
    acc = torch.empty((T, N), dtype=torch.int32, device=codes.device)
    partial = torch.empty(8 * T * N * 4 if tile == TILE_SPLIT_K else 16, dtype=torch.uint8, device=codes.device)
    _check(lib().hbl_test_gemm_i32_tile(_ptr(codes), code_form, T, K, _ptr(Wq_packed), N, _ptr(acc), tile,
                                        _ptr(partial), partial.numel(), _stream()), "test_gemm_i32_tile")
    return acc


class trace:
    """``with hbl.trace(n) as tr: ...`` - per-launch kernel durations of the library calls made inside the
    block (hbl_trace_begin / hbl_trace_end).  Afterwards ``tr.launches`` is a list of (kernel name, ms) in
    launch order and ``tr.seen`` the number of launches (those beyond ``n`` are not timed)."""

    def __init__(self, max_launches: int):
        self.n = int(max_launches)
        self.launches, self.seen = [], 0

    def __enter__(self):
        _check(lib().hbl_trace_begin(self.n), "trace_begin")
        return self

    def __exit__(self, *exc):
        ms = (ctypes.c_float * self.n)()
        names = (ctypes.c_char_p * self.n)()
        seen = ctypes.c_int(0)
        _check(lib().hbl_trace_end(ms, names, self.n, ctypes.byref(seen)), "trace_end")
        self.seen = seen.value
        k = min(self.seen, self.n)
        self.launches = [((names[i] or b"?").decode(), float(ms[i])) for i in range(k)]
        return False

    def mean_ms(self, kernel: str) -> float:
        v = [ms for name, ms in self.launches if name == kernel]
        return sum(v) / len(v) if v else float("nan")


def gemm_dequant_bf16(codes: torch.Tensor, s_dequant: torch.Tensor, code_sum: torch.Tensor, Wq_packed: torch.Tensor,
                      N: int, w_scales: torch.Tensor, y: Optional[torch.Tensor] = None,
                      code_offset: int = 0, K: Optional[int] = None) -> torch.Tensor:
    """Second launch of the forward on caller-held intermediates: y bf16 [T,N].  With ``CODES_BF6`` the codes are
    the flat record image and K must be given (T is the length of ``s_dequant``)."""
    _dev_check(codes, s_dequant, code_sum, Wq_packed, w_scales, y)
    if code_offset == CODES_BF6:
        T = s_dequant.numel()
        _check_records(codes, T, K)
    else:
        T, K = codes.shape
    _check_projection(T, K, N, Wq_packed, w_scales, y)
    if (s_dequant.dtype != torch.float32 or s_dequant.numel() < T or code_sum.dtype != torch.int32
            or code_sum.numel() < T):
        raise ValueError("s_dequant must be float32 [T] and code_sum int32 [T]")
    if y is None:
        y = torch.empty((T, N), dtype=torch.bfloat16, device=codes.device)
    _check(lib().hbl_gemm_dequant_bf16(_ptr(codes), code_offset, _ptr(s_dequant), _ptr(code_sum), T, K, _ptr(Wq_packed), N,
                                       _ptr(w_scales), w_scales.numel(), _ptr(y), _stream()), "gemm_dequant_bf16")
    return y


def fwht_quant_into(x: torch.Tensor, bits: int, hadamard: bool, codes: torch.Tensor, s_dequant: torch.Tensor,
                    code_sum: torch.Tensor, eps: float = EPS, code_offset: int = 0) -> None:
    """hbl_fwht_quant into caller-held buffers (no allocation)."""
    T, K = x.shape
    _check(lib().hbl_fwht_quant(_ptr(x), _x_dtype(x), T, K, bits, eps, int(hadamard), code_offset, _ptr(codes),
                                _ptr(s_dequant), _ptr(code_sum), _stream()), "fwht_quant")


def make_problems(items) -> "ctypes.Array":
    """items: iterable of (x, Wq_packed, N, w_scales, bits, hadamard, y[, ln_gain, ln_eps]) -> ``hbl_problem`` array."""
    items = list(items)
    arr = (Problem * max(len(items), 1))()
    for i, it in enumerate(items):
        x, Wq_packed, N, w_scales, bits, hadamard, y = it[:7]
        ln_gain, ln_eps = (it[7], it[8]) if len(it) > 7 else (None, 0.0)
        _dev_check(x, Wq_packed, w_scales, y, ln_gain)
        T, K = x.shape
        _check_projection(T, K, N, Wq_packed, w_scales, y)
        if ln_gain is not None and (ln_gain.dtype != torch.float32 or ln_gain.numel() != K):
            raise ValueError("ln_gain must be float32 [K]")
        arr[i] = Problem(_ptr(x), _x_dtype(x), bits, int(bool(hadamard)), 0, T, K, N, _ptr(Wq_packed),
                         _ptr(w_scales), w_scales.numel(), _ptr(y), _ptr(ln_gain), ln_eps)
    return arr


def grouped_workspace_bytes(problems, n: int) -> int:
    return int(lib().hbl_grouped_workspace_bytes(problems, n))


def bitlinear_forward_grouped(items, eps: float = EPS, workspace: Optional[torch.Tensor] = None,
                              problems=None):
    """Several independent projections in one call.  ``items`` as for :func:`make_problems`, with y
    possibly None (allocated here); returns the list of y tensors.  Pass ``problems`` (from
    :func:`make_problems`) and ``workspace`` to call again without marshalling or allocation."""
    items = [list(it) for it in items]
    for it in items:
        if it[6] is None:
            it[6] = torch.empty((it[0].shape[0], it[2]), dtype=torch.bfloat16, device=it[0].device)
    if problems is None:
        problems = make_problems(items)
    n = len(items)
    if workspace is None:
        workspace = torch.empty(grouped_workspace_bytes(problems, n), dtype=torch.uint8, device="cuda")
    _check(lib().hbl_bitlinear_forward_grouped(problems, n, eps, _ptr(workspace), workspace.numel(), _stream()),
           "bitlinear_forward_grouped")
    return [it[6] for it in items]


def fwht(x: torch.Tensor, out_dtype: Optional[torch.dtype] = None, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Eq. 3-4 alone (and the backward pass of Eq. 8 when x holds gradient rows): Hadamard(x) row by row."""
    _dev_check(x, out)
    T, K = x.shape
    if out is None:
        out = torch.empty((T, K), dtype=out_dtype or torch.float32, device=x.device)
    _check(lib().hbl_fwht(_ptr(x), _x_dtype(x), T, K, _ptr(out), _x_dtype(out), _stream()), "fwht")
    return out


def ln_bitlinear_forward(x: torch.Tensor, ln_gain: torch.Tensor, ln_eps: float, hadamard: bool,
                         Wq_packed: torch.Tensor, N: int, w_scales: torch.Tensor, bits: int = 4, eps: float = EPS,
                         y: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Eq. 7 with its LN (RMS normalisation with gain ``ln_gain`` [K] fp32) fused into the quantiser launch."""
    _dev_check(x, ln_gain, Wq_packed, w_scales, y, workspace)
    T, K = x.shape
    _check_projection(T, K, N, Wq_packed, w_scales, y, workspace)
    if ln_gain.dtype != torch.float32 or ln_gain.numel() != K:
        raise ValueError("ln_gain must be float32 [K]")
    if y is None:
        y = torch.empty((T, N), dtype=torch.bfloat16, device=x.device)
    if workspace is None:
        workspace = alloc_workspace(T, K, N, bits, x.device)
    _check(lib().hbl_ln_bitlinear_forward(_ptr(x), _x_dtype(x), T, K, _ptr(ln_gain), ln_eps, int(bool(hadamard)),
                                          _ptr(Wq_packed), N, _ptr(w_scales), w_scales.numel(), bits, eps, _ptr(y),
                                          _ptr(workspace), workspace.numel(), _stream()), "ln_bitlinear_forward")
    return y


def ln_fwht_quant(x: torch.Tensor, ln_gain: torch.Tensor, ln_eps: float, bits: int, hadamard: bool = True,
                  eps: float = EPS, code_offset: int = 0):
    """RMS normalisation + Eq. 3-6 -> (codes, s_dequant, code_sum) as :func:`fwht_quant`."""
    _dev_check(x, ln_gain)
    T, K = x.shape
    codes = _alloc_codes(T, K, code_offset, x.device)
    sd = torch.empty(T, dtype=torch.float32, device=x.device)
    cs = torch.empty(T, dtype=torch.int32, device=x.device)
    _check(lib().hbl_ln_fwht_quant(_ptr(x), _x_dtype(x), T, K, _ptr(ln_gain), ln_eps, bits, eps, int(hadamard),
                                   code_offset, _ptr(codes), _ptr(sd), _ptr(cs), _stream()), "ln_fwht_quant")
    return codes, sd, cs


def grouped_plan(shapes):
    """Host-only: launch plan of the small-batch GEMM for [(T, K, N, hadamard), ...] ->
    (ksplit list, gemm workgroups, arrival counters = groups of four row tiles whose K range is split over
    workgroups and reduced by the last of them, list of "single call streams" flags)."""
    n = len(shapes)
    arr = (Problem * n)(*[Problem(0, BF16, 4, int(bool(h)), 0, T, K, N, 0, 0, 1, 0) for (T, K, N, h) in shapes])
    ks = (ctypes.c_int * n)()
    st = (ctypes.c_int * n)()
    wgs, counters = ctypes.c_int(0), ctypes.c_int(0)
    _check(lib().hbl_test_grouped_plan(arr, n, ks, ctypes.byref(wgs), ctypes.byref(counters), st), "grouped_plan")
    return list(ks), wgs.value, counters.value, [bool(v) for v in st]


def kv_quant_absmax(x: torch.Tensor, bits: int, eps: float = EPS, packed: Optional[torch.Tensor] = None,
                    scales: Optional[torch.Tensor] = None):
    """Low-bit head states (Section 3.1, Main Results): x [rows, d] -> (packed uint8 [rows, d*bits/8], scales fp32 [rows])."""
    _dev_check(x)
    rows, d = x.shape
    nbytes = lib().hbl_kv_packed_bytes(rows, d, bits)
    if packed is None:
        packed = torch.empty((rows, d * bits // 8) if nbytes or rows == 0 else (0,), dtype=torch.uint8, device=x.device)
    if scales is None:
        scales = torch.empty(rows, dtype=torch.float32, device=x.device)
    _check(lib().hbl_kv_quant_absmax(_ptr(x), _x_dtype(x), rows, d, bits, eps, _ptr(packed), _ptr(scales), _stream()),
           "kv_quant_absmax")
    return packed, scales


def kv_dequant(packed: torch.Tensor, scales: torch.Tensor, d: int, bits: int, out_dtype=torch.bfloat16,
               out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Inverse map of :func:`kv_quant_absmax`: -> [rows, d] bf16 or fp32."""
    _dev_check(packed, scales)
    rows = scales.shape[0]
    if out is None:
        out = torch.empty((rows, d), dtype=out_dtype, device=packed.device)
    _check(lib().hbl_kv_dequant(_ptr(packed), _ptr(scales), rows, d, bits, _ptr(out),
                                BF16 if out.dtype == torch.bfloat16 else F32, _stream()), "kv_dequant")
    return out
