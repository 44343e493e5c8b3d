"""ctypes binding over the C ABI declared in include/asi.h.

Argument marshalling only: every step of the path runs in the HIP kernels of
libasi_hip.so.  torch is used for device memory and the current stream.  There
is no CPU fallback: a missing library raises at import of the first call.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import torch

from .build import LIB_PATH

ASI_OK = 0
STATUS_NAMES = {0: "ASI_OK", 1: "ASI_ERR_INVALID_ARG", 2: "ASI_ERR_UNSUPPORTED",
                3: "ASI_ERR_WORKSPACE", 4: "ASI_ERR_HIP", 5: "ASI_ERR_NUMERIC", 6: "ASI_ERR_INFEASIBLE"}
ASI_F32, ASI_BF16 = 0, 1

STATIC_SCRATCH_BYTES = 16 << 20      # ASI_STATIC_SCRATCH_BYTES of include/asi.h

EXPORTS = ["asi_workspace_bytes", "asi_compress", "asi_compress_cold", "asi_cold_start_matrix", "asi_compress_static", "asi_core_project", "asi_weight_grad_conv2d",
           "asi_weight_grad_linear", "asi_compress_batch", "asi_core_project_batch",
           "asi_weight_grad_conv2d_batch", "asi_weight_grad_linear_batch", "asi_status_string", "asi_version",
           "asi_profile_enable", "asi_profile_report", "asi_activation_memory", "asi_mode_spectrum_workspace_bytes",
           "asi_mode_spectrum", "asi_explained_variance_ranks", "asi_frobenius_diff", "asi_rank_select"]
FROBENIUS_WS_BYTES = 8192            # ASI_FROBENIUS_WS_BYTES of include/asi.h
MAX_BATCH = 8


class TensorDesc(C.Structure):
    _fields_ = [("ndim", C.c_int32), ("dims", C.c_int64 * 4), ("ranks", C.c_int32 * 4), ("dtype", C.c_int32)]


class Conv2dDesc(C.Structure):
    _fields_ = [("cout", C.c_int64), ("kh", C.c_int32), ("kw", C.c_int32),
                ("stride_h", C.c_int32), ("stride_w", C.c_int32), ("pad_h", C.c_int32), ("pad_w", C.c_int32),
                ("dil_h", C.c_int32), ("dil_w", C.c_int32), ("groups", C.c_int32)]


class AsiError(RuntimeError):
    def __init__(self, status: int, where: str):
        super().__init__(f"{where}: {STATUS_NAMES.get(status, status)}")
        self.status = status


_lib = None


def lib() -> C.CDLL:
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is not built; run `python -m paper_2505_05086_amd.build` "
                               "(the ASI path has no CPU fallback)")
        L = C.CDLL(LIB_PATH)
        pp = C.POINTER(C.c_void_p)
        L.asi_workspace_bytes.restype = C.c_size_t
        L.asi_workspace_bytes.argtypes = [C.POINTER(TensorDesc), C.POINTER(Conv2dDesc), C.c_int64]
        L.asi_compress.restype = C.c_int
        L.asi_compress.argtypes = [C.POINTER(TensorDesc), C.c_void_p, pp, pp, C.c_void_p, C.c_size_t,
                                   C.c_void_p, C.c_void_p]
        L.asi_compress_cold.restype = C.c_int
        L.asi_compress_cold.argtypes = [C.POINTER(TensorDesc), C.c_void_p, C.c_uint64, pp, C.c_void_p, C.c_size_t,
                                        C.c_void_p, C.c_void_p]
        L.asi_cold_start_matrix.restype = C.c_int
        L.asi_cold_start_matrix.argtypes = [C.POINTER(TensorDesc), C.c_int32, C.c_uint64, C.c_void_p, C.c_void_p]
        L.asi_compress_static.restype = C.c_int
        L.asi_compress_static.argtypes = [C.POINTER(TensorDesc), C.c_void_p, pp, pp, C.c_void_p, C.c_void_p]
        L.asi_core_project.restype = C.c_int
        L.asi_core_project.argtypes = [C.POINTER(TensorDesc), C.c_void_p, pp, C.c_void_p, C.c_void_p,
                                       C.c_size_t, C.c_void_p]
        L.asi_weight_grad_conv2d.restype = C.c_int
        L.asi_weight_grad_conv2d.argtypes = [C.POINTER(TensorDesc), C.c_void_p, pp, C.c_void_p,
                                             C.POINTER(Conv2dDesc), C.c_void_p, C.c_int, C.c_void_p,
                                             C.c_size_t, C.c_void_p]
        L.asi_weight_grad_linear.restype = C.c_int
        L.asi_weight_grad_linear.argtypes = [C.POINTER(TensorDesc), C.c_void_p, pp, C.c_void_p, C.c_int64,
                                             C.c_void_p, C.c_int, C.c_void_p, C.c_size_t, C.c_void_p]
        vp = C.c_void_p
        L.asi_compress_batch.restype = C.c_int
        L.asi_compress_batch.argtypes = [C.c_int32, vp, vp, vp, vp, vp, vp, vp, vp]
        L.asi_core_project_batch.restype = C.c_int
        L.asi_core_project_batch.argtypes = [C.c_int32, vp, vp, vp, vp, vp, vp, vp]
        L.asi_weight_grad_conv2d_batch.restype = C.c_int
        L.asi_weight_grad_conv2d_batch.argtypes = [C.c_int32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.asi_weight_grad_linear_batch.restype = C.c_int
        L.asi_weight_grad_linear_batch.argtypes = [C.c_int32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.asi_status_string.restype = C.c_char_p
        L.asi_status_string.argtypes = [C.c_int]
        L.asi_version.restype = C.c_int32
        L.asi_version.argtypes = []
        L.asi_profile_enable.restype = C.c_int32
        L.asi_profile_enable.argtypes = [C.c_int32]
        L.asi_profile_report.restype = C.c_int64
        L.asi_profile_report.argtypes = [C.c_char_p, C.c_int64]
        L.asi_activation_memory.restype = C.c_int64
        L.asi_activation_memory.argtypes = [C.POINTER(TensorDesc)]
        L.asi_mode_spectrum_workspace_bytes.restype = C.c_size_t
        L.asi_mode_spectrum_workspace_bytes.argtypes = [C.POINTER(TensorDesc), C.c_int32]
        L.asi_mode_spectrum.restype = C.c_int
        L.asi_mode_spectrum.argtypes = [C.POINTER(TensorDesc), vp, C.c_int32, vp, vp, vp, C.c_size_t,
                                        C.POINTER(C.c_int32), vp]
        L.asi_explained_variance_ranks.restype = C.c_int
        L.asi_explained_variance_ranks.argtypes = [vp, C.c_int32, C.POINTER(C.c_double), C.c_int32, vp, vp]
        L.asi_frobenius_diff.restype = C.c_int
        L.asi_frobenius_diff.argtypes = [vp, vp, C.c_int64, vp, vp, C.c_size_t, vp]
        L.asi_rank_select.restype = C.c_int
        L.asi_rank_select.argtypes = [C.c_int32, C.c_int32, C.POINTER(C.c_double), C.POINTER(C.c_int64), C.c_int64,
                                      C.POINTER(C.c_int32), C.POINTER(C.c_double)]
        _lib = L
    return _lib


def make_desc(dims: Sequence[int], ranks: Sequence[int], dtype: str = "f32") -> TensorDesc:
    d = TensorDesc()
    d.ndim = len(dims)
    for i in range(4):
        d.dims[i] = int(dims[i]) if i < len(dims) else 0
        d.ranks[i] = int(ranks[i]) if i < len(ranks) else 0
    d.dtype = {"f32": ASI_F32, "bf16": ASI_BF16}.get(dtype, 99) if isinstance(dtype, str) else int(dtype)
    return d


def make_conv(cout, kh, kw, stride=(1, 1), pad=(0, 0), dil=(1, 1), groups=1) -> Conv2dDesc:
    c = Conv2dDesc()
    c.cout, c.kh, c.kw = int(cout), int(kh), int(kw)
    c.stride_h, c.stride_w = int(stride[0]), int(stride[1])
    c.pad_h, c.pad_w = int(pad[0]), int(pad[1])
    c.dil_h, c.dil_w = int(dil[0]), int(dil[1])
    c.groups = int(groups)
    return c


def _ptr(t: Optional[torch.Tensor]) -> C.c_void_p:
    return C.c_void_p(0 if t is None else t.data_ptr())


def _ptr_array(ts: Sequence[torch.Tensor]):
    arr = (C.c_void_p * 4)()
    for i in range(4):
        arr[i] = ts[i].data_ptr() if i < len(ts) and ts[i] is not None else None
    return arr


def _stream() -> C.c_void_p:
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check_dev(*ts):
    for t in ts:
        if t is None:
            continue
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError("ASI binding needs contiguous device tensors")


def _check(status: int, where: str):
    if status != ASI_OK:
        raise AsiError(status, where)


def asi_workspace_bytes(desc: TensorDesc, conv: Optional[Conv2dDesc] = None, dout: int = 0) -> int:
    return int(lib().asi_workspace_bytes(C.byref(desc), C.byref(conv) if conv is not None else None, int(dout)))


def alloc_workspace(desc: TensorDesc, conv: Optional[Conv2dDesc] = None, dout: int = 0,
                    device="cuda") -> torch.Tensor:
    n = asi_workspace_bytes(desc, conv, dout)
    if n == 0:
        raise AsiError(1, "asi_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def asi_compress(desc: TensorDesc, A: torch.Tensor, U_prev: Sequence[torch.Tensor],
                 U_out: Sequence[torch.Tensor], ws: torch.Tensor, info: Optional[torch.Tensor] = None) -> None:
    _check_dev(A, ws, info, *U_prev, *U_out)
    _check(lib().asi_compress(C.byref(desc), _ptr(A), _ptr_array(U_prev), _ptr_array(U_out), _ptr(ws),
                              ws.numel(), _ptr(info), _stream()), "asi_compress")


def asi_compress_cold(desc: TensorDesc, A: torch.Tensor, seed: int, U_out: Sequence[torch.Tensor], ws: torch.Tensor,
                      info: Optional[torch.Tensor] = None) -> None:
    """Alg. 1's first iteration: V drawn from the counter-based generator keyed by `seed`."""
    _check_dev(A, ws, info, *U_out)
    _check(lib().asi_compress_cold(C.byref(desc), _ptr(A), int(seed) & (2 ** 64 - 1), _ptr_array(U_out), _ptr(ws),
                                   ws.numel(), _ptr(info), _stream()), "asi_compress_cold")


def asi_cold_start_matrix(desc: TensorDesc, mode: int, seed: int, V: torch.Tensor) -> None:
    """The generated V of one mode written to V (numel / dims[mode], ranks[mode]) fp32."""
    _check_dev(V)
    _check(lib().asi_cold_start_matrix(C.byref(desc), int(mode), int(seed) & (2 ** 64 - 1), _ptr(V), _stream()),
           "asi_cold_start_matrix")


def asi_compress_static(desc: TensorDesc, A: torch.Tensor, U_prev: Sequence[torch.Tensor],
                        U_out: Sequence[torch.Tensor], info: Optional[torch.Tensor] = None) -> None:
    """asi_compress on the library's static scratch array: no workspace argument, nothing allocated."""
    _check_dev(A, info, *U_prev, *U_out)
    _check(lib().asi_compress_static(C.byref(desc), _ptr(A), _ptr_array(U_prev), _ptr_array(U_out), _ptr(info),
                                     _stream()), "asi_compress_static")


def asi_core_project(desc: TensorDesc, A: torch.Tensor, U: Sequence[torch.Tensor], S: torch.Tensor,
                     ws: torch.Tensor) -> None:
    _check_dev(A, ws, S, *U)
    _check(lib().asi_core_project(C.byref(desc), _ptr(A), _ptr_array(U), _ptr(S), _ptr(ws), ws.numel(),
                                  _stream()), "asi_core_project")


def asi_weight_grad_conv2d(desc: TensorDesc, S: torch.Tensor, U: Sequence[torch.Tensor], grad_out: torch.Tensor,
                           conv: Conv2dDesc, dW: torch.Tensor, accumulate: bool, ws: torch.Tensor) -> None:
    _check_dev(S, grad_out, dW, ws, *U)
    _check(lib().asi_weight_grad_conv2d(C.byref(desc), _ptr(S), _ptr_array(U), _ptr(grad_out), C.byref(conv),
                                        _ptr(dW), int(bool(accumulate)), _ptr(ws), ws.numel(), _stream()),
           "asi_weight_grad_conv2d")


def asi_weight_grad_linear(desc: TensorDesc, S: torch.Tensor, U: Sequence[torch.Tensor], grad_out: torch.Tensor,
                           dout: int, dW: torch.Tensor, accumulate: bool, ws: torch.Tensor) -> None:
    _check_dev(S, grad_out, dW, ws, *U)
    _check(lib().asi_weight_grad_linear(C.byref(desc), _ptr(S), _ptr_array(U), _ptr(grad_out), int(dout),
                                        _ptr(dW), int(bool(accumulate)), _ptr(ws), ws.numel(), _stream()),
           "asi_weight_grad_linear")


# ---- batched forms: host arrays of per-layer arguments ---------------------------------------
def _desc_array(descs: Sequence[TensorDesc]):
    arr = (TensorDesc * len(descs))()
    for i, d in enumerate(descs):
        arr[i] = d
    return arr


def _pp(ts: Sequence[Optional[torch.Tensor]]):
    """Host array of device pointers, one per layer."""
    arr = (C.c_void_p * len(ts))()
    for i, t in enumerate(ts):
        arr[i] = None if t is None else t.data_ptr()
    return arr


def _ppp(tss: Sequence[Sequence[torch.Tensor]]):
    """Host array of host arrays of device pointers (per layer, per mode); returns (outer, keepalive)."""
    inner = [_ptr_array(ts) for ts in tss]
    outer = (C.c_void_p * len(tss))()
    for i, a in enumerate(inner):
        outer[i] = C.addressof(a)
    return outer, inner


def _sizes(ws: Sequence[torch.Tensor]):
    arr = (C.c_size_t * len(ws))()
    for i, w in enumerate(ws):
        arr[i] = w.numel()
    return arr


def _ints(vals: Sequence[int], ctype):
    arr = (ctype * len(vals))()
    for i, v in enumerate(vals):
        arr[i] = int(v)
    return arr


def asi_compress_batch(descs, A, U_prev, U_out, ws, info=None) -> None:
    n = len(descs)
    for l in range(n):
        _check_dev(A[l], ws[l], None if info is None else info[l], *U_prev[l], *U_out[l])
    up, k1 = _ppp(U_prev)
    uo, k2 = _ppp(U_out)
    _check(lib().asi_compress_batch(n, _desc_array(descs), _pp(A), up, uo, _pp(ws), _sizes(ws),
                                    None if info is None else _pp(info), _stream()), "asi_compress_batch")


def asi_core_project_batch(descs, A, U, S, ws) -> None:
    n = len(descs)
    for l in range(n):
        _check_dev(A[l], ws[l], S[l], *U[l])
    u, keep = _ppp(U)
    _check(lib().asi_core_project_batch(n, _desc_array(descs), _pp(A), u, _pp(S), _pp(ws), _sizes(ws), _stream()),
           "asi_core_project_batch")


def asi_weight_grad_conv2d_batch(descs, S, U, grad_out, convs, dW, accumulate, ws) -> None:
    n = len(descs)
    for l in range(n):
        _check_dev(S[l], grad_out[l], dW[l], ws[l], *U[l])
    u, keep = _ppp(U)
    carr = (Conv2dDesc * n)()
    for i, c in enumerate(convs):
        carr[i] = c
    _check(lib().asi_weight_grad_conv2d_batch(n, _desc_array(descs), _pp(S), u, _pp(grad_out), carr, _pp(dW),
                                              _ints([int(bool(a)) for a in accumulate], C.c_int32), _pp(ws),
                                              _sizes(ws), _stream()), "asi_weight_grad_conv2d_batch")


def asi_weight_grad_linear_batch(descs, S, U, grad_out, dout, dW, accumulate, ws) -> None:
    n = len(descs)
    for l in range(n):
        _check_dev(S[l], grad_out[l], dW[l], ws[l], *U[l])
    u, keep = _ppp(U)
    _check(lib().asi_weight_grad_linear_batch(n, _desc_array(descs), _pp(S), u, _pp(grad_out),
                                              _ints(dout, C.c_int64), _pp(dW),
                                              _ints([int(bool(a)) for a in accumulate], C.c_int32), _pp(ws),
                                              _sizes(ws), _stream()), "asi_weight_grad_linear_batch")


def asi_status_string(status: int) -> str:
    return lib().asi_status_string(int(status)).decode()


def asi_version() -> int:
    return int(lib().asi_version())


def asi_activation_memory(desc: TensorDesc) -> int:
    """Eq. 5 in elements."""
    v = int(lib().asi_activation_memory(C.byref(desc)))
    if v < 0:
        raise AsiError(1, "asi_activation_memory")
    return v


def asi_mode_spectrum_workspace_bytes(desc: TensorDesc, mode: int) -> int:
    return int(lib().asi_mode_spectrum_workspace_bytes(C.byref(desc), int(mode)))


def asi_mode_spectrum(desc: TensorDesc, A: torch.Tensor, mode: int, eigenvalues: torch.Tensor,
                      eigenvectors: Optional[torch.Tensor], ws: torch.Tensor) -> int:
    """Eigenvalues (fp64, descending) and eigenvectors (fp32, columns) of A_m A_m^T.  Waits for the stream.
    Returns the number of Jacobi sweeps."""
    _check_dev(A, eigenvalues, eigenvectors, ws)
    if eigenvalues.dtype != torch.float64 or (eigenvectors is not None and eigenvectors.dtype != torch.float32):
        raise ValueError("eigenvalues are fp64, eigenvectors fp32")
    sweeps = C.c_int32(0)
    _check(lib().asi_mode_spectrum(C.byref(desc), _ptr(A), int(mode), _ptr(eigenvalues), _ptr(eigenvectors), _ptr(ws),
                                   ws.numel(), C.byref(sweeps), _stream()), "asi_mode_spectrum")
    return int(sweeps.value)


def asi_explained_variance_ranks(eigenvalues: torch.Tensor, eps: Sequence[float], ranks: torch.Tensor) -> None:
    _check_dev(eigenvalues, ranks)
    if eigenvalues.dtype != torch.float64 or ranks.dtype != torch.int32 or ranks.numel() < len(eps):
        raise ValueError("eigenvalues are fp64, ranks int32 with one entry per threshold")
    arr = (C.c_double * len(eps))(*[float(e) for e in eps])
    _check(lib().asi_explained_variance_ranks(_ptr(eigenvalues), eigenvalues.numel(), arr, len(eps), _ptr(ranks),
                                              _stream()), "asi_explained_variance_ranks")


def asi_frobenius_diff(a: torch.Tensor, b: torch.Tensor, out: torch.Tensor, ws: torch.Tensor) -> None:
    _check_dev(a, b, out, ws)
    if a.dtype != torch.float32 or b.dtype != torch.float32 or out.dtype != torch.float64 or a.numel() != b.numel():
        raise ValueError("two fp32 tensors of one size, fp64 result")
    _check(lib().asi_frobenius_diff(_ptr(a), _ptr(b), a.numel(), _ptr(out), _ptr(ws), ws.numel(), _stream()),
           "asi_frobenius_diff")


def asi_rank_select(P, M, budget: int):
    """Eq. 8-9 on host tables P, M (layers x thresholds, nested sequences).  Returns (choice per layer, total)."""
    n, e = len(P), len(P[0])
    if any(len(row) != e for row in P) or len(M) != n or any(len(row) != e for row in M):
        raise ValueError("P and M are (layers x thresholds)")
    Pa = (C.c_double * (n * e))(*[float(x) for row in P for x in row])
    Ma = (C.c_int64 * (n * e))(*[int(x) for row in M for x in row])
    choice = (C.c_int32 * n)()
    total = C.c_double(0.0)
    _check(lib().asi_rank_select(n, e, Pa, Ma, int(budget), choice, C.byref(total)), "asi_rank_select")
    return [int(c) for c in choice], float(total.value)


def asi_profile_enable(on: bool) -> bool:
    return bool(lib().asi_profile_enable(1 if on else 0))


def asi_profile_report() -> dict:
    """{site: {"launches", "ms", "bytes", "flops", "workgroups"}} for the launches recorded since enable."""
    need = int(lib().asi_profile_report(None, 0))
    if need < 0:
        raise AsiError(4, "asi_profile_report")
    buf = C.create_string_buffer(max(need, 1))
    if lib().asi_profile_report(buf, need) < 0:
        raise AsiError(4, "asi_profile_report")
    out = {}
    for line in buf.value.decode().splitlines():
        site, cnt, ms, by, fl, wg = line.rsplit(",", 5)      # the site itself may contain commas
        out[site] = {"launches": int(cnt), "ms": float(ms), "bytes": float(by), "flops": float(fl),
                     "workgroups": float(wg)}
    return out
