"""ctypes binding of liblaplex (``include/laplex.h``): same names, argument
marshalling only.  Tensors are torch tensors on the GPU (torch is used for
device memory and streams, nothing else); every step of the path runs inside
the library's kernels.  A missing or unloadable library raises; there is no
fallback of any kind.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblaplex.so")

LAPLEX_OK = 0
LAPLEX_ERR_NULL = -1
LAPLEX_ERR_SIZE = -2
LAPLEX_ERR_LD = -3
LAPLEX_ERR_WORKSPACE = -4
LAPLEX_ERR_FLAGS = -5
LAPLEX_ERR_HIP = -6
LAPLEX_ERR_ALIGN = -7
LAPLEX_ERR_VALUE = -8

LAPLEX_A_SORTED = 1
LAPLEX_B_SORTED = 2
LAPLEX_REUSE_PLAN = 4
LAPLEX_SAVE_SCANS = 8

LAPLEX_MAX_MERGED = 4294967294

EXPORTS = (
    "laplex_workspace_bytes", "laplex_apply", "laplex_apply_backward", "laplex_gram",
    "laplex_gram_backward", "laplex_get_perm", "laplex_get_plan_status", "laplex_status_string", "laplex_last_hip_error",
    "laplex_apply_static",
    "laplex_phased_workspace_bytes", "laplex_phased_apply", "laplex_phased_apply_backward",
    "laplex_apply_tau", "laplex_apply_backward_tau", "laplex_gram_tau", "laplex_gram_backward_tau",
    "laplex_wgram_workspace_bytes", "laplex_wgram",
    "laplex_mix_workspace_bytes", "laplex_mix_apply", "laplex_mix_apply_backward",
    "laplex_wgram_f64_workspace_bytes", "laplex_wgram_f64",
)

# include/laplex_diag.h: hooks for benchmarks and tests
DIAG_EXPORTS = (
    "laplex_profile_begin", "laplex_profile_end", "laplex_profile_family", "laplex_scan_tile_rows",
    "laplex_diag_move_rows", "laplex_diag_set_plan_status", "laplex_diag_set_route_min",
)
LAPLEX_STATIC_WORKSPACE_BYTES = 32 << 20

_lib = None
_P, _I, _Z, _U = ctypes.c_void_p, ctypes.c_int64, ctypes.c_size_t, ctypes.c_uint32


class LaplexError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        msg = lib().laplex_status_string(status).decode()
        if status == LAPLEX_ERR_HIP:
            msg += ": " + lib().laplex_last_hip_error().decode()
        super().__init__(f"liblaplex status {status}: {msg}")


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library (raw entry points, for tests of the error paths)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is not built; run `python -m paper_2605_24584_amd.build` "
                "(or __graft_entry__.build()).  There is no fallback path.")
        L = ctypes.CDLL(LIB_PATH)
        L.laplex_workspace_bytes.argtypes = [_I, _I, _I, ctypes.POINTER(_Z)]
        L.laplex_apply.argtypes = [_P, _I, _P, _I, _P, _I, _I, _P, _I, _P, _Z, _U, _P]
        L.laplex_apply_backward.argtypes = [_P, _I, _P, _I, _P, _I, _P, _I, _I, _P, _I, _P, _P, _P, _Z, _U, _P]
        L.laplex_gram.argtypes = [_P, _I, _P, _I, _I, _P, _I, _P, _Z, _U, _P]
        L.laplex_gram_backward.argtypes = [_P, _I, _P, _I, _P, _I, _I, _P, _I, _P, _P, _Z, _U, _P]
        L.laplex_get_perm.argtypes = [_P, _Z, _I, _P, _P]
        L.laplex_get_plan_status.argtypes = [_P, _Z, _I, _P, _P]
        L.laplex_status_string.argtypes = [ctypes.c_int]
        L.laplex_status_string.restype = ctypes.c_char_p
        L.laplex_last_hip_error.argtypes = []
        L.laplex_last_hip_error.restype = ctypes.c_char_p
        L.laplex_profile_begin.argtypes = [ctypes.c_char_p]
        L.laplex_profile_end.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64)]
        L.laplex_profile_family.argtypes = [_I, ctypes.c_char_p, _Z, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64)]
        L.laplex_scan_tile_rows.argtypes = [_I, ctypes.c_int, ctypes.POINTER(_I)]
        L.laplex_diag_move_rows.argtypes = [_P, _P, _P, _I, _I, _P]
        L.laplex_diag_set_plan_status.argtypes = [_P, _Z, _I, _U, _P]
        L.laplex_diag_set_route_min.argtypes = [_I]
        L.laplex_apply_static.argtypes = [_P, _I, _P, _I, _P, _I, _I, _P, _I, _U, _P]
        L.laplex_phased_workspace_bytes.argtypes = [_I, _I, _I, ctypes.POINTER(_Z)]
        L.laplex_phased_apply.argtypes = [_P, _P, _I, _P, _P, _I, _P, _I, _I, _P, _I, _P, _Z, _U, _P]
        L.laplex_phased_apply_backward.argtypes = [_P, _P, _I, _P, _P, _I, _P, _I, _P, _I, _I,
                                                   _P, _I, _P, _P, _P, _P, _P, _Z, _U, _P]
        _F = ctypes.c_float
        L.laplex_apply_tau.argtypes = [_P, _I, _P, _I, _F, _P, _I, _I, _P, _I, _P, _Z, _U, _P]
        L.laplex_apply_backward_tau.argtypes = [_P, _I, _P, _I, _F, _P, _I, _P, _I, _I, _P, _I, _P, _P, _P, _P, _Z, _U, _P]
        L.laplex_gram_tau.argtypes = [_P, _I, _F, _P, _I, _I, _P, _I, _P, _Z, _U, _P]
        L.laplex_gram_backward_tau.argtypes = [_P, _I, _F, _P, _I, _P, _I, _I, _P, _I, _P, _P, _P, _Z, _U, _P]
        L.laplex_wgram_workspace_bytes.argtypes = [_I, _I, ctypes.POINTER(ctypes.c_size_t)]
        L.laplex_wgram.argtypes = [_P, _I, _P, _I, _P, _P, _I, _P, _Z, _U, _P]
        L.laplex_wgram_f64_workspace_bytes.argtypes = [_I, _I, ctypes.POINTER(ctypes.c_size_t)]
        L.laplex_wgram_f64.argtypes = [_P, _I, _P, _I, _P, _P, _I, _P, _Z, _U, _P]
        L.laplex_mix_workspace_bytes.argtypes = [_I, _I, _I, _I, ctypes.POINTER(ctypes.c_size_t)]
        L.laplex_mix_apply.argtypes = [_P, _P, _P, _I, _I, _I, _P, _I, _I, _P, _I, _P, _Z, _U, _P]
        L.laplex_mix_apply_backward.argtypes = [_P, _P, _P, _I, _I, _I, _P, _I, _P, _I, _I, _P, _I, _P, _P, _P,
                                                _P, _Z, _U, _P]
        for name in EXPORTS + DIAG_EXPORTS:
            if name not in ("laplex_status_string", "laplex_last_hip_error"):
                getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def _check(status: int) -> None:
    if status != LAPLEX_OK:
        raise LaplexError(status)


def _ptr(t):
    return None if t is None else t.data_ptr()


def _ld(t):
    """leading dimension of a (rows, batch) tensor whose batch axis is contiguous"""
    if t is None:
        return 0
    if t.dim() == 1:
        return 1
    assert t.dim() == 2
    if t.shape[0] <= 1 or t.shape[1] == 0:
        return max(t.shape[1], 1)
    assert t.shape[1] == 1 or t.stride(1) == 1, "batch axis must be contiguous"
    return t.stride(0)


def _batch(t):
    return 1 if t.dim() == 1 else t.shape[1]


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


def laplex_workspace_bytes(k: int, n: int, batch: int) -> int:
    out = _Z(0)
    _check(lib().laplex_workspace_bytes(k, n, batch, ctypes.byref(out)))
    return out.value


def laplex_apply(a, b, x, y, ws, flags: int = 0, stream=None) -> None:
    """y (k, batch) <- L(a, b) x, x (n, batch); ws a uint8 workspace tensor."""
    _check(lib().laplex_apply(_ptr(a), a.numel(), _ptr(b), b.numel(), _ptr(x), _ld(x), _batch(x),
                              _ptr(y), _ld(y), _ptr(ws), ws.numel(), flags, _stream(stream)))


def laplex_apply_static(a, b, x, y, flags: int = 0, stream=None) -> None:
    """laplex_apply with the workspace inside the library (problems up to LAPLEX_STATIC_WORKSPACE_BYTES of it)."""
    _check(lib().laplex_apply_static(_ptr(a), a.numel(), _ptr(b), b.numel(), _ptr(x), _ld(x), _batch(x),
                                     _ptr(y), _ld(y), flags, _stream(stream)))


def laplex_apply_backward(a, b, x, gy, gx, ga, gb, ws, flags: int = 0, stream=None) -> None:
    """gx (n, batch), ga (k), gb (n) <- gradients of sum(gy * y); any may be None."""
    _check(lib().laplex_apply_backward(
        _ptr(a), a.numel(), _ptr(b), b.numel(), _ptr(x), _ld(x), _ptr(gy), _ld(gy), _batch(gy),
        _ptr(gx), _ld(gx), _ptr(ga), _ptr(gb), _ptr(ws), ws.numel(), flags, _stream(stream)))


def laplex_gram(a, x, y, ws, flags: int = 0, stream=None) -> None:
    _check(lib().laplex_gram(_ptr(a), a.numel(), _ptr(x), _ld(x), _batch(x), _ptr(y), _ld(y),
                             _ptr(ws), ws.numel(), flags, _stream(stream)))


def laplex_gram_backward(a, x, gy, gx, ga, ws, flags: int = 0, stream=None) -> None:
    _check(lib().laplex_gram_backward(
        _ptr(a), a.numel(), _ptr(x), _ld(x), _ptr(gy), _ld(gy), _batch(gy),
        _ptr(gx), _ld(gx), _ptr(ga), _ptr(ws), ws.numel(), flags, _stream(stream)))


def laplex_get_perm(ws, count: int, perm_out, stream=None) -> None:
    """perm_out: int32 tensor of `count` elements (bit pattern of the u32 ids)."""
    _check(lib().laplex_get_perm(_ptr(ws), ws.numel(), count, _ptr(perm_out), _stream(stream)))


def laplex_get_plan_status(ws, count: int, status_out, stream=None) -> None:
    """status_out: int32 tensor of one element: 0 = the plan was built normally, 1 = the radix sort gave up a wait."""
    _check(lib().laplex_get_plan_status(_ptr(ws), ws.numel(), count, _ptr(status_out), _stream(stream)))


def laplex_diag_set_plan_status(ws, count: int, value: int, stream=None) -> None:
    """Test hook: overwrite the status word of the plan in ws (0 = valid, 1 = invalid)."""
    _check(lib().laplex_diag_set_plan_status(_ptr(ws), ws.numel(), count, value, _stream(stream)))


def laplex_diag_set_route_min(merged_positions: int) -> None:
    """Test hook: batch-1 problems from this many merged positions on take the routes without random accesses."""
    _check(lib().laplex_diag_set_route_min(merged_positions))


def laplex_diag_move_rows(src, dst, row_ids, stream=None) -> None:
    """Diagnostics: rows row_ids[r] of src (rows x cols, contiguous) are read (dst None) or copied to the same rows of dst."""
    _check(lib().laplex_diag_move_rows(_ptr(src), _ptr(dst), _ptr(row_ids), row_ids.numel(), src.shape[1], _stream(stream)))


def laplex_status_string(status: int) -> str:
    return lib().laplex_status_string(status).decode()


def laplex_last_hip_error() -> str:
    return lib().laplex_last_hip_error().decode()


def laplex_profile_begin(family: str) -> None:
    _check(lib().laplex_profile_begin(family.encode()))


def laplex_profile_end():
    """(summed milliseconds, launches) of the family named at laplex_profile_begin."""
    ms, cnt = ctypes.c_double(0.0), ctypes.c_int64(0)
    _check(lib().laplex_profile_end(ctypes.byref(ms), ctypes.byref(cnt)))
    return ms.value, cnt.value


def laplex_profile_families():
    """{family: (summed milliseconds, launches)} of the measurement that laplex_profile_end closed (family "*": all)."""
    out, i = {}, 0
    while True:
        name = ctypes.create_string_buffer(128)
        ms, cnt = ctypes.c_double(0.0), ctypes.c_int64(0)
        rc = lib().laplex_profile_family(i, name, 128, ctypes.byref(ms), ctypes.byref(cnt))
        if rc == LAPLEX_ERR_SIZE:
            return out
        _check(rc)
        out[name.value.decode()] = (ms.value, cnt.value)
        i += 1


def laplex_scan_tile_rows(batch: int, wide: bool) -> int:
    rows = _I(0)
    _check(lib().laplex_scan_tile_rows(batch, 1 if wide else 0, ctypes.byref(rows)))
    return rows.value


def laplex_phased_workspace_bytes(k: int, n: int, batch: int) -> int:
    out = _Z(0)
    _check(lib().laplex_phased_workspace_bytes(k, n, batch, ctypes.byref(out)))
    return out.value


def laplex_phased_apply(a, phi, b, psi, x, y, ws, flags: int = 0, stream=None) -> None:
    """y (k, batch) <- P x with P_ij = exp(-|a_i - b_j|) cos(phi_i - psi_j)."""
    _check(lib().laplex_phased_apply(
        _ptr(a), _ptr(phi), a.numel(), _ptr(b), _ptr(psi), b.numel(), _ptr(x), _ld(x), _batch(x),
        _ptr(y), _ld(y), _ptr(ws), ws.numel(), flags, _stream(stream)))


def laplex_phased_apply_backward(a, phi, b, psi, x, gy, gx, ga, gb, gphi, gpsi, ws, flags: int = 0, stream=None) -> None:
    """gradients of sum(gy * y) of the phased product; any output may be None."""
    _check(lib().laplex_phased_apply_backward(
        _ptr(a), _ptr(phi), a.numel(), _ptr(b), _ptr(psi), b.numel(), _ptr(x), _ld(x), _ptr(gy), _ld(gy), _batch(gy),
        _ptr(gx), _ld(gx), _ptr(ga), _ptr(gb), _ptr(gphi), _ptr(gpsi), _ptr(ws), ws.numel(), flags, _stream(stream)))


def laplex_apply_tau(a, b, tau: float, x, y, ws, flags: int = 0, stream=None) -> None:
    """y <- L_tau(a, b) x with L_tau = exp(-tau |a_i - b_j|) (inverse temperature tau > 0)."""
    _check(lib().laplex_apply_tau(_ptr(a), a.numel(), _ptr(b), b.numel(), tau, _ptr(x), _ld(x), _batch(x),
                                  _ptr(y), _ld(y), _ptr(ws), ws.numel(), flags, _stream(stream)))


def laplex_apply_backward_tau(a, b, tau: float, x, gy, gx, ga, gb, gtau, ws, flags: int = 0, stream=None) -> None:
    _check(lib().laplex_apply_backward_tau(
        _ptr(a), a.numel(), _ptr(b), b.numel(), tau, _ptr(x), _ld(x), _ptr(gy), _ld(gy), _batch(gy),
        _ptr(gx), _ld(gx), _ptr(ga), _ptr(gb), _ptr(gtau), _ptr(ws), ws.numel(), flags, _stream(stream)))


def laplex_gram_tau(a, tau: float, x, y, ws, flags: int = 0, stream=None) -> None:
    _check(lib().laplex_gram_tau(_ptr(a), a.numel(), tau, _ptr(x), _ld(x), _batch(x), _ptr(y), _ld(y),
                                 _ptr(ws), ws.numel(), flags, _stream(stream)))


def laplex_gram_backward_tau(a, tau: float, x, gy, gx, ga, gtau, ws, flags: int = 0, stream=None) -> None:
    _check(lib().laplex_gram_backward_tau(
        _ptr(a), a.numel(), tau, _ptr(x), _ld(x), _ptr(gy), _ld(gy), _batch(gy),
        _ptr(gx), _ld(gx), _ptr(ga), _ptr(gtau), _ptr(ws), ws.numel(), flags, _stream(stream)))


def laplex_wgram_workspace_bytes(k: int, n: int) -> int:
    out = ctypes.c_size_t(0)
    _check(lib().laplex_wgram_workspace_bytes(k, n, ctypes.byref(out)))
    return out.value


def laplex_wgram(a, b, d, m, ws, flags: int = 0, stream=None) -> None:
    """m (k, k) <- A diag(d) A^T with A = L(a, b): the weighted Gram matrix."""
    _check(lib().laplex_wgram(_ptr(a), a.numel(), _ptr(b), b.numel(), _ptr(d), _ptr(m), _ld(m),
                              _ptr(ws), ws.numel(), flags, _stream(stream)))


def laplex_mix_workspace_bytes(r: int, k: int, n: int, batch: int) -> int:
    out = ctypes.c_size_t(0)
    _check(lib().laplex_mix_workspace_bytes(r, k, n, batch, ctypes.byref(out)))
    return out.value


def laplex_mix_apply(a, b, w, x, y, ws, flags: int = 0, stream=None) -> None:
    """y <- sum_q w[q] L(a[q], b[q]) x;  a (r, k), b (r, n) contiguous, w (r,) on the device."""
    _check(lib().laplex_mix_apply(_ptr(a), _ptr(b), _ptr(w), a.shape[0], a.shape[1], b.shape[1],
                                  _ptr(x), _ld(x), _batch(x), _ptr(y), _ld(y), _ptr(ws), ws.numel(), flags, _stream(stream)))


def laplex_mix_apply_backward(a, b, w, x, gy, gx, ga, gb, gw, ws, flags: int = 0, stream=None) -> None:
    _check(lib().laplex_mix_apply_backward(
        _ptr(a), _ptr(b), _ptr(w), a.shape[0], a.shape[1], b.shape[1], _ptr(x), _ld(x), _ptr(gy), _ld(gy), _batch(gy),
        _ptr(gx), _ld(gx), _ptr(ga), _ptr(gb), _ptr(gw), _ptr(ws), ws.numel(), flags, _stream(stream)))


def laplex_wgram_f64_workspace_bytes(k: int, n: int) -> int:
    out = ctypes.c_size_t(0)
    _check(lib().laplex_wgram_f64_workspace_bytes(k, n, ctypes.byref(out)))
    return out.value


def laplex_wgram_f64(a, b, d, m, ws, flags: int = 0, stream=None) -> None:
    """m (k, k) fp64 <- A diag(d) A^T, fp32 anchors, fp64 weights and arithmetic."""
    _check(lib().laplex_wgram_f64(_ptr(a), a.numel(), _ptr(b), b.numel(), _ptr(d), _ptr(m), _ld(m),
                                  _ptr(ws), ws.numel(), flags, _stream(stream)))
