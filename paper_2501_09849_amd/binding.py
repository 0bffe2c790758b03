"""Thin ctypes binding of libcdl.so: same names and arguments as include/cdl.h.

Tensors are torch CUDA (ROCm) tensors used only as device memory; every step
of the computation runs in the library's kernels.  There is no fallback: if
the shared library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libcdl.so")
_LIB = None

EXPORTS = (
    "cdl_quantize_workspace_bytes", "cdl_qgemm_fwd_workspace_bytes", "cdl_qgemm_bwd_workspace_bytes",
    "cdl_qgemm_fwd_offset_workspace_bytes", "cdl_index_offset", "cdl_qgemm_fwd_offset", "cdl_qgemm_bwd_offset",
    "cdl_qgemm_bwd_quantize_bwd", "cdl_qconv_fwd_workspace_bytes", "cdl_qconv_fwd", "cdl_qgemm_fwd_quantize",
    "cdl_qconv_bwd_weights_workspace_bytes", "cdl_qconv_bwd_weights",
    "cdl_qconv_bwd_activations_workspace_bytes", "cdl_qconv_bwd_activations",
    "cdl_quantize_fwd", "cdl_quantize_fwd_static", "cdl_static_scratch_bytes", "cdl_quantize_bwd", "cdl_marginal_entropy", "cdl_qgemm_fwd", "cdl_qgemm_bwd",
    "cdl_quantize_draw", "cdl_entropy_bwd", "cdl_huffman_workspace_bytes", "cdl_huffman_bits",
    "cdl_profile_enable", "cdl_profile_collect", "cdl_profile_only", "cdl_probe_mfma_int8",
    "cdl_status_string", "cdl_last_hip_error", "cdl_version",
)


class CdlError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = load().cdl_status_string(status).decode()
        if status == -6:
            msg += " [hipError %d]" % load().cdl_last_hip_error()
        super().__init__("%s: %s (status %d)" % (where, msg, status))


class QParams(ctypes.Structure):
    """struct cdl_qparams"""
    _fields_ = [("lo", ctypes.c_int32), ("n_levels", ctypes.c_int32),
                ("delta", ctypes.c_float), ("alpha", ctypes.c_float), ("top_k", ctypes.c_int32)]


class ProfileRecord(ctypes.Structure):
    """struct cdl_profile_record"""
    _fields_ = [("kernel", ctypes.c_char * 56), ("ms", ctypes.c_float)]


def lib_path() -> str:
    return _LIB_PATH


def load():
    """Load libcdl.so (built beforehand by paper_2501_09849_amd.build / __graft_entry__.build)."""
    global _LIB
    if _LIB is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError("libcdl.so is not built: run `python -m paper_2501_09849_amd.build` "
                               "(or __graft_entry__.build()) first; there is no fallback path")
        from . import build as _build
        if _LIB_PATH == _build.LIB_PATH and _build.is_stale():
            raise RuntimeError("libcdl.so was not built from the sources now in the tree (csrc/*.hip, csrc/*.h, "
                               "include/*.h or the compiler flags changed since): run `python -m "
                               "paper_2501_09849_amd.build` again; a stale binary is never loaded")
        # PyTorch-ROCm carries its own copy of the HIP runtime and loads it by path.  If libcdl.so came first,
        # the system's copy would be in the process as well, the two would not share a device context, and
        # every launch on torch's memory would fail with hipErrorNoDevice: let torch's be the first one.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        L = ctypes.CDLL(_LIB_PATH)
        vp, i64, i32, f32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_float, ctypes.c_size_t
        qp = ctypes.POINTER(QParams)
        L.cdl_quantize_workspace_bytes.restype = sz
        L.cdl_quantize_workspace_bytes.argtypes = [i64, i32]
        L.cdl_qgemm_fwd_workspace_bytes.restype = sz
        L.cdl_qgemm_fwd_workspace_bytes.argtypes = [i32, i32, i32]
        L.cdl_qgemm_bwd_workspace_bytes.restype = sz
        L.cdl_qgemm_bwd_workspace_bytes.argtypes = [i32, i32, i32]
        L.cdl_quantize_fwd.restype = ctypes.c_int
        L.cdl_quantize_fwd.argtypes = [vp, i64, qp, vp, vp, vp, vp, vp, sz, vp]
        L.cdl_quantize_fwd_static.restype = ctypes.c_int
        L.cdl_quantize_fwd_static.argtypes = [vp, i64, qp, vp, vp, vp, vp, vp]
        L.cdl_static_scratch_bytes.restype = sz
        L.cdl_static_scratch_bytes.argtypes = []
        L.cdl_quantize_bwd.restype = ctypes.c_int
        L.cdl_quantize_bwd.argtypes = [vp, vp, i64, qp, vp, vp, vp, vp, sz, vp]
        L.cdl_marginal_entropy.restype = ctypes.c_int
        L.cdl_marginal_entropy.argtypes = [vp, i64, qp, vp, vp, vp, sz, vp]
        L.cdl_quantize_draw.restype = ctypes.c_int
        L.cdl_quantize_draw.argtypes = [vp, vp, i64, qp, vp, vp]
        L.cdl_entropy_bwd.restype = ctypes.c_int
        L.cdl_entropy_bwd.argtypes = [vp, vp, vp, i64, qp, f32, vp, vp, vp, vp, sz, vp]
        L.cdl_huffman_workspace_bytes.restype = sz
        L.cdl_huffman_workspace_bytes.argtypes = [i64]
        L.cdl_huffman_bits.restype = ctypes.c_int
        L.cdl_huffman_bits.argtypes = [vp, i64, i32, i32, vp, vp, vp, vp, sz, vp]
        L.cdl_qgemm_fwd.restype = ctypes.c_int
        L.cdl_qgemm_fwd.argtypes = [vp, vp, i32, i32, i32, f32, f32, vp, vp, vp, sz, vp]
        L.cdl_qgemm_bwd.restype = ctypes.c_int
        L.cdl_qgemm_bwd.argtypes = [vp, vp, vp, i32, i32, i32, f32, f32, vp, vp, vp, sz, vp]
        L.cdl_qgemm_fwd_offset_workspace_bytes.restype = sz
        L.cdl_qgemm_fwd_offset_workspace_bytes.argtypes = [i32, i32, i32]
        L.cdl_index_offset.restype = i32
        L.cdl_index_offset.argtypes = [qp]
        L.cdl_qgemm_fwd_offset.restype = ctypes.c_int
        L.cdl_qgemm_fwd_offset.argtypes = [vp, vp, i32, i32, i32, f32, f32, i32, i32, vp, vp, vp, sz, vp]
        L.cdl_qconv_bwd_weights_workspace_bytes.restype = ctypes.c_size_t
        L.cdl_qconv_bwd_weights_workspace_bytes.argtypes = [i32] * 9
        L.cdl_qconv_bwd_weights.restype = ctypes.c_int
        L.cdl_qconv_bwd_weights.argtypes = [vp, vp] + [i32] * 9 + [f32, i32, vp, vp, sz, vp]
        L.cdl_qconv_bwd_activations_workspace_bytes.restype = ctypes.c_size_t
        L.cdl_qconv_bwd_activations_workspace_bytes.argtypes = [i32] * 9
        L.cdl_qconv_bwd_activations.restype = ctypes.c_int
        L.cdl_qconv_bwd_activations.argtypes = [vp, vp] + [i32] * 9 + [f32, vp, vp, sz, vp]
        L.cdl_qgemm_fwd_quantize.restype = ctypes.c_int
        L.cdl_qgemm_fwd_quantize.argtypes = [vp, qp, vp, i32, i32, i32, f32, vp, vp]
        L.cdl_qconv_fwd_workspace_bytes.restype = ctypes.c_size_t
        L.cdl_qconv_fwd_workspace_bytes.argtypes = [i32, i32]
        L.cdl_qconv_fwd.restype = ctypes.c_int
        L.cdl_qconv_fwd.argtypes = [vp, vp] + [i32] * 9 + [f32, f32, i32, vp, vp, vp, sz, vp]
        L.cdl_qgemm_bwd_quantize_bwd.restype = ctypes.c_int
        L.cdl_qgemm_bwd_quantize_bwd.argtypes = [vp, vp, vp, i32, i32, i32, vp, qp, f32, i32, vp, vp, vp, vp, vp, qp, vp, vp, vp, vp, sz, vp]
        L.cdl_qgemm_bwd_offset.restype = ctypes.c_int
        L.cdl_qgemm_bwd_offset.argtypes = [vp, vp, vp, i32, i32, i32, f32, f32, i32, i32, vp, vp, vp, sz, vp]
        L.cdl_profile_enable.restype = ctypes.c_int
        L.cdl_profile_enable.argtypes = [ctypes.c_int]
        L.cdl_profile_only.restype = ctypes.c_int
        L.cdl_profile_only.argtypes = [ctypes.c_char_p]
        L.cdl_profile_collect.restype = ctypes.c_int
        L.cdl_profile_collect.argtypes = [ctypes.POINTER(ProfileRecord), ctypes.c_int]
        L.cdl_status_string.restype = ctypes.c_char_p
        L.cdl_status_string.argtypes = [ctypes.c_int]
        L.cdl_last_hip_error.restype = ctypes.c_int
        L.cdl_version.restype = ctypes.c_int
        _LIB = L
    return _LIB


def _ptr(t) -> Optional[int]:
    """Device address of a torch tensor (None -> NULL); a bare int passes through."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return t.data_ptr()


def _ws(ws):
    if ws is None:
        return None, 0
    return ws.data_ptr(), ws.numel() * ws.element_size()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def _qp(lo: int, n_levels: int, delta: float, alpha: float, top_k: int = 0) -> QParams:
    return QParams(int(lo), int(n_levels), float(delta), float(alpha), int(top_k))


def quantize_workspace_bytes(n: int, n_levels: int) -> int:
    return int(load().cdl_quantize_workspace_bytes(n, n_levels))


def qgemm_fwd_workspace_bytes(M: int, N: int, K: int) -> int:
    return int(load().cdl_qgemm_fwd_workspace_bytes(M, N, K))


def qgemm_bwd_workspace_bytes(M: int, N: int, K: int) -> int:
    return int(load().cdl_qgemm_bwd_workspace_bytes(M, N, K))


def qgemm_fwd_offset_workspace_bytes(M: int, N: int, K: int) -> int:
    return int(load().cdl_qgemm_fwd_offset_workspace_bytes(M, N, K))


def cdl_index_offset(lo: int, n_levels: int, delta: float = 1.0, alpha: float = 1.0) -> int:
    q = _qp(lo, n_levels, delta, alpha)
    off = int(load().cdl_index_offset(ctypes.byref(q)))
    if off < 0:
        raise CdlError(off, "cdl_index_offset")
    return off


def _check(rc: int, where: str):
    if rc != 0:
        raise CdlError(rc, where)


def cdl_quantize_fwd(theta, n, lo, n_levels, delta, alpha, idx, soft=None, marg=None, entropy_bits=None,
                     ws=None, stream=None, top_k=0):
    wp, wb = _ws(ws)
    q = _qp(lo, n_levels, delta, alpha, top_k)
    _check(load().cdl_quantize_fwd(_ptr(theta), n, ctypes.byref(q), _ptr(idx), _ptr(soft), _ptr(marg),
                                   _ptr(entropy_bits), wp, wb, _stream(stream)), "cdl_quantize_fwd")


def static_scratch_bytes() -> int:
    return int(load().cdl_static_scratch_bytes())


def cdl_quantize_fwd_static(theta, n, lo, n_levels, delta, alpha, idx, soft=None, marg=None, entropy_bits=None,
                            stream=None, top_k=0):
    q = _qp(lo, n_levels, delta, alpha, top_k)
    _check(load().cdl_quantize_fwd_static(_ptr(theta), n, ctypes.byref(q), _ptr(idx), _ptr(soft), _ptr(marg),
                                          _ptr(entropy_bits), _stream(stream)), "cdl_quantize_fwd_static")


def cdl_quantize_bwd(theta, g, n, lo, n_levels, delta, alpha, dtheta=None, d_delta=None, d_alpha=None,
                     ws=None, stream=None, top_k=0):
    wp, wb = _ws(ws)
    q = _qp(lo, n_levels, delta, alpha, top_k)
    _check(load().cdl_quantize_bwd(_ptr(theta), _ptr(g), n, ctypes.byref(q), _ptr(dtheta), _ptr(d_delta),
                                   _ptr(d_alpha), wp, wb, _stream(stream)), "cdl_quantize_bwd")


def cdl_marginal_entropy(theta, n, lo, n_levels, delta, alpha, marg=None, entropy_bits=None, ws=None, stream=None,
                         top_k=0):
    wp, wb = _ws(ws)
    q = _qp(lo, n_levels, delta, alpha, top_k)
    _check(load().cdl_marginal_entropy(_ptr(theta), n, ctypes.byref(q), _ptr(marg), _ptr(entropy_bits),
                                       wp, wb, _stream(stream)), "cdl_marginal_entropy")


def cdl_quantize_draw(theta, u, n, lo, n_levels, delta, alpha, idx, stream=None, top_k=0):
    q = _qp(lo, n_levels, delta, alpha, top_k)
    _check(load().cdl_quantize_draw(_ptr(theta), _ptr(u), n, ctypes.byref(q), _ptr(idx), _stream(stream)),
           "cdl_quantize_draw")


def cdl_entropy_bwd(theta, marg, n, lo, n_levels, delta, alpha, scale=1.0, g_in=None, dtheta=None, d_delta=None,
                    d_alpha=None, ws=None, stream=None, top_k=0):
    wp, wb = _ws(ws)
    q = _qp(lo, n_levels, delta, alpha, top_k)
    _check(load().cdl_entropy_bwd(_ptr(theta), _ptr(marg), _ptr(g_in), n, ctypes.byref(q), float(scale),
                                  _ptr(dtheta), _ptr(d_delta), _ptr(d_alpha), wp, wb, _stream(stream)),
           "cdl_entropy_bwd")


def huffman_workspace_bytes(n: int) -> int:
    return int(load().cdl_huffman_workspace_bytes(n))


def cdl_huffman_bits(idx, n, lo, n_levels, counts=None, total_bits=None, bits_per_entry=None, ws=None, stream=None):
    wp, wb = _ws(ws)
    _check(load().cdl_huffman_bits(_ptr(idx), n, lo, n_levels, _ptr(counts), _ptr(total_bits), _ptr(bits_per_entry),
                                   wp, wb, _stream(stream)), "cdl_huffman_bits")


def cdl_qgemm_fwd(a_idx, b_idx, M, N, K, delta_a, delta_b, acc=None, y=None, ws=None, stream=None):
    wp, wb = _ws(ws)
    _check(load().cdl_qgemm_fwd(_ptr(a_idx), _ptr(b_idx), M, N, K, delta_a, delta_b, _ptr(acc), _ptr(y),
                                wp, wb, _stream(stream)), "cdl_qgemm_fwd")


def cdl_qgemm_fwd_offset(a_idx, b_idx, M, N, K, delta_a, delta_b, a_offset, b_offset, acc=None, y=None, ws=None, stream=None):
    wp, wb = _ws(ws)
    _check(load().cdl_qgemm_fwd_offset(_ptr(a_idx), _ptr(b_idx), M, N, K, delta_a, delta_b, int(a_offset), int(b_offset),
                                       _ptr(acc), _ptr(y), wp, wb, _stream(stream)), "cdl_qgemm_fwd_offset")


def cdl_qgemm_bwd_offset(g, a_idx, b_idx, M, N, K, delta_a, delta_b, a_offset, b_offset, d_a_hat=None, d_b_hat=None,
                         ws=None, stream=None):
    wp, wb = _ws(ws)
    _check(load().cdl_qgemm_bwd_offset(_ptr(g), _ptr(a_idx), _ptr(b_idx), M, N, K, delta_a, delta_b, int(a_offset), int(b_offset),
                                       _ptr(d_a_hat), _ptr(d_b_hat), wp, wb, _stream(stream)), "cdl_qgemm_bwd_offset")


def cdl_qgemm_bwd_quantize_bwd(g, a_idx, b_idx, M, N, K, theta_a, lo_a, n_levels_a, delta_a, alpha_a, delta_b, d_theta_a,
                               d_delta_a=None, d_alpha_a=None, d_b_hat=None, ws=None, stream=None, b_offset=0, top_k=0,
                               theta_b=None, qparams_b=None, d_theta_b=None, d_delta_b=None, d_alpha_b=None):
    """qparams_b: (lo, n_levels, delta, alpha[, top_k]) of the weight quantizer, with theta_b and d_theta_b."""
    wp, wb = _ws(ws)
    q = _qp(lo_a, n_levels_a, delta_a, alpha_a, top_k)
    qb = _qp(*qparams_b) if qparams_b is not None else None
    _check(load().cdl_qgemm_bwd_quantize_bwd(_ptr(g), _ptr(a_idx), _ptr(b_idx), M, N, K, _ptr(theta_a), ctypes.byref(q), delta_b,
                                             int(b_offset), _ptr(d_theta_a), _ptr(d_delta_a), _ptr(d_alpha_a), _ptr(d_b_hat),
                                             _ptr(theta_b), ctypes.byref(qb) if qb is not None else None, _ptr(d_theta_b),
                                             _ptr(d_delta_b), _ptr(d_alpha_b), wp, wb, _stream(stream)), "cdl_qgemm_bwd_quantize_bwd")


def qconv_bwd_weights_workspace_bytes(B, H, W, C, N, R, S, stride, pad) -> int:
    return int(load().cdl_qconv_bwd_weights_workspace_bytes(B, H, W, C, N, R, S, stride, pad))


def cdl_qconv_bwd_weights(g, x_idx, B, H, W, C, N, R, S, stride, pad, delta_x, d_w_hat, ws, stream=None, x_offset=0):
    wp, wb = _ws(ws)
    _check(load().cdl_qconv_bwd_weights(_ptr(g), _ptr(x_idx), B, H, W, C, N, R, S, stride, pad, delta_x, int(x_offset),
                                        _ptr(d_w_hat), wp, wb, _stream(stream)), "cdl_qconv_bwd_weights")


def qconv_bwd_activations_workspace_bytes(B, H, W, C, N, R, S, stride, pad) -> int:
    return int(load().cdl_qconv_bwd_activations_workspace_bytes(B, H, W, C, N, R, S, stride, pad))


def cdl_qconv_bwd_activations(g, w_idx, B, H, W, C, N, R, S, stride, pad, delta_w, d_x_hat, ws, stream=None):
    wp, wb = _ws(ws)
    _check(load().cdl_qconv_bwd_activations(_ptr(g), _ptr(w_idx), B, H, W, C, N, R, S, stride, pad, delta_w,
                                            _ptr(d_x_hat), wp, wb, _stream(stream)), "cdl_qconv_bwd_activations")


def cdl_qgemm_fwd_quantize(x, lo_a, n_levels_a, delta_a, alpha_a, b_idx, M, N, K, delta_b, y, stream=None):
    q = _qp(lo_a, n_levels_a, delta_a, alpha_a, 0)
    _check(load().cdl_qgemm_fwd_quantize(_ptr(x), ctypes.byref(q), _ptr(b_idx), M, N, K, delta_b, _ptr(y), _stream(stream)),
           "cdl_qgemm_fwd_quantize")


def qconv_fwd_workspace_bytes(N: int, x_offset: int = 0) -> int:
    return int(load().cdl_qconv_fwd_workspace_bytes(N, x_offset))


def cdl_qconv_fwd(x_idx, w_idx, B, H, W, C, N, R, S, stride, pad, delta_x, delta_w, acc=None, y=None, ws=None, stream=None,
                  x_offset=0):
    wp, wb = _ws(ws)
    _check(load().cdl_qconv_fwd(_ptr(x_idx), _ptr(w_idx), B, H, W, C, N, R, S, stride, pad, delta_x, delta_w, int(x_offset),
                                _ptr(acc), _ptr(y), wp, wb, _stream(stream)), "cdl_qconv_fwd")


def cdl_qgemm_bwd(g, a_idx, b_idx, M, N, K, delta_a, delta_b, d_a_hat=None, d_b_hat=None, ws=None, stream=None):
    wp, wb = _ws(ws)
    _check(load().cdl_qgemm_bwd(_ptr(g), _ptr(a_idx), _ptr(b_idx), M, N, K, delta_a, delta_b,
                                _ptr(d_a_hat), _ptr(d_b_hat), wp, wb, _stream(stream)), "cdl_qgemm_bwd")


def cdl_probe_mfma_int8(iters: int, random_operands: bool, blocks: int, sink, stream=None) -> float:
    """Enqueues the register-resident int8 MFMA probe; returns the integer operations it performs."""
    ops = ctypes.c_double(0.0)
    f = load().cdl_probe_mfma_int8
    f.restype = ctypes.c_int
    f.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.POINTER(ctypes.c_double), ctypes.c_void_p]
    _check(f(iters, 1 if random_operands else 0, blocks, _ptr(sink), ctypes.byref(ops), _stream(stream)), "cdl_probe_mfma_int8")
    return ops.value


def cdl_profile_enable(enable: bool) -> None:
    _check(load().cdl_profile_enable(1 if enable else 0), "cdl_profile_enable")


def cdl_profile_only(kernel: Optional[str]) -> None:
    """Time only launches recorded under this kernel name; None = all launches."""
    _check(load().cdl_profile_only(kernel.encode() if kernel else None), "cdl_profile_only")


def cdl_profile_collect(max_records: int = 65536):
    """Waits for the recorded events; returns [(kernel name, milliseconds), ...] in launch order."""
    buf = (ProfileRecord * max_records)()
    n = load().cdl_profile_collect(buf, max_records)
    if n < 0:
        raise CdlError(n, "cdl_profile_collect")
    return [(buf[i].kernel.decode(), float(buf[i].ms)) for i in range(n)]
