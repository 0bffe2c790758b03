"""ctypes front end of the CPU oracle (oracle/cdl_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
CPU-baseline leg of the benchmark.  The GPU package never imports it and it
never imports the GPU package.

The shared object is compiled with gcc next to this file; `build()` does it
explicitly and `lib()` does it on first use when the object is missing or
older than its source.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "cdl_oracle.c")
_SO = os.path.join(_HERE, "libcdl_oracle.so")
_LIB = None


def build(force: bool = True) -> str:
    """Compile the oracle with gcc (-O2, OpenMP over elements/rows only)."""
    if force or (not os.path.exists(_SO)) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        tmp = _SO + ".tmp.%d" % os.getpid()
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off",
               "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _SO)
    return _SO


_f32p = ctypes.POINTER(ctypes.c_float)
_f64p = ctypes.POINTER(ctypes.c_double)
_i32p = ctypes.POINTER(ctypes.c_int32)
_i16p = ctypes.POINTER(ctypes.c_int16)


def lib():
    global _LIB
    if _LIB is None:
        build(force=False)
        L = ctypes.CDLL(_SO)
        L.cdl_oracle_num_threads.restype = ctypes.c_int
        L.cdl_oracle_cpmf.restype = ctypes.c_int
        L.cdl_oracle_cpmf.argtypes = [ctypes.c_double, ctypes.c_int, ctypes.c_int, ctypes.c_double,
                                      ctypes.c_double, _f64p, _f64p]
        L.cdl_oracle_element.restype = None
        L.cdl_oracle_element.argtypes = [ctypes.c_double, ctypes.c_int, ctypes.c_int, ctypes.c_double,
                                         ctypes.c_double, _i32p, _f64p, _f64p, _f64p, _f64p, _f64p]
        L.cdl_oracle_lemma1_raw.restype = None
        L.cdl_oracle_lemma1_raw.argtypes = [ctypes.c_double, ctypes.c_int, ctypes.c_int, ctypes.c_double,
                                            ctypes.c_double, _f64p, _f64p]
        L.cdl_oracle_quantize_fwd.restype = None
        L.cdl_oracle_quantize_fwd.argtypes = [_f32p, ctypes.c_int64, ctypes.c_int, ctypes.c_int,
                                              ctypes.c_float, ctypes.c_float, _i32p, _f64p, _f64p]
        L.cdl_oracle_marginal_entropy.restype = None
        L.cdl_oracle_marginal_entropy.argtypes = [_f32p, ctypes.c_int64, ctypes.c_int, ctypes.c_int,
                                                  ctypes.c_float, ctypes.c_float, _f64p, _f64p]
        L.cdl_oracle_quantize_bwd.restype = None
        L.cdl_oracle_quantize_bwd.argtypes = [_f32p, _f32p, ctypes.c_int64, ctypes.c_int, ctypes.c_int,
                                              ctypes.c_float, ctypes.c_float, _f64p, _f64p, _f64p]
        L.cdl_oracle_moments_k.restype = None
        L.cdl_oracle_moments_k.argtypes = [_f32p, ctypes.c_int64, ctypes.c_int, ctypes.c_int,
                                           ctypes.c_float, ctypes.c_float, ctypes.c_int, _f64p, _f64p, _f64p]
        L.cdl_oracle_cpmf_k.restype = ctypes.c_int
        L.cdl_oracle_cpmf_k.argtypes = [ctypes.c_double, ctypes.c_int, ctypes.c_int, ctypes.c_double,
                                        ctypes.c_double, ctypes.c_int, _f64p, _f64p]
        L.cdl_oracle_element_k.restype = None
        L.cdl_oracle_element_k.argtypes = [ctypes.c_double, ctypes.c_int, ctypes.c_int, ctypes.c_double,
                                           ctypes.c_double, ctypes.c_int, _i32p, _f64p, _f64p, _f64p, _f64p, _f64p]
        L.cdl_oracle_quantize_fwd_k.restype = None
        L.cdl_oracle_quantize_fwd_k.argtypes = [_f32p, ctypes.c_int64, ctypes.c_int, ctypes.c_int,
                                                ctypes.c_float, ctypes.c_float, ctypes.c_int, _i32p, _f64p, _f64p]
        L.cdl_oracle_marginal_entropy_k.restype = None
        L.cdl_oracle_marginal_entropy_k.argtypes = [_f32p, ctypes.c_int64, ctypes.c_int, ctypes.c_int,
                                                    ctypes.c_float, ctypes.c_float, ctypes.c_int, _f64p, _f64p]
        L.cdl_oracle_quantize_bwd_k.restype = None
        L.cdl_oracle_quantize_bwd_k.argtypes = [_f32p, _f32p, ctypes.c_int64, ctypes.c_int, ctypes.c_int,
                                                ctypes.c_float, ctypes.c_float, ctypes.c_int,
                                                _f64p, _f64p, _f64p]
        L.cdl_oracle_quantize_draw.restype = None
        L.cdl_oracle_quantize_draw.argtypes = [_f32p, _f32p, ctypes.c_int64, ctypes.c_int, ctypes.c_int,
                                               ctypes.c_float, ctypes.c_float, ctypes.c_int, _i32p, _f64p]
        L.cdl_oracle_entropy_bwd.restype = None
        L.cdl_oracle_entropy_bwd.argtypes = [_f32p, ctypes.c_int64, ctypes.c_int, ctypes.c_int,
                                             ctypes.c_float, ctypes.c_float, ctypes.c_int, _f64p, ctypes.c_double,
                                             _f64p, _f64p, _f64p, _f64p, _f64p]
        L.cdl_oracle_huffman_bits.restype = None
        L.cdl_oracle_huffman_bits.argtypes = [_i16p, ctypes.c_int64, ctypes.c_int, ctypes.c_int,
                                              ctypes.POINTER(ctypes.c_int64), _f64p, _f64p]
        L.cdl_oracle_qgemm_fwd.restype = None
        L.cdl_oracle_qgemm_fwd.argtypes = [_i16p, _i16p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                           ctypes.c_float, ctypes.c_float, _i32p, _f64p]
        L.cdl_oracle_qconv_fwd.restype = None
        L.cdl_oracle_qconv_fwd.argtypes = [_i16p, _i16p] + [ctypes.c_int] * 9 + [ctypes.c_float, ctypes.c_float, _i32p, _f64p]
        L.cdl_oracle_qconv_bwd.restype = None
        L.cdl_oracle_qconv_bwd.argtypes = [_f32p, _i16p, _i16p] + [ctypes.c_int] * 9 + [ctypes.c_float, ctypes.c_float, _f64p, _f64p]
        L.cdl_oracle_qgemm_bwd.restype = None
        L.cdl_oracle_qgemm_bwd.argtypes = [_f32p, _i16p, _i16p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                           ctypes.c_float, ctypes.c_float, _f64p, _f64p]
        _LIB = L
    return _LIB


def num_threads() -> int:
    return int(lib().cdl_oracle_num_threads())


def _c(a: np.ndarray, dtype) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def _ptr(a: Optional[np.ndarray], ptype):
    return a.ctypes.data_as(ptype) if a is not None else ptype()


# ----------------------------------------------------------------- one element (double in, double out)

def cpmf(theta: float, lo: int, n_levels: int, delta: float, alpha: float, top_k: int = 0) -> Tuple[np.ndarray, int, float]:
    """CPMF over the levels for one element; returns (P, mode index, top-two score gap).

    top_k > 0: the CPMF truncated to its top_k most probable levels and renormalised (the paper uses 5 for activations)."""
    P = np.empty(n_levels, dtype=np.float64)
    gap = ctypes.c_double()
    mode = lib().cdl_oracle_cpmf_k(float(theta), lo, n_levels, float(delta), float(alpha), int(top_k),
                                   _ptr(P, _f64p), ctypes.byref(gap))
    return P, int(mode), gap.value


def element(theta: float, lo: int, n_levels: int, delta: float, alpha: float, top_k: int = 0) -> dict:
    """idx, soft value, score gap and the three partial derivatives of Q_d for one element."""
    idx = ctypes.c_int32()
    v = [ctypes.c_double() for _ in range(5)]
    lib().cdl_oracle_element_k(float(theta), lo, n_levels, float(delta), float(alpha), int(top_k), ctypes.byref(idx),
                               *[ctypes.byref(x) for x in v])
    return dict(idx=idx.value, soft=v[0].value, gap=v[1].value,
                dtheta=v[2].value, ddelta=v[3].value, dalpha=v[4].value)


def lemma1_raw(theta: float, lo: int, n_levels: int, delta: float, alpha: float) -> Tuple[float, float]:
    a, b = ctypes.c_double(), ctypes.c_double()
    lib().cdl_oracle_lemma1_raw(float(theta), lo, n_levels, float(delta), float(alpha),
                                ctypes.byref(a), ctypes.byref(b))
    return a.value, b.value


# ----------------------------------------------------------------- tensors (fp32 in, double out)

def quantize_fwd(theta: np.ndarray, lo: int, n_levels: int, delta: float, alpha: float,
                 want_soft: bool = True, want_gap: bool = True, top_k: int = 0):
    """Returns (idx int32[n], soft float64[n] | None, score_gap float64[n] | None)."""
    th = _c(theta, np.float32).reshape(-1)
    n = th.size
    idx = np.empty(n, dtype=np.int32)
    soft = np.empty(n, dtype=np.float64) if want_soft else None
    gap = np.empty(n, dtype=np.float64) if want_gap else None
    lib().cdl_oracle_quantize_fwd_k(_ptr(th, _f32p), n, lo, n_levels, float(delta), float(alpha), int(top_k),
                                    _ptr(idx, _i32p), _ptr(soft, _f64p), _ptr(gap, _f64p))
    return idx, soft, gap


def marginal_entropy(theta: np.ndarray, lo: int, n_levels: int, delta: float, alpha: float, top_k: int = 0):
    """Returns (marg float64[n_levels], entropy in bits)."""
    th = _c(theta, np.float32).reshape(-1)
    marg = np.empty(n_levels, dtype=np.float64)
    H = ctypes.c_double()
    lib().cdl_oracle_marginal_entropy_k(_ptr(th, _f32p), th.size, lo, n_levels, float(delta), float(alpha), int(top_k),
                                        _ptr(marg, _f64p), ctypes.byref(H))
    return marg, H.value


def quantize_bwd(theta: np.ndarray, g: np.ndarray, lo: int, n_levels: int, delta: float, alpha: float,
                 want_dtheta: bool = True, top_k: int = 0) -> dict:
    """dtheta float64[n] (None if not wanted), d_delta, d_alpha."""
    th = _c(theta, np.float32).reshape(-1)
    gg = _c(g, np.float32).reshape(-1)
    assert th.size == gg.size
    dth = np.empty(th.size, dtype=np.float64) if want_dtheta else None
    s = [ctypes.c_double() for _ in range(2)]
    lib().cdl_oracle_quantize_bwd_k(_ptr(th, _f32p), _ptr(gg, _f32p), th.size, lo, n_levels,
                                    float(delta), float(alpha), int(top_k), _ptr(dth, _f64p),
                                    *[ctypes.byref(x) for x in s])
    return dict(dtheta=dth, d_delta=s[0].value, d_alpha=s[1].value)


def moments(theta: np.ndarray, lo: int, n_levels: int, delta: float, alpha: float, top_k: int = 0):
    """Per entry, the three quantities of Lemma 1: (E{Q_p}, Var{Q_p}, Skew_u{Q_p}), float64[n] each."""
    th = _c(theta, np.float32).reshape(-1)
    out = [np.empty(th.size, dtype=np.float64) for _ in range(3)]
    lib().cdl_oracle_moments_k(_ptr(th, _f32p), th.size, lo, n_levels, float(delta), float(alpha), int(top_k),
                               *[_ptr(o, _f64p) for o in out])
    return tuple(out)


def quantize_draw(theta: np.ndarray, u: np.ndarray, lo: int, n_levels: int, delta: float, alpha: float,
                  top_k: int = 0):
    """The probabilistic quantizer Q_p by inversion with the uniforms u in [0,1): (idx int32[n], margin float64[n])."""
    th = _c(theta, np.float32).reshape(-1)
    uu = _c(u, np.float32).reshape(-1)
    assert th.size == uu.size
    idx = np.empty(th.size, dtype=np.int32)
    margin = np.empty(th.size, dtype=np.float64)
    lib().cdl_oracle_quantize_draw(_ptr(th, _f32p), _ptr(uu, _f32p), th.size, lo, n_levels, float(delta), float(alpha),
                                   int(top_k), _ptr(idx, _i32p), _ptr(margin, _f64p))
    return idx, margin


def entropy_bwd(theta: np.ndarray, marg: np.ndarray, lo: int, n_levels: int, delta: float, alpha: float,
                scale: float = 1.0, want_dtheta: bool = True, top_k: int = 0, want_terms: bool = False) -> dict:
    """scale * dH/d(theta, delta, alpha) of the entropy of the marginal PMF `marg` (float64[n_levels]);
    want_terms: also the contribution of every entry to d_delta and d_alpha (float64[n] each)."""
    th = _c(theta, np.float32).reshape(-1)
    mm = _c(marg, np.float64).reshape(-1)
    assert mm.size == n_levels
    dth = np.empty(th.size, dtype=np.float64) if want_dtheta else None
    td = np.empty(th.size, dtype=np.float64) if want_terms else None
    ta = np.empty(th.size, dtype=np.float64) if want_terms else None
    s = [ctypes.c_double() for _ in range(2)]
    lib().cdl_oracle_entropy_bwd(_ptr(th, _f32p), th.size, lo, n_levels, float(delta), float(alpha), int(top_k),
                                 _ptr(mm, _f64p), float(scale), _ptr(dth, _f64p), ctypes.byref(s[0]), ctypes.byref(s[1]),
                                 _ptr(td, _f64p), _ptr(ta, _f64p))
    return dict(dtheta=dth, d_delta=s[0].value, d_alpha=s[1].value, term_delta=td, term_alpha=ta)


def huffman_bits(idx: np.ndarray, lo: int, n_levels: int):
    """Huffman-coded size of a tensor of level indices: (counts int64[n_levels], total bits, bits per entry)."""
    ii = _c(idx, np.int16).reshape(-1)
    counts = np.zeros(n_levels, dtype=np.int64)
    tot, avg = ctypes.c_double(), ctypes.c_double()
    lib().cdl_oracle_huffman_bits(_ptr(ii, _i16p), ii.size, lo, n_levels,
                                  counts.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), ctypes.byref(tot), ctypes.byref(avg))
    return counts, tot.value, avg.value


def qgemm_fwd(a_idx: np.ndarray, b_idx: np.ndarray, delta_a: float, delta_b: float,
              want_y: bool = True):
    """a_idx [M,K], b_idx [N,K] level indices (any integer type, values within int16) -> (acc int32[M,N], y float64[M,N] | None)."""
    a = _c(a_idx, np.int16)
    b = _c(b_idx, np.int16)
    M, K = a.shape
    N, K2 = b.shape
    assert K == K2
    acc = np.empty((M, N), dtype=np.int32)
    y = np.empty((M, N), dtype=np.float64) if want_y else None
    lib().cdl_oracle_qgemm_fwd(_ptr(a, _i16p), _ptr(b, _i16p), M, N, K, float(delta_a), float(delta_b),
                               _ptr(acc, _i32p), _ptr(y, _f64p))
    return acc, y


def qconv_fwd(x_idx: np.ndarray, w_idx: np.ndarray, stride: int, pad: int, delta_x: float, delta_w: float,
              want_y: bool = True):
    """x_idx [B,H,W,C], w_idx [N,R,S,C] level indices -> (acc int32[B,P,Q,N], y float64[B,P,Q,N] | None)."""
    x = _c(x_idx, np.int16)
    w = _c(w_idx, np.int16)
    B, H, W, C = x.shape
    N, R, S, C2 = w.shape
    assert C == C2 and stride >= 1 and pad >= 0
    P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
    assert P >= 1 and Q >= 1
    acc = np.empty((B, P, Q, N), dtype=np.int32)
    y = np.empty((B, P, Q, N), dtype=np.float64) if want_y else None
    lib().cdl_oracle_qconv_fwd(_ptr(x, _i16p), _ptr(w, _i16p), B, H, W, C, N, R, S, int(stride), int(pad),
                               float(delta_x), float(delta_w), _ptr(acc, _i32p), _ptr(y, _f64p))
    return acc, y


def qconv_bwd(g: np.ndarray, x_idx: np.ndarray, w_idx: np.ndarray, stride: int, pad: int, delta_x: float, delta_w: float,
              want_dx: bool = True, want_dw: bool = True):
    """g fp32[B,P,Q,N] -> (d_x_hat float64[B,H,W,C] | None, d_w_hat float64[N,R,S,C] | None)."""
    gg = _c(g, np.float32)
    x = _c(x_idx, np.int16)
    w = _c(w_idx, np.int16)
    B, H, W, C = x.shape
    N, R, S, C2 = w.shape
    P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
    assert C == C2 and gg.shape == (B, P, Q, N)
    dx = np.empty((B, H, W, C), dtype=np.float64) if want_dx else None
    dw = np.empty((N, R, S, C), dtype=np.float64) if want_dw else None
    lib().cdl_oracle_qconv_bwd(_ptr(gg, _f32p), _ptr(x, _i16p), _ptr(w, _i16p), B, H, W, C, N, R, S, int(stride), int(pad),
                               float(delta_x), float(delta_w), _ptr(dx, _f64p), _ptr(dw, _f64p))
    return dx, dw


def qgemm_bwd(g: np.ndarray, a_idx: np.ndarray, b_idx: np.ndarray, delta_a: float, delta_b: float,
              want_da: bool = True, want_db: bool = True):
    """g fp32[M,N] -> (d_a_hat float64[M,K] | None, d_b_hat float64[N,K] | None)."""
    gg = _c(g, np.float32)
    a = _c(a_idx, np.int16)
    b = _c(b_idx, np.int16)
    M, K = a.shape
    N, K2 = b.shape
    assert K == K2 and gg.shape == (M, N)
    da = np.empty((M, K), dtype=np.float64) if want_da else None
    db = np.empty((N, K), dtype=np.float64) if want_db else None
    lib().cdl_oracle_qgemm_bwd(_ptr(gg, _f32p), _ptr(a, _i16p), _ptr(b, _i16p), M, N, K,
                               float(delta_a), float(delta_b), _ptr(da, _f64p), _ptr(db, _f64p))
    return da, db
