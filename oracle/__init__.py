"""CPU oracle (binary64) for convolution on native points -- TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper over oracle/pcpp_oracle.c, which holds the definitions
(Sec. 3.2 triplet construction; Eq. (1), Sec. 3.3.3 gradients, Eq. (5)).  Only the
tests, the smoke check and the benchmark's cpu_baseline leg may import this
package; it never imports the GPU package and shares no code with it.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

from .build import LIB, build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build(force=False)
        L = ctypes.CDLL(path)
        i64, i32, f32 = ctypes.c_int64, ctypes.c_int, ctypes.c_float
        p = ctypes.c_void_p
        L.oracle_build_triplets.restype = i64
        L.oracle_build_triplets.argtypes = [p, i64, p, i64, f32, i32, p, p, p, i64, p]
        for name in ("oracle_mvmr_fwd", "oracle_mvmr_bwd_input", "oracle_mvmr_bwd_weight"):
            f = getattr(L, name)
            f.restype = None
            f.argtypes = [p, p, p, i64, i64, i32, i32, i32, p, p, p, i64]
        L.oracle_num_threads.restype = i32
        L.oracle_build_triplets_general.restype = i64
        L.oracle_build_triplets_general.argtypes = [p, p, p, p, i32, f32, i32, i32, p, p, p, i64, p]
        L.oracle_voxel_subsample.restype = i64
        L.oracle_voxel_subsample.argtypes = [p, i64, f32, p]
        _lib = L
    return _lib


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def _ptr(a):
    return ctypes.c_void_p(a.ctypes.data) if a is not None else None


def _f32xyz(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    assert a.ndim == 2 and a.shape[1] == 3
    return a


def count_triplets(in_xyz, out_xyz, radius, t) -> int:
    """|T| by brute force (Sec. 3.2 / fixed-radius search of Sec. 4.1)."""
    a, b = _f32xyz(in_xyz), _f32xyz(out_xyz)
    return int(lib().oracle_build_triplets(_ptr(a), len(a), _ptr(b), len(b), float(np.float32(radius)),
                                           int(t), None, None, None, 0, None))


def build_triplets(in_xyz, out_xyz, radius, t):
    """Brute-force triplet set in (k, o, i) order.

    Returns (tri_o, tri_i, tri_k int32 arrays, seg_offsets int64[K+1]).
    """
    a, b = _f32xyz(in_xyz), _f32xyz(out_xyz)
    r = float(np.float32(radius))
    n = int(lib().oracle_build_triplets(_ptr(a), len(a), _ptr(b), len(b), r, int(t),
                                        None, None, None, 0, None))
    K = int(t) ** 3
    o = np.empty(n, np.int32); i = np.empty(n, np.int32); k = np.empty(n, np.int32)
    seg = np.zeros(K + 1, np.int64)
    m = int(lib().oracle_build_triplets(_ptr(a), len(a), _ptr(b), len(b), r, int(t),
                                        _ptr(o), _ptr(i), _ptr(k), n, _ptr(seg)))
    assert m == n
    return o, i, k, seg


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def mvmr_fwd(x, w, tri_o, tri_i, tri_k, n_out):
    """Eq. (1): out[o] = sum_{(o,i,k) in T} W[k] x[i]; x [n_in,c_in], w [K,c_out,c_in] -> float64 [n_out,c_out]."""
    x, w = _f64(x), _f64(w)
    K, c_out, c_in = w.shape
    assert x.shape[1] == c_in
    o, i, k = _i32(tri_o), _i32(tri_i), _i32(tri_k)
    out = np.empty((n_out, c_out), np.float64)
    lib().oracle_mvmr_fwd(_ptr(x), _ptr(w), _ptr(out), x.shape[0], n_out, c_in, c_out, K,
                          _ptr(o), _ptr(i), _ptr(k), len(o))
    return out


def mvmr_bwd_input(dy, w, tri_o, tri_i, tri_k, n_in):
    """Sec. 3.3.3: dx[i] = sum_{(o,i,k) in T} W[k]^T dy[o] -> float64 [n_in,c_in]."""
    dy, w = _f64(dy), _f64(w)
    K, c_out, c_in = w.shape
    assert dy.shape[1] == c_out
    o, i, k = _i32(tri_o), _i32(tri_i), _i32(tri_k)
    dx = np.empty((n_in, c_in), np.float64)
    lib().oracle_mvmr_bwd_input(_ptr(dy), _ptr(w), _ptr(dx), n_in, dy.shape[0], c_in, c_out, K,
                                _ptr(o), _ptr(i), _ptr(k), len(o))
    return dx


def mvmr_bwd_weight(x, dy, tri_o, tri_i, tri_k, K):
    """Eq. (5): dW[k] = sum_{(o,i,k) in T} dy[o] (outer) x[i] -> float64 [K,c_out,c_in]."""
    x, dy = _f64(x), _f64(dy)
    c_in, c_out = x.shape[1], dy.shape[1]
    o, i, k = _i32(tri_o), _i32(tri_i), _i32(tri_k)
    dw = np.empty((K, c_out, c_in), np.float64)
    lib().oracle_mvmr_bwd_weight(_ptr(x), _ptr(dy), _ptr(dw), x.shape[0], dy.shape[0], c_in, c_out, K,
                                 _ptr(o), _ptr(i), _ptr(k), len(o))
    return dw


MODE_BALL, MODE_VOXEL = 0, 1


def build_triplets_general(in_xyz, out_xyz, size, t, mode=MODE_BALL, in_offsets=None, out_offsets=None):
    """Triplets over a batch of clouds (offsets into the concatenated arrays; None = one cloud), in ball mode
    (size = radius, Sec. 3.2 "Definition") or voxel mode (size = voxel pitch, the degraded operator of Sec. 3.2
    "Voxel Convolution as a Special Case").  Returns (tri_o, tri_i, tri_k, seg_offsets) in (k, o, i) order."""
    a, b = _f32xyz(in_xyz), _f32xyz(out_xyz)
    io = np.ascontiguousarray([0, len(a)] if in_offsets is None else in_offsets, dtype=np.int64)
    oo = np.ascontiguousarray([0, len(b)] if out_offsets is None else out_offsets, dtype=np.int64)
    assert len(io) == len(oo) and io[0] == 0 and oo[0] == 0 and io[-1] == len(a) and oo[-1] == len(b)
    nb = len(io) - 1
    sz = float(np.float32(size))
    args = (_ptr(a), _ptr(b), _ptr(io), _ptr(oo), nb, sz, int(t), int(mode))
    n = int(lib().oracle_build_triplets_general(*args, None, None, None, 0, None))
    if n < 0:
        raise ValueError("voxel mode needs an odd t")
    K = int(t) ** 3
    o = np.empty(n, np.int32); i = np.empty(n, np.int32); k = np.empty(n, np.int32)
    seg = np.zeros(K + 1, np.int64)
    m = int(lib().oracle_build_triplets_general(*args, _ptr(o), _ptr(i), _ptr(k), n, _ptr(seg)))
    assert m == n
    return o, i, k, seg


def voxel_subsample(xyz, pitch):
    """Indices (ascending) of the lowest-index point of every occupied voxel of the given pitch (Sec. 4.1)."""
    a = _f32xyz(xyz)
    kept = np.empty(len(a), np.int32)
    m = int(lib().oracle_voxel_subsample(_ptr(a), len(a), float(np.float32(pitch)), _ptr(kept)))
    return kept[:m].copy()
