"""ctypes binding of libpcpp.so: argument marshalling only (torch tensors -> device pointers)."""
from __future__ import annotations

import ctypes
import os
import threading
from dataclasses import dataclass

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libpcpp.so")

PCPP_F32, PCPP_BF16 = 0, 1
PLAN_FWD, PLAN_BWD_INPUT, PLAN_SPATIAL = 1, 2, 4
BUILD_TEST_SHORT_LISTS, BUILD_TEST_WIDE_KEYS, BUILD_VOXEL = 0x100, 0x200, 0x400
PLAN_MASK = PLAN_FWD | PLAN_BWD_INPUT | PLAN_SPATIAL
ERR_CAPACITY = -2

EXPORTS = ("pcpp_last_error", "pcpp_version", "pcpp_build_triplets_workspace_bytes",
           "pcpp_build_triplets_workspace_bytes_for", "pcpp_plan_bytes",
           "pcpp_build_triplets", "pcpp_mvmr_workspace_bytes", "pcpp_mvmr_fwd", "pcpp_mvmr_bwd_input",
           "pcpp_mvmr_bwd_weight", "pcpp_static_scratch_bytes", "pcpp_mvmr_fwd_static",
           "pcpp_build_triplets_batched", "pcpp_voxel_subsample_workspace_bytes", "pcpp_voxel_subsample")


class PcppError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"pcpp error {code}: {message}")
        self.code = code


_lib = None


def library() -> ctypes.CDLL:
    """Load libpcpp.so (building it first only if no built library exists).  Raises if unavailable."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        from .build import build
        build()
    L = ctypes.CDLL(LIB_PATH)
    i64, i32, f32, vp, sz = ctypes.c_int64, ctypes.c_int, ctypes.c_float, ctypes.c_void_p, ctypes.c_size_t
    L.pcpp_last_error.restype = ctypes.c_char_p
    L.pcpp_last_error.argtypes = []
    L.pcpp_version.restype = i32
    L.pcpp_build_triplets_workspace_bytes.restype = sz
    L.pcpp_build_triplets_workspace_bytes.argtypes = [i64, i64, i32]
    L.pcpp_build_triplets_workspace_bytes_for.restype = sz
    L.pcpp_build_triplets_workspace_bytes_for.argtypes = [i64, i64, i32, i64]
    L.pcpp_plan_bytes.restype = sz
    L.pcpp_plan_bytes.argtypes = [i64, i64, i32, i64, i32]
    L.pcpp_build_triplets.restype = i32
    L.pcpp_build_triplets.argtypes = [vp, i64, vp, i64, f32, i32, vp, vp, vp, i64, vp,
                                      ctypes.POINTER(i64), vp, sz, i32, vp, sz, vp]
    L.pcpp_build_triplets_batched.restype = i32
    L.pcpp_build_triplets_batched.argtypes = [vp, i64, vp, i64, vp, vp, i32, f32, i32, vp, vp, vp, i64, vp,
                                              ctypes.POINTER(i64), vp, sz, i32, vp, sz, vp]
    L.pcpp_voxel_subsample_workspace_bytes.restype = sz
    L.pcpp_voxel_subsample_workspace_bytes.argtypes = [i64]
    L.pcpp_voxel_subsample.restype = i32
    L.pcpp_voxel_subsample.argtypes = [vp, i64, f32, vp, ctypes.POINTER(i64), vp, sz, vp]
    L.pcpp_mvmr_workspace_bytes.restype = sz
    L.pcpp_mvmr_workspace_bytes.argtypes = [i32, i64, i64, i64, i32, i32, i32, i32]
    head = [i64, i64, i32, i32, i32, vp, vp, vp, vp, i64, vp, sz, i32]     # sizes, triplets, plan
    tail = head + [vp, sz, vp]                                             # workspace, stream
    L.pcpp_mvmr_fwd.restype = i32
    L.pcpp_mvmr_fwd.argtypes = [vp, vp, vp, i32, i32] + tail
    L.pcpp_mvmr_bwd_input.restype = i32
    L.pcpp_mvmr_bwd_input.argtypes = [vp, vp, vp, i32, i32] + tail
    L.pcpp_mvmr_bwd_weight.restype = i32
    L.pcpp_mvmr_bwd_weight.argtypes = [vp, vp, vp, i32] + tail
    L.pcpp_tune_workspace_bytes.restype = sz
    L.pcpp_tune_workspace_bytes.argtypes = [i64, i64, i32, i64, i32, i32, i32, i32]
    L.pcpp_tune_plan_order.restype = i32
    L.pcpp_tune_plan_order.argtypes = [vp, i64, vp, i64, f32, i32, i32, i64, i32, i32, i32, i32, vp, sz,
                                       ctypes.POINTER(i32), ctypes.POINTER(f32), ctypes.POINTER(f32), vp]
    L.pcpp_static_scratch_bytes.restype = sz
    L.pcpp_static_scratch_bytes.argtypes = []
    L.pcpp_mvmr_fwd_static.restype = i32
    L.pcpp_mvmr_fwd_static.argtypes = [vp, vp, vp, i32, i32] + head + [vp]
    _lib = L
    return L


_landing = threading.local()


def _landing_word():
    """Pinned host word that pcpp_build_triplets lets the device write |T| into (one per host thread)."""
    if getattr(_landing, "word", None) is None:
        _landing.word = torch.zeros(8, dtype=torch.int64, pin_memory=True)
    return _landing.word


def _check(rc: int):
    if rc != 0:
        raise PcppError(rc, library().pcpp_last_error().decode())


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else None


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return PCPP_F32
    if t.dtype == torch.bfloat16:
        return PCPP_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _bytes(n: int, device) -> torch.Tensor:
    return torch.empty(max(int(n), 256), dtype=torch.uint8, device=device)


@dataclass
class Triplets:
    """Result of pcpp_build_triplets: T in (k, o, i) order plus the plan the compute calls read."""
    tri_o: torch.Tensor
    tri_i: torch.Tensor
    tri_k: torch.Tensor
    seg_offsets: torch.Tensor
    n_triplets: int
    n_in: int
    n_out: int
    t: int
    plan: torch.Tensor
    plan_flags: int

    @property
    def K(self) -> int:
        return self.t ** 3


def pcpp_count_triplets(in_xyz: torch.Tensor, out_xyz: torch.Tensor, radius: float, t: int,
                        workspace: torch.Tensor | None = None) -> int:
    L = library()
    n_in, n_out = in_xyz.shape[0], out_xyz.shape[0]
    ws_bytes = L.pcpp_build_triplets_workspace_bytes(n_in, n_out, t)
    ws = workspace if workspace is not None else _bytes(ws_bytes, in_xyz.device)
    n = _landing_word()
    _check(L.pcpp_build_triplets(_ptr(in_xyz), n_in, _ptr(out_xyz), n_out, float(radius), int(t), None, None, None,
                                 0, None, ctypes.cast(n.data_ptr(), ctypes.POINTER(ctypes.c_int64)), None, 0, 0,
                                 _ptr(ws), ws.numel(), _stream()))
    return int(n[0])


def pcpp_build_triplets(in_xyz: torch.Tensor, out_xyz: torch.Tensor, radius: float, t: int,
                        plan_flags: int = PLAN_FWD | PLAN_BWD_INPUT, capacity: int | None = None,
                        buffers: dict | None = None, in_offsets: torch.Tensor | None = None,
                        out_offsets: torch.Tensor | None = None) -> Triplets:
    """Triplet construction (Sec. 3.2 with the fixed-radius search of Sec. 4.1) and reordering by (k, o, i).

    in_xyz [n_in,3], out_xyz [n_out,3]: contiguous float32 CUDA tensors.  Without `capacity` room for 48
    triplets per output point is provided; if that is too little the call reports the exact count and is
    repeated once with it (so the search runs once in the common case).  `buffers` may carry preallocated
    'tri_o','tri_i','tri_k','seg_offsets','plan','workspace' tensors to reuse.  plan_flags may include
    PLAN_SPATIAL (tiles follow a space-filling order; for wide layers), BUILD_VOXEL (the degraded, sparse-voxel
    operator of Sec. 3.2: `radius` is the voxel pitch) and the BUILD_TEST_* aids.  in_offsets / out_offsets: int32
    CUDA tensors [n_batches + 1] for a batch of clouds held as concatenated arrays (Sec. 4.1).
    """
    if capacity is None:
        guess = max(48 * int(out_xyz.shape[0]), 1024)
        try:
            return pcpp_build_triplets(in_xyz, out_xyz, radius, t, plan_flags, guess, buffers, in_offsets, out_offsets)
        except PcppError as e:
            if e.code != ERR_CAPACITY:
                raise
            return pcpp_build_triplets(in_xyz, out_xyz, radius, t, plan_flags, e.needed, buffers, in_offsets, out_offsets)
    L = library()
    assert in_xyz.is_cuda and out_xyz.is_cuda and in_xyz.dtype == torch.float32 and out_xyz.dtype == torch.float32
    assert in_xyz.is_contiguous() and out_xyz.is_contiguous()
    dev = in_xyz.device
    n_in, n_out = int(in_xyz.shape[0]), int(out_xyz.shape[0])
    K = t ** 3
    buffers = buffers or {}
    ws_bytes = L.pcpp_build_triplets_workspace_bytes(n_in, n_out, t)
    if ws_bytes == 0:
        raise PcppError(-1, "invalid sizes or t")
    ws = buffers.get("workspace")
    cap = max(int(capacity), 1)
    # room for the neighbour lists that let the second pass skip its search
    ws_bytes = max(ws_bytes, L.pcpp_build_triplets_workspace_bytes_for(n_in, n_out, t, cap))
    if ws is None or ws.numel() < ws_bytes:
        ws = _bytes(ws_bytes, dev)

    def buf(name, numel, dtype):
        b = buffers.get(name)
        if b is None or b.numel() < numel or b.dtype != dtype:
            b = torch.empty(numel, dtype=dtype, device=dev)
        return b

    tri_o, tri_i, tri_k = (buf(nm, cap, torch.int32) for nm in ("tri_o", "tri_i", "tri_k"))
    seg = buf("seg_offsets", K + 1, torch.int64)
    want_plan = bool(plan_flags & PLAN_MASK)
    plan_bytes = L.pcpp_plan_bytes(n_in, n_out, t, cap, plan_flags & PLAN_MASK) if want_plan else 0
    plan = buffers.get("plan")
    if want_plan and (plan is None or plan.numel() < plan_bytes):
        plan = _bytes(plan_bytes, dev)
    n = _landing_word()
    n_batches = 1
    if in_offsets is not None or out_offsets is not None:
        assert in_offsets is not None and out_offsets is not None and in_offsets.is_cuda and out_offsets.is_cuda
        assert in_offsets.dtype == torch.int32 and out_offsets.dtype == torch.int32
        assert in_offsets.numel() == out_offsets.numel() >= 2
        n_batches = in_offsets.numel() - 1
    rc = L.pcpp_build_triplets_batched(_ptr(in_xyz), n_in, _ptr(out_xyz), n_out, _ptr(in_offsets), _ptr(out_offsets),
                                       n_batches, float(radius), int(t),
                                       _ptr(tri_o), _ptr(tri_i), _ptr(tri_k), cap, _ptr(seg),
                                       ctypes.cast(n.data_ptr(), ctypes.POINTER(ctypes.c_int64)),
                                       _ptr(plan) if want_plan else None, plan.numel() if want_plan else 0, plan_flags,
                                       _ptr(ws), ws.numel(), _stream())
    nt = int(n[0])
    if rc == ERR_CAPACITY:
        err = PcppError(rc, f"capacity {cap} too small, need {nt}")
        err.needed = nt
        raise err
    _check(rc)
    return Triplets(tri_o[:nt], tri_i[:nt], tri_k[:nt], seg[:K + 1], nt, n_in, n_out, t, plan, plan_flags & PLAN_MASK)


def pcpp_voxel_subsample(xyz: torch.Tensor, pitch: float) -> torch.Tensor:
    """Voxel-grid down-sampling that keeps original coordinates (Sec. 4.1): indices (ascending, int32) of the
    lowest-index point of every occupied voxel of the given pitch."""
    L = library()
    assert xyz.is_cuda and xyz.is_contiguous() and xyz.dtype == torch.float32
    n = int(xyz.shape[0])
    kept = torch.empty(max(n, 1), dtype=torch.int32, device=xyz.device)
    ws = _bytes(L.pcpp_voxel_subsample_workspace_bytes(n), xyz.device)
    cnt = _landing_word()
    _check(L.pcpp_voxel_subsample(_ptr(xyz), n, float(pitch), _ptr(kept),
                                  ctypes.cast(cnt.data_ptr(), ctypes.POINTER(ctypes.c_int64)), _ptr(ws), ws.numel(),
                                  _stream()))
    return kept[:int(cnt[0])]


def pcpp_tune_plan_order(in_xyz: torch.Tensor, out_xyz: torch.Tensor, radius: float, t: int, n_triplets: int,
                         c_in: int, c_out: int, dtype: torch.dtype, ops: int = PLAN_FWD | PLAN_BWD_INPUT,
                         build_flags: int = 0) -> tuple[int, float, float]:
    """The plan order (Sec. 3.3.2, closing remark on auto-tuning) that runs this layer faster on this cloud:
    returns (plan flags to build with, ms per pass in index order, ms per pass in spatial order)."""
    L = library()
    assert in_xyz.is_cuda and in_xyz.is_contiguous() and out_xyz.is_contiguous() and in_xyz.dtype == torch.float32
    n_in, n_out = int(in_xyz.shape[0]), int(out_xyz.shape[0])
    code = 1 if dtype == torch.bfloat16 else 0
    ws = _bytes(L.pcpp_tune_workspace_bytes(n_in, n_out, t, n_triplets, c_in, c_out, code, ops), in_xyz.device)
    best, ms_a, ms_b = ctypes.c_int32(0), ctypes.c_float(0), ctypes.c_float(0)
    _check(L.pcpp_tune_plan_order(_ptr(in_xyz), n_in, _ptr(out_xyz), n_out, float(radius), t, build_flags, n_triplets,
                                  c_in, c_out, code, ops, _ptr(ws), ws.numel(), ctypes.byref(best), ctypes.byref(ms_a),
                                  ctypes.byref(ms_b), _stream()))
    return int(best.value), float(ms_a.value), float(ms_b.value)


def _plan_args(T: Triplets):
    if T.plan is None:
        return None, 0, T.plan_flags
    return _ptr(T.plan), T.plan.numel(), T.plan_flags


def _mvmr_ws(op, T: Triplets, c_in, c_out, code, dev, workspace):
    need = library().pcpp_mvmr_workspace_bytes(op, T.n_in, T.n_out, T.n_triplets, c_in, c_out, T.K, code)
    if workspace is None or workspace.numel() < need:
        workspace = _bytes(need, dev)
    return workspace


def pcpp_mvmr_fwd(x: torch.Tensor, w: torch.Tensor, T: Triplets, out: torch.Tensor | None = None,
                  out_dtype: torch.dtype = torch.float32, workspace: torch.Tensor | None = None) -> torch.Tensor:
    """Eq. (1): out[o] = sum_{(o,i,k) in T} W[k] x[i];  x [n_in,c_in], w [K,c_out,c_in] -> out [n_out,c_out]."""
    L = library()
    assert x.is_cuda and x.is_contiguous() and w.is_contiguous() and x.dtype == w.dtype
    K, c_out, c_in = w.shape
    assert K == T.K and x.shape == (T.n_in, c_in)
    if out is None:
        out = torch.empty((T.n_out, c_out), dtype=out_dtype, device=x.device)
    ws = _mvmr_ws(0, T, c_in, c_out, _dtype_code(x), x.device, workspace)
    _check(L.pcpp_mvmr_fwd(_ptr(x), _ptr(w), _ptr(out), _dtype_code(x), _dtype_code(out), T.n_in, T.n_out, c_in, c_out,
                           K, _ptr(T.tri_o), _ptr(T.tri_i), _ptr(T.tri_k), _ptr(T.seg_offsets), T.n_triplets,
                           *_plan_args(T), _ptr(ws), ws.numel(), _stream()))
    return out


def pcpp_mvmr_fwd_static(x: torch.Tensor, w: torch.Tensor, T: Triplets, out: torch.Tensor,
                         out_dtype: torch.dtype = torch.float32) -> torch.Tensor:
    """pcpp_mvmr_fwd without a workspace: the packed weights go to the library's own device array, and the call
    allocates nothing (`out` must be given)."""
    L = library()
    assert x.is_cuda and x.is_contiguous() and w.is_contiguous() and x.dtype == w.dtype
    K, c_out, c_in = w.shape
    assert K == T.K and x.shape == (T.n_in, c_in) and out.shape == (T.n_out, c_out)
    _check(L.pcpp_mvmr_fwd_static(_ptr(x), _ptr(w), _ptr(out), _dtype_code(x), _dtype_code(out), T.n_in, T.n_out, c_in,
                                  c_out, K, _ptr(T.tri_o), _ptr(T.tri_i), _ptr(T.tri_k), _ptr(T.seg_offsets),
                                  T.n_triplets, *_plan_args(T), _stream()))
    return out


def pcpp_mvmr_bwd_input(dy: torch.Tensor, w: torch.Tensor, T: Triplets, dx: torch.Tensor | None = None,
                        out_dtype: torch.dtype = torch.float32, workspace: torch.Tensor | None = None) -> torch.Tensor:
    """Sec. 3.3.3: dx[i] = sum_{(o,i,k) in T} W[k]^T dy[o];  dy [n_out,c_out] -> dx [n_in,c_in]."""
    L = library()
    assert dy.is_cuda and dy.is_contiguous() and w.is_contiguous() and dy.dtype == w.dtype
    K, c_out, c_in = w.shape
    assert K == T.K and dy.shape == (T.n_out, c_out)
    if not (T.plan_flags & PLAN_BWD_INPUT):
        raise PcppError(-1, "triplets were built without PLAN_BWD_INPUT")
    if dx is None:
        dx = torch.empty((T.n_in, c_in), dtype=out_dtype, device=dy.device)
    ws = _mvmr_ws(1, T, c_in, c_out, _dtype_code(dy), dy.device, workspace)
    _check(L.pcpp_mvmr_bwd_input(_ptr(dy), _ptr(w), _ptr(dx), _dtype_code(dy), _dtype_code(dx), T.n_in, T.n_out, c_in,
                                 c_out, K, _ptr(T.tri_o), _ptr(T.tri_i), _ptr(T.tri_k), _ptr(T.seg_offsets),
                                 T.n_triplets, *_plan_args(T), _ptr(ws), ws.numel(), _stream()))
    return dx


def pcpp_mvmr_bwd_weight(x: torch.Tensor, dy: torch.Tensor, T: Triplets, dw: torch.Tensor | None = None,
                         workspace: torch.Tensor | None = None) -> torch.Tensor:
    """Eq. (5): dW[k] = sum_{(o,i,k) in T} dy[o] (outer) x[i] -> float32 [K,c_out,c_in]."""
    L = library()
    assert x.is_cuda and x.is_contiguous() and dy.is_contiguous() and x.dtype == dy.dtype
    c_in, c_out = x.shape[1], dy.shape[1]
    assert x.shape[0] == T.n_in and dy.shape[0] == T.n_out
    if dw is None:
        dw = torch.empty((T.K, c_out, c_in), dtype=torch.float32, device=x.device)
    ws = _mvmr_ws(2, T, c_in, c_out, _dtype_code(x), x.device, workspace)
    _check(L.pcpp_mvmr_bwd_weight(_ptr(x), _ptr(dy), _ptr(dw), _dtype_code(x), T.n_in, T.n_out, c_in, c_out, T.K,
                                  _ptr(T.tri_o), _ptr(T.tri_i), _ptr(T.tri_k), _ptr(T.seg_offsets), T.n_triplets,
                                  *_plan_args(T), _ptr(ws), ws.numel(), _stream()))
    return dw
