"""Thin Python binding of libdepsync.so (argument marshalling only).

Every step of a chain runs in the library's HIP kernels; this module only turns torch
tensors into device pointers and streams into hipStream_t handles, and mirrors the names of
include/depsync.h.  There is no fallback: if the shared library is missing or a call fails,
an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libdepsync.so")

# enums of include/depsync.h
ROWSYNC, TILESYNC, STRIDEDSYNC, AUTOSYNC = 0, 1, 2, 3
MODE_FINE, MODE_STREAMSYNC, MODE_PLAIN, MODE_FUSED = 0, 1, 2, 3
MID_NONE, MID_GELU, MID_RELU, MID_SWIGLU, MID_CAUSAL_ATTN = 0, 1, 2, 3, 4
BF16, FP16 = 0, 1
(TILE_AUTO, TILE_256x256, TILE_256x128, TILE_128x256, TILE_128x128, TILE_64x128, TILE_64x64,
 TILE_256x192, TILE_128x192, TILE_256x64, TILE_64x64_DEEP, TILE_64x192, TILE_128x192_DEEP, TILE_128x128_DEEP) = range(14)
W_ROWS, W_KBLOCKED = 0, 1
FLAG_NO_REORDER, FLAG_COUNT, FLAG_REVERSE_ORDER, FLAG_HW_ORDER, FLAG_TRACE, FLAG_QUEUE_ORDER = 1, 2, 4, 8, 16, 32
OK, EINVAL, ENOMEM, EHIP, ETIMEOUT, ENOTIMPL, ELIMIT = 0, -1, -2, -3, -4, -5, -6

EXPORTS = [
    "sync_policy_create", "sync_policy_destroy", "dep_chain_reset", "depsync_last_status", "depsync_read_trace",
    "dep_gemm_chain", "dep_conv_chain", "depsync_gemm_chain_plan", "depsync_conv_chain_plan",
    "depsync_row_major", "depsync_policy_sem", "depsync_policy_value", "depsync_wave_model",
    "depsync_sync_count", "depsync_simulate_chain", "depsync_strerror", "depsync_last_hip_error",
    "depsync_tile_shape", "depsync_device_info", "depsync_gemm_chain_autotune", "depsync_conv_chain_autotune",
    "depsync_gemm_chain_tuned", "depsync_conv_chain_tuned", "depsync_gemm_chain_set_tuned", "depsync_conv_chain_set_tuned",
    "depsync_mfma_calibration", "dep_copy_chain", "depsync_copy_chain_plan",
    "dep_conv_chain_n", "depsync_conv_chain_n_plan", "depsync_conv_chain_n_autotune", "depsync_workspace_bytes",
    "depsync_gemm_chain_check_waits", "depsync_conv_chain_n_check_waits", "dep_gemm_chain_static",
    "depsync_gemm_chain_autotune_policy", "depsync_conv_chain_n_autotune_policy", "depsync_gemm_chain_policy",
    "depsync_conv_chain_n_policy",
]


class DepsyncError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        msg = _lib().depsync_strerror(status).decode()
        if status == EHIP:
            msg += f" [hip error {_lib().depsync_last_hip_error()}]"
        super().__init__(f"{what}: {msg} ({status})")


class PolicyParams(ctypes.Structure):
    _fields_ = [("stride", ctypes.c_uint32), ("count", ctypes.c_uint32), ("flags", ctypes.c_uint32),
                ("spin_limit", ctypes.c_uint32), ("delay_tile", ctypes.c_uint32),
                ("delay_iters", ctypes.c_uint32), ("ksplit", ctypes.c_uint32)]


class Status(ctypes.Structure):
    _fields_ = [("timed_out", ctypes.c_int32), ("first_timeout", ctypes.c_int32),
                ("posts", ctypes.c_uint32), ("waits", ctypes.c_uint32),
                ("polling_waits", ctypes.c_uint32), ("launches", ctypes.c_uint32)]


class TraceRec(ctypes.Structure):
    _fields_ = [("rel", ctypes.c_uint32), ("where", ctypes.c_uint32), ("tx", ctypes.c_uint32), ("ty", ctypes.c_uint32),
                ("t_enter", ctypes.c_uint64), ("t_start", ctypes.c_uint64), ("t_ready", ctypes.c_uint64), ("t_end", ctypes.c_uint64)]


class PlanInfo(ctypes.Structure):
    _fields_ = [("tile_prod", ctypes.c_int32), ("tile_mid", ctypes.c_int32), ("tile_cons", ctypes.c_int32),
                ("prod_grid_x", ctypes.c_int32), ("prod_grid_y", ctypes.c_int32),
                ("mid_grid_x", ctypes.c_int32), ("mid_grid_y", ctypes.c_int32),
                ("cons_grid_x", ctypes.c_int32), ("cons_grid_y", ctypes.c_int32),
                ("n_prod", ctypes.c_int32), ("n_mid", ctypes.c_int32), ("n_cons", ctypes.c_int32),
                ("n_sems", ctypes.c_int32), ("slots", ctypes.c_int32),
                ("waves_streamsync", ctypes.c_int32), ("waves_fine", ctypes.c_int32),
                ("flops", ctypes.c_double), ("bytes", ctypes.c_double)]

    def as_dict(self):
        return {k: getattr(self, k) for k, _ in self._fields_}


class GemmChainDesc(ctypes.Structure):
    _fields_ = [("M", ctypes.c_int32), ("K1", ctypes.c_int32), ("N1", ctypes.c_int32), ("N2", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("mid", ctypes.c_int32),
                ("X", ctypes.c_void_p), ("ldx", ctypes.c_int64),
                ("W1t", ctypes.c_void_p), ("ldw1", ctypes.c_int64),
                ("H", ctypes.c_void_p), ("ldh", ctypes.c_int64),
                ("W2t", ctypes.c_void_p), ("ldw2", ctypes.c_int64),
                ("Y", ctypes.c_void_p), ("ldy", ctypes.c_int64),
                ("T", ctypes.c_void_p), ("ldt", ctypes.c_int64),
                ("batch", ctypes.c_int32), ("seq", ctypes.c_int32), ("heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32),
                ("tile_prod", ctypes.c_int32), ("tile_cons", ctypes.c_int32), ("w_layout", ctypes.c_int32),
                ("k_cache", ctypes.c_void_p), ("v_cache", ctypes.c_void_p), ("ld_cache", ctypes.c_int64),
                ("cached", ctypes.c_int32)]


class ConvChainDesc(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("W", ctypes.c_int32), ("C", ctypes.c_int32),
                ("K1", ctypes.c_int32), ("K2", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("inp", ctypes.c_void_p), ("w1", ctypes.c_void_p), ("mid", ctypes.c_void_p),
                ("w2", ctypes.c_void_p), ("out", ctypes.c_void_p),
                ("tile_prod", ctypes.c_int32), ("tile_cons", ctypes.c_int32)]


class ConvChainNDesc(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("W", ctypes.c_int32), ("C", ctypes.c_int32),
                ("n", ctypes.c_int32), ("K", ctypes.c_int32 * 4), ("dtype", ctypes.c_int32),
                ("inp", ctypes.c_void_p), ("w", ctypes.c_void_p * 4), ("out", ctypes.c_void_p * 4),
                ("tile_prod", ctypes.c_int32), ("tile_cons", ctypes.c_int32)]


class CopyChainDesc(ctypes.Structure):
    _fields_ = [("src", ctypes.c_void_p), ("mid", ctypes.c_void_p), ("dst", ctypes.c_void_p),
                ("bytes", ctypes.c_uint64), ("tile_bytes", ctypes.c_uint32)]


_LIB = None


def _lib() -> ctypes.CDLL:
    global _LIB
    if _LIB is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it first (python -m paper_2305_13450_amd.build or "
                "__graft_entry__.build()); there is no fallback path")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32 = ctypes.c_void_p, ctypes.c_int
        L.sync_policy_create.argtypes = [i32, ctypes.POINTER(PolicyParams), ctypes.POINTER(vp)]
        L.sync_policy_destroy.argtypes = [vp]
        L.dep_chain_reset.argtypes = [vp, vp]
        L.depsync_last_status.argtypes = [vp, ctypes.POINTER(Status)]
        L.depsync_read_trace.argtypes = [vp, ctypes.POINTER(TraceRec), i32]
        L.dep_gemm_chain.argtypes = [ctypes.POINTER(GemmChainDesc), vp, i32, vp, vp]
        L.dep_conv_chain.argtypes = [ctypes.POINTER(ConvChainDesc), vp, i32, vp, vp]
        L.depsync_gemm_chain_plan.argtypes = [ctypes.POINTER(GemmChainDesc), vp, i32, ctypes.POINTER(PlanInfo)]
        L.depsync_conv_chain_plan.argtypes = [ctypes.POINTER(ConvChainDesc), vp, i32, ctypes.POINTER(PlanInfo)]
        L.depsync_gemm_chain_autotune.argtypes = [ctypes.POINTER(GemmChainDesc), vp, vp, i32, ctypes.POINTER(i32)]
        L.depsync_conv_chain_autotune.argtypes = [ctypes.POINTER(ConvChainDesc), vp, vp, i32, ctypes.POINTER(i32)]
        L.dep_conv_chain_n.argtypes = [ctypes.POINTER(ConvChainNDesc), vp, i32, vp, vp]
        L.depsync_conv_chain_n_plan.argtypes = [ctypes.POINTER(ConvChainNDesc), vp, i32, ctypes.POINTER(PlanInfo)]
        L.depsync_conv_chain_n_autotune.argtypes = [ctypes.POINTER(ConvChainNDesc), vp, vp, i32, ctypes.POINTER(i32)]
        L.dep_copy_chain.argtypes = [ctypes.POINTER(CopyChainDesc), vp, i32, vp, vp]
        L.depsync_copy_chain_plan.argtypes = [ctypes.POINTER(CopyChainDesc), vp, i32, ctypes.POINTER(PlanInfo)]
        L.depsync_mfma_calibration.argtypes = [i32, i32, ctypes.POINTER(ctypes.c_double)]
        L.depsync_gemm_chain_tuned.argtypes = [ctypes.POINTER(GemmChainDesc), vp, ctypes.POINTER(i32), ctypes.POINTER(i32)]
        L.depsync_conv_chain_tuned.argtypes = [ctypes.POINTER(ConvChainDesc), vp, ctypes.POINTER(i32), ctypes.POINTER(i32)]
        L.depsync_gemm_chain_set_tuned.argtypes = [ctypes.POINTER(GemmChainDesc), vp, i32, i32]
        L.depsync_conv_chain_set_tuned.argtypes = [ctypes.POINTER(ConvChainDesc), vp, i32, i32]
        i64p = ctypes.POINTER(ctypes.c_int64)
        L.depsync_gemm_chain_check_waits.argtypes = [ctypes.POINTER(GemmChainDesc), i32, ctypes.POINTER(PolicyParams), i32, i64p]
        L.depsync_conv_chain_n_check_waits.argtypes = [ctypes.POINTER(ConvChainNDesc), i32, ctypes.POINTER(PolicyParams), i32, i64p]
        f3 = ctypes.POINTER(ctypes.c_float)
        L.depsync_gemm_chain_autotune_policy.argtypes = [ctypes.POINTER(GemmChainDesc), vp, vp, i32, ctypes.POINTER(i32), ctypes.POINTER(i32), f3]
        L.depsync_conv_chain_n_autotune_policy.argtypes = [ctypes.POINTER(ConvChainNDesc), vp, vp, i32, ctypes.POINTER(i32), ctypes.POINTER(i32), f3]
        L.depsync_gemm_chain_policy.argtypes = [ctypes.POINTER(GemmChainDesc), vp, ctypes.POINTER(i32)]
        L.depsync_conv_chain_n_policy.argtypes = [ctypes.POINTER(ConvChainNDesc), vp, ctypes.POINTER(i32)]
        L.dep_gemm_chain_static.argtypes = [ctypes.POINTER(GemmChainDesc), i32, ctypes.POINTER(PolicyParams), vp]
        L.depsync_row_major.argtypes = [i32] * 4
        L.depsync_policy_sem.argtypes = [i32] * 6
        L.depsync_policy_value.argtypes = [i32] * 4
        L.depsync_wave_model.argtypes = [i32, i32, i32, ctypes.POINTER(i32), ctypes.POINTER(ctypes.c_double)]
        L.depsync_sync_count.argtypes = [i32] * 6
        L.depsync_simulate_chain.argtypes = [i32, i32, i32, ctypes.c_double, i32, i32, ctypes.c_double, i32, i32]
        L.depsync_simulate_chain.restype = ctypes.c_double
        L.depsync_strerror.argtypes = [i32]
        L.depsync_strerror.restype = ctypes.c_char_p
        L.depsync_last_hip_error.argtypes = []
        L.depsync_tile_shape.argtypes = [i32, ctypes.POINTER(i32), ctypes.POINTER(i32)]
        L.depsync_device_info.argtypes = [ctypes.POINTER(i32), ctypes.POINTER(i32)]
        _LIB = L
    return _LIB


def _check(status: int, what: str) -> None:
    if status != OK:
        raise DepsyncError(status, what)


def _stream_handle(stream) -> Optional[int]:
    """torch.cuda.Stream | raw handle | None -> hipStream_t as an integer (None = NULL)."""
    if stream is None:
        return None
    if hasattr(stream, "cuda_stream"):
        return int(stream.cuda_stream) or None
    return int(stream) or None


def _tile_pair(tile):
    """A macro-tile id for every stage, or a (producer, consumer) pair of ids."""
    if isinstance(tile, (tuple, list)):
        prod, cons = tile
        return int(prod), int(cons)
    return int(tile), int(tile)


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float16:
        return FP16
    raise TypeError(f"unsupported element type {t.dtype}")


def _dev2d(t, name: str):
    if not t.is_cuda:
        raise ValueError(f"{name} must be a device tensor")
    if t.dim() != 2 or t.stride(1) != 1:
        raise ValueError(f"{name} must be 2-D with contiguous rows")
    return t.data_ptr(), t.stride(0)


class SyncPolicy:
    """Owner of a sync_policy_t (policy kind + semaphore workspace)."""

    def __init__(self, kind: int, stride: int = 0, count: int = 0, flags: int = 0, spin_limit: int = 0,
                 delay_tile: int = 0, delay_iters: int = 0, ksplit: int = 0):
        self.kind = kind
        params = PolicyParams(stride, count, flags, spin_limit, delay_tile, delay_iters, ksplit)
        h = ctypes.c_void_p()
        _check(_lib().sync_policy_create(kind, ctypes.byref(params), ctypes.byref(h)), "sync_policy_create")
        self._h = h

    @property
    def handle(self):
        if self._h is None:
            raise RuntimeError("policy already destroyed")
        return self._h

    def destroy(self):
        if self._h is not None:
            _check(_lib().sync_policy_destroy(self._h), "sync_policy_destroy")
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def reset(self, stream=None):
        _check(_lib().dep_chain_reset(self.handle, _stream_handle(stream)), "dep_chain_reset")

    def read_trace(self, n_tiles: int):
        """Per-tile timing records of the last chain run with FLAG_TRACE (list of TraceRec)."""
        buf = (TraceRec * n_tiles)()
        n = _lib().depsync_read_trace(self.handle, buf, n_tiles)
        if n < 0:
            raise DepsyncError(n, "depsync_read_trace")
        return list(buf[:n])

    def status(self, raise_on_timeout: bool = True) -> Status:
        st = Status()
        rc = _lib().depsync_last_status(self.handle, ctypes.byref(st))
        if rc == ETIMEOUT and not raise_on_timeout:
            return st
        _check(rc, "depsync_last_status")
        return st


def sync_policy_create(kind: int, **params) -> SyncPolicy:
    return SyncPolicy(kind, **params)


def pack_weights_kblocked(Wt):
    """[N x K] (K contiguous) -> the K-blocked layout [K/64][N][64]: a pure re-arrangement."""
    n, k = Wt.shape
    if k % 64:
        raise ValueError("K must be a multiple of 64")
    return Wt.reshape(n, k // 64, 64).permute(1, 0, 2).contiguous()


def _dev_w(t, name: str):
    """A weight operand: 2-D [N x K] row-major, or 3-D [K/64][N][64] (K-blocked).  -> (ptr, ld, N, K, blocked)"""
    if t.dim() == 3:
        if not t.is_cuda or not t.is_contiguous() or t.shape[2] != 64:
            raise ValueError(f"{name}: K-blocked weights must be a contiguous [K/64, N, 64] device tensor")
        return t.data_ptr(), 0, t.shape[1], t.shape[0] * 64, True
    ptr, ld = _dev2d(t, name)
    return ptr, ld, t.shape[0], t.shape[1], False


def _gemm_desc(X, W1t, H, W2t, Y, mid, tile, T=None, batch=0, seq=0, heads=0, head_dim=0,
               k_cache=None, v_cache=None) -> GemmChainDesc:
    d = GemmChainDesc()
    d.X, d.ldx = _dev2d(X, "X")
    d.W1t, d.ldw1, w1n, w1k, b1 = _dev_w(W1t, "W1t")
    d.H, d.ldh = _dev2d(H, "H")
    d.W2t, d.ldw2, w2n, w2k, b2 = _dev_w(W2t, "W2t")
    if b1 != b2:
        raise ValueError("both weight operands must use the same layout")
    d.w_layout = W_KBLOCKED if b1 else W_ROWS
    d.Y, d.ldy = _dev2d(Y, "Y")
    d.M, d.K1 = X.shape
    d.N1 = H.shape[1]
    d.N2 = Y.shape[1]
    d.dtype = _dtype_code(X)
    for t in (W1t, H, W2t, Y):
        if t.dtype != X.dtype:
            raise TypeError("all tensors of a chain must share one element type")
    d.mid = mid
    if T is not None:
        d.T, d.ldt = _dev2d(T, "T")
    d.batch, d.seq, d.heads, d.head_dim = batch, seq, heads, head_dim
    if k_cache is not None or v_cache is not None:
        # [batch, cached, heads*head_dim] device tensors of earlier tokens' keys and values
        for t, name in ((k_cache, "k_cache"), (v_cache, "v_cache")):
            if t is None or not t.is_cuda or t.dim() != 3 or t.stride(2) != 1 or t.dtype != X.dtype:
                raise ValueError(f"{name} must be a 3-D device tensor of the chain's element type")
            if t.shape[0] != batch or t.stride(0) != t.shape[1] * t.stride(1):
                raise ValueError(f"{name}: one block of rows per sequence, equally spaced")
        if k_cache.shape != v_cache.shape or k_cache.stride() != v_cache.stride():
            raise ValueError("k_cache and v_cache must have the same shape and strides")
        d.k_cache, d.v_cache = k_cache.data_ptr(), v_cache.data_ptr()
        d.ld_cache, d.cached = k_cache.stride(1), k_cache.shape[1]
    d.tile_prod, d.tile_cons = _tile_pair(tile)
    rows1 = 2 * d.N1 if mid == MID_SWIGLU else d.N1
    k2 = heads * head_dim if mid == MID_CAUSAL_ATTN else d.N1
    if (w1n, w1k) != (rows1, d.K1) or (w2n, w2k) != (d.N2, k2) or H.shape[0] != d.M or Y.shape[0] != d.M:
        raise ValueError("operand shapes do not form a chain")
    return d


def dep_gemm_chain(X, W1t, H, W2t, Y, policy: SyncPolicy, mode: int = MODE_FINE, mid: int = MID_GELU,
                   tile: int = TILE_AUTO, stream_producer=None, stream_consumer=None, T=None,
                   batch: int = 0, seq: int = 0, heads: int = 0, head_dim: int = 0,
                   k_cache=None, v_cache=None) -> None:
    """Enqueue Y = mid(X W1) W2 with W1t = W1^T [N1 x K1] and W2t = W2^T [N2 x K2] (row-major)."""
    d = _gemm_desc(X, W1t, H, W2t, Y, mid, tile, T, batch, seq, heads, head_dim, k_cache, v_cache)
    _check(_lib().dep_gemm_chain(ctypes.byref(d), policy.handle, mode, _stream_handle(stream_producer),
                                 _stream_handle(stream_consumer)), "dep_gemm_chain")


def dep_gemm_chain_static(X, W1t, H, W2t, Y, kind: int, mid: int = MID_GELU, tile: int = TILE_AUTO, stream=None,
                          T=None, batch: int = 0, seq: int = 0, heads: int = 0, head_dim: int = 0,
                          k_cache=None, v_cache=None, **params) -> None:
    """The chain in one dispatch on `stream` with the library's fixed device workspace: no policy
    object, no allocation.  `params`: fields of PolicyParams (flags, ksplit, ...)."""
    d = _gemm_desc(X, W1t, H, W2t, Y, mid, tile, T, batch, seq, heads, head_dim, k_cache, v_cache)
    pp = PolicyParams(**params)
    _check(_lib().dep_gemm_chain_static(ctypes.byref(d), kind, ctypes.byref(pp), _stream_handle(stream)),
           "dep_gemm_chain_static")


def gemm_chain_plan(X, W1t, H, W2t, Y, policy: Optional[SyncPolicy], mid: int = MID_GELU, tile: int = TILE_AUTO,
                    n_cu: int = 0, **attn) -> PlanInfo:
    d = _gemm_desc(X, W1t, H, W2t, Y, mid, tile, **attn)
    info = PlanInfo()
    _check(_lib().depsync_gemm_chain_plan(ctypes.byref(d), policy.handle if policy else None, n_cu,
                                          ctypes.byref(info)), "depsync_gemm_chain_plan")
    return info


def gemm_chain_autotune(X, W1t, H, W2t, Y, policy: SyncPolicy, mid: int = MID_GELU, stream=None, reps: int = 3,
                        **attn) -> int:
    """Time every macro-tile shape on this chain and make the fastest the library's choice for it."""
    d = _gemm_desc(X, W1t, H, W2t, Y, mid, TILE_AUTO, **attn)
    tile = ctypes.c_int(0)
    _check(_lib().depsync_gemm_chain_autotune(ctypes.byref(d), policy.handle, _stream_handle(stream), reps,
                                              ctypes.byref(tile)), "depsync_gemm_chain_autotune")
    return tile.value


def conv_chain_autotune(x, w1, mid, w2, out, policy: SyncPolicy, stream=None, reps: int = 3) -> int:
    d = _conv_desc(x, w1, mid, w2, out, TILE_AUTO)
    tile = ctypes.c_int(0)
    _check(_lib().depsync_conv_chain_autotune(ctypes.byref(d), policy.handle, _stream_handle(stream), reps,
                                              ctypes.byref(tile)), "depsync_conv_chain_autotune")
    return tile.value


def gemm_chain_autotune_policy(X, W1t, H, W2t, Y, policy: SyncPolicy, mid: int = MID_GELU, stream=None, reps: int = 3, **attn):
    """Autotune the chain under every policy kind and remember the fastest for its shape (what AUTOSYNC
    policies resolve to).  Returns (kind, tile, [us under ROWSYNC, TILESYNC, STRIDEDSYNC; -1 = cannot run])."""
    d = _gemm_desc(X, W1t, H, W2t, Y, mid, TILE_AUTO, **attn)
    kind, tile, us = ctypes.c_int(-1), ctypes.c_int(0), (ctypes.c_float * 3)()
    _check(_lib().depsync_gemm_chain_autotune_policy(ctypes.byref(d), policy.handle, _stream_handle(stream), reps,
                                                     ctypes.byref(kind), ctypes.byref(tile), us), "depsync_gemm_chain_autotune_policy")
    return kind.value, tile.value, list(us)


def conv_chain_n_autotune_policy(x, ws, outs, policy: SyncPolicy, stream=None, reps: int = 3):
    d = _conv_n_desc(x, ws, outs, TILE_AUTO)
    kind, tile, us = ctypes.c_int(-1), ctypes.c_int(0), (ctypes.c_float * 3)()
    _check(_lib().depsync_conv_chain_n_autotune_policy(ctypes.byref(d), policy.handle, _stream_handle(stream), reps,
                                                       ctypes.byref(kind), ctypes.byref(tile), us), "depsync_conv_chain_n_autotune_policy")
    return kind.value, tile.value, list(us)


def gemm_chain_policy(X, W1t, H, W2t, Y, policy: SyncPolicy, mid: int = MID_GELU, **attn) -> int:
    """The policy kind a chain of this shape runs under with `policy` (what AUTOSYNC resolves to)."""
    d = _gemm_desc(X, W1t, H, W2t, Y, mid, TILE_AUTO, **attn)
    kind = ctypes.c_int(-1)
    _check(_lib().depsync_gemm_chain_policy(ctypes.byref(d), policy.handle, ctypes.byref(kind)), "depsync_gemm_chain_policy")
    return kind.value


TUNED_NO_SPLIT, TUNED_HW_ORDER = 1, 2


def gemm_chain_tuned(X, W1t, H, W2t, Y, policy: SyncPolicy, mid: int = MID_GELU, **attn):
    """(tile, flags) the library remembers for this chain; tile 0 when it remembers nothing."""
    d = _gemm_desc(X, W1t, H, W2t, Y, mid, TILE_AUTO, **attn)
    tile, flags = ctypes.c_int(0), ctypes.c_int(0)
    _check(_lib().depsync_gemm_chain_tuned(ctypes.byref(d), policy.handle, ctypes.byref(tile), ctypes.byref(flags)),
           "depsync_gemm_chain_tuned")
    return tile.value, flags.value


def gemm_chain_set_tuned(X, W1t, H, W2t, Y, policy: SyncPolicy, tile: int, flags: int = 0, mid: int = MID_GELU, **attn):
    d = _gemm_desc(X, W1t, H, W2t, Y, mid, TILE_AUTO, **attn)
    _check(_lib().depsync_gemm_chain_set_tuned(ctypes.byref(d), policy.handle, tile, flags), "depsync_gemm_chain_set_tuned")


def conv_chain_tuned(x, w1, mid, w2, out, policy: SyncPolicy):
    d = _conv_desc(x, w1, mid, w2, out, TILE_AUTO)
    tile, flags = ctypes.c_int(0), ctypes.c_int(0)
    _check(_lib().depsync_conv_chain_tuned(ctypes.byref(d), policy.handle, ctypes.byref(tile), ctypes.byref(flags)),
           "depsync_conv_chain_tuned")
    return tile.value, flags.value


def conv_chain_set_tuned(x, w1, mid, w2, out, policy: SyncPolicy, tile: int, flags: int = 0):
    d = _conv_desc(x, w1, mid, w2, out, TILE_AUTO)
    _check(_lib().depsync_conv_chain_set_tuned(ctypes.byref(d), policy.handle, tile, flags), "depsync_conv_chain_set_tuned")


def _conv_desc(x, w1, mid, w2, out, tile) -> ConvChainDesc:
    for t, name in ((x, "x"), (w1, "w1"), (mid, "mid"), (w2, "w2"), (out, "out")):
        if not t.is_cuda or not t.is_contiguous() or t.dim() != 4:
            raise ValueError(f"{name} must be a contiguous 4-D device tensor")
        if t.dtype != x.dtype:
            raise TypeError("all tensors of a chain must share one element type")
    d = ConvChainDesc()
    d.B, d.H, d.W, d.C = x.shape
    d.K1, d.K2 = w1.shape[0], w2.shape[0]
    if (tuple(w1.shape) != (d.K1, 3, 3, d.C) or tuple(w2.shape) != (d.K2, 3, 3, d.K1)
            or tuple(mid.shape) != (d.B, d.H, d.W, d.K1) or tuple(out.shape) != (d.B, d.H, d.W, d.K2)):
        raise ValueError("operand shapes do not form a conv chain")
    d.dtype = _dtype_code(x)
    d.inp, d.w1, d.mid, d.w2, d.out = x.data_ptr(), w1.data_ptr(), mid.data_ptr(), w2.data_ptr(), out.data_ptr()
    d.tile_prod, d.tile_cons = _tile_pair(tile)
    return d


def dep_conv_chain(x, w1, mid, w2, out, policy: SyncPolicy, mode: int = MODE_FINE, tile: int = TILE_AUTO,
                   stream_producer=None, stream_consumer=None) -> None:
    """Enqueue out = conv3x3(relu(conv3x3(x, w1)), w2); NHWC activations, [K,3,3,C] weights."""
    d = _conv_desc(x, w1, mid, w2, out, tile)
    _check(_lib().dep_conv_chain(ctypes.byref(d), policy.handle, mode, _stream_handle(stream_producer),
                                 _stream_handle(stream_consumer)), "dep_conv_chain")


def conv_chain_plan(x, w1, mid, w2, out, policy: Optional[SyncPolicy], tile: int = TILE_AUTO, n_cu: int = 0) -> PlanInfo:
    d = _conv_desc(x, w1, mid, w2, out, tile)
    info = PlanInfo()
    _check(_lib().depsync_conv_chain_plan(ctypes.byref(d), policy.handle if policy else None, n_cu,
                                          ctypes.byref(info)), "depsync_conv_chain_plan")
    return info


def _conv_n_desc(x, ws, outs, tile) -> ConvChainNDesc:
    n = len(ws)
    if n != len(outs) or not 2 <= n <= 4:
        raise ValueError("a conv chain has 2 to 4 convolutions, one output buffer each")
    for t in [x, *ws, *outs]:
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError("tensors must be contiguous device tensors")
    d = ConvChainNDesc()
    d.B, d.H, d.W, d.C = x.shape
    d.n = n
    d.dtype = _dtype_code(x)
    d.inp = x.data_ptr()
    cin = d.C
    for i, (w, o) in enumerate(zip(ws, outs)):
        if tuple(w.shape[1:]) != (3, 3, cin) or tuple(o.shape) != (d.B, d.H, d.W, w.shape[0]) or w.dtype != x.dtype or o.dtype != x.dtype:
            raise ValueError(f"conv {i}: weights [K,3,3,{cin}] and output [B,H,W,K] of the input's type expected")
        d.K[i], d.w[i], d.out[i] = w.shape[0], w.data_ptr(), o.data_ptr()
        cin = w.shape[0]
    d.tile_prod, d.tile_cons = _tile_pair(tile)
    return d


def dep_conv_chain_n(x, ws, outs, policy: SyncPolicy, mode: int = MODE_FINE, tile: int = TILE_AUTO,
                     stream_producer=None, stream_consumer=None) -> None:
    """Enqueue 2..4 chained 3x3 convolutions, ReLU between them: outs[i] = conv(relu-ed outs[i-1], ws[i])."""
    d = _conv_n_desc(x, ws, outs, tile)
    _check(_lib().dep_conv_chain_n(ctypes.byref(d), policy.handle, mode, _stream_handle(stream_producer),
                                   _stream_handle(stream_consumer)), "dep_conv_chain_n")


def conv_chain_n_plan(x, ws, outs, policy: Optional[SyncPolicy], tile: int = TILE_AUTO, n_cu: int = 0) -> PlanInfo:
    d = _conv_n_desc(x, ws, outs, tile)
    info = PlanInfo()
    _check(_lib().depsync_conv_chain_n_plan(ctypes.byref(d), policy.handle if policy else None, n_cu,
                                            ctypes.byref(info)), "depsync_conv_chain_n_plan")
    return info


def conv_chain_n_autotune(x, ws, outs, policy: SyncPolicy, stream=None, reps: int = 3) -> int:
    d = _conv_n_desc(x, ws, outs, TILE_AUTO)
    tile = ctypes.c_int(0)
    _check(_lib().depsync_conv_chain_n_autotune(ctypes.byref(d), policy.handle, _stream_handle(stream), reps,
                                                ctypes.byref(tile)), "depsync_conv_chain_n_autotune")
    return tile.value


def _copy_desc(src, mid, dst, tile_bytes: int) -> CopyChainDesc:
    n = src.numel() * src.element_size()
    for t, name in ((src, "src"), (mid, "mid"), (dst, "dst")):
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError(f"{name} must be a contiguous device tensor")
        if t.numel() * t.element_size() != n:
            raise ValueError("src, mid and dst must have the same size in bytes")
    d = CopyChainDesc()
    d.src, d.mid, d.dst = src.data_ptr(), mid.data_ptr(), dst.data_ptr()
    d.bytes, d.tile_bytes = n, tile_bytes
    return d


def dep_copy_chain(src, mid, dst, policy: SyncPolicy, mode: int = MODE_FINE, tile_bytes: int = 0,
                   stream_producer=None, stream_consumer=None) -> None:
    """Enqueue mid = src then dst = mid as two dependent tiled stages (the synchronisation-overhead chain)."""
    d = _copy_desc(src, mid, dst, tile_bytes)
    _check(_lib().dep_copy_chain(ctypes.byref(d), policy.handle, mode, _stream_handle(stream_producer),
                                 _stream_handle(stream_consumer)), "dep_copy_chain")


def copy_chain_plan(src, mid, dst, policy: SyncPolicy, tile_bytes: int = 0, n_cu: int = 0) -> PlanInfo:
    d = _copy_desc(src, mid, dst, tile_bytes)
    info = PlanInfo()
    _check(_lib().depsync_copy_chain_plan(ctypes.byref(d), policy.handle, n_cu, ctypes.byref(info)),
           "depsync_copy_chain_plan")
    return info


def gemm_chain_check_waits(desc: GemmChainDesc, kind: int, n_cu: int = 0, **params) -> int:
    """(row tile, K part) pairs of the planned chain with an operand slice no wait covers (0 = sound)."""
    pp = PolicyParams(**params)
    n = ctypes.c_int64(-1)
    _check(_lib().depsync_gemm_chain_check_waits(ctypes.byref(desc), kind, ctypes.byref(pp), n_cu, ctypes.byref(n)),
           "depsync_gemm_chain_check_waits")
    return n.value


def conv_chain_n_check_waits(desc: ConvChainNDesc, kind: int, n_cu: int = 0, **params) -> int:
    pp = PolicyParams(**params)
    n = ctypes.c_int64(-1)
    _check(_lib().depsync_conv_chain_n_check_waits(ctypes.byref(desc), kind, ctypes.byref(pp), n_cu, ctypes.byref(n)),
           "depsync_conv_chain_n_check_waits")
    return n.value


# ---- host mirrors -------------------------------------------------------------------------

def row_major(tile_x, tile_y, grid_x, grid_y) -> int:
    return _lib().depsync_row_major(tile_x, tile_y, grid_x, grid_y)


def policy_sem(kind, tile_x, tile_y, grid_x, grid_y, stride=0) -> int:
    return _lib().depsync_policy_sem(kind, tile_x, tile_y, grid_x, grid_y, stride)


def policy_value(kind, grid_x, grid_y, stride=0) -> int:
    return _lib().depsync_policy_value(kind, grid_x, grid_y, stride)


def wave_model(n_tiles, occupancy, n_cu):
    w, u = ctypes.c_int(), ctypes.c_double()
    _check(_lib().depsync_wave_model(n_tiles, occupancy, n_cu, ctypes.byref(w), ctypes.byref(u)), "depsync_wave_model")
    return w.value, u.value


def sync_count(kind, prod_grid, cons_grid, prod_rows_per_cons_row=1) -> int:
    return _lib().depsync_sync_count(kind, prod_grid[0], prod_grid[1], cons_grid[0], cons_grid[1],
                                     prod_rows_per_cons_row)


def mfma_calibration(zero_operands: bool = False, milliseconds: int = 200) -> float:
    """TFLOP/s a register-only bf16 MFMA loop sustains on this device (zero or random operands)."""
    out = ctypes.c_double(0.0)
    _check(_lib().depsync_mfma_calibration(int(zero_operands), milliseconds, ctypes.byref(out)), "depsync_mfma_calibration")
    return out.value


def simulate_chain(slots, prod_grid, d1, cons_grid, d2, halo=0, stream_sync=False) -> float:
    return _lib().depsync_simulate_chain(slots, prod_grid[0], prod_grid[1], d1, cons_grid[0], cons_grid[1], d2,
                                         halo, int(stream_sync))


def tile_shape(tile):
    r, c = ctypes.c_int(), ctypes.c_int()
    _check(_lib().depsync_tile_shape(tile, ctypes.byref(r), ctypes.byref(c)), "depsync_tile_shape")
    return r.value, c.value


def workspace_bytes() -> int:
    """Device memory a policy's workspace takes (split-K partial tiles not included)."""
    f = _lib().depsync_workspace_bytes
    f.restype = ctypes.c_size_t
    return int(f())


def device_info():
    n, k = ctypes.c_int(), ctypes.c_int()
    _check(_lib().depsync_device_info(ctypes.byref(n), ctypes.byref(k)), "depsync_device_info")
    return n.value, k.value
