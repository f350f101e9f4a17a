"""Thin ctypes binding of libstreamindex: same names as include/streamindex.h, argument
marshalling only.  Tensors are torch tensors living on the GPU; every step of the path runs
in the library's HIP kernels.  There is no CPU fallback: a missing library is an error."""
from __future__ import annotations

import ctypes
import os
from ctypes import (POINTER, Structure, byref, c_char_p, c_double, c_float, c_int32, c_int64, c_size_t,
                    c_uint64, c_void_p)

import torch  # first: makes the process use torch's HIP runtime, which the library then shares

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libstreamindex.so")

SI_OK = 0
SI_ERR_INVALID_ARG = -1
SI_ERR_UNSUPPORTED_SHAPE = -2
SI_ERR_WORKSPACE_TOO_SMALL = -3
SI_ERR_HIP = -4
SI_MASK_NONE = 0
SI_MASK_CAUSAL_BLOCK = 1
SI_PROFILE_CLASSES = 7
PROFILE_CLASS_NAMES = ("score_tile", "filter_scores", "compact", "finalize", "init", "fused", "fused_narrow")

EXPORTS = (
    "si_plan_tiles", "si_workspace_bytes", "si_indexer_topk", "si_indexer_topk_tiled",
    "si_fused_workspace_bytes", "si_indexer_topk_fused", "si_indexer_topk_fused_shape",
    "si_fused_shape_for", "si_indexer_topk_static", "si_sparse_attention",
    "si_score_tile", "si_topk_from_scores", "si_materialize_bytes", "si_profile_enable",
    "si_profile_reset", "si_profile_read", "si_profile_phases", "si_wall_clock_khz", "si_strerror",
    "si_last_hip_error",
    "si_version",
)


class si_dims(Structure):
    _fields_ = [("B", c_int32), ("S", c_int32), ("H_I", c_int32), ("D", c_int32), ("T", c_int32)]


class si_plan(Structure):
    _fields_ = [("c_S", c_int32), ("c_T", c_int32), ("workspace_bytes", c_size_t)]


class StreamIndexError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {si_strerror(status)} (status {status}, hip error {si_last_hip_error()})")


_lib = None


def load():
    """Loads the in-tree shared library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2605_02568_amd.build` "
            "(there is no fallback path)")
    L = ctypes.CDLL(LIB_PATH)
    L.si_plan_tiles.restype = c_int32
    L.si_plan_tiles.argtypes = [POINTER(si_dims), c_int32, c_int32, c_int32, c_size_t, POINTER(si_plan)]
    L.si_workspace_bytes.restype = c_size_t
    L.si_workspace_bytes.argtypes = [POINTER(si_dims), c_int32, c_int32, c_int32]
    L.si_indexer_topk.restype = c_int32
    L.si_indexer_topk.argtypes = [c_void_p, c_void_p, c_void_p, POINTER(si_dims), c_int32, c_int32,
                                  c_int32, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]
    L.si_indexer_topk_tiled.restype = c_int32
    L.si_indexer_topk_tiled.argtypes = [c_void_p, c_void_p, c_void_p, POINTER(si_dims), c_int32,
                                        c_int32, c_int32, c_int32, c_int32, c_void_p, c_void_p,
                                        c_void_p, c_size_t, c_void_p]
    L.si_fused_workspace_bytes.restype = c_size_t
    L.si_fused_workspace_bytes.argtypes = [POINTER(si_dims), c_int32, c_int32]
    L.si_indexer_topk_fused.restype = c_int32
    L.si_indexer_topk_fused.argtypes = [c_void_p, c_void_p, c_void_p, POINTER(si_dims), c_int32,
                                        c_int32, c_int32, c_int32, c_void_p, c_void_p, c_void_p,
                                        c_size_t, c_void_p]
    L.si_indexer_topk_fused_shape.restype = c_int32
    L.si_indexer_topk_fused_shape.argtypes = [c_void_p, c_void_p, c_void_p, POINTER(si_dims), c_int32,
                                              c_int32, c_int32, c_int32, c_int32, c_void_p, c_void_p,
                                              c_void_p, c_size_t, c_void_p]
    L.si_fused_shape_for.restype = c_int32
    L.si_fused_shape_for.argtypes = [POINTER(si_dims), c_int32, c_int32, c_int32]
    L.si_indexer_topk_static.restype = c_int32
    L.si_indexer_topk_static.argtypes = [c_void_p, c_void_p, c_void_p, POINTER(si_dims), c_int32,
                                         c_int32, c_int32, c_void_p, c_void_p, c_void_p]
    L.si_sparse_attention.restype = c_int32
    L.si_sparse_attention.argtypes = [c_void_p, c_void_p, c_void_p, POINTER(si_dims), c_int32, c_int32,
                                      c_int32, c_int32, c_float, c_void_p, c_void_p]
    L.si_score_tile.restype = c_int32
    L.si_score_tile.argtypes = [c_void_p, c_void_p, c_void_p, POINTER(si_dims), c_int32, c_int32,
                                c_int32, c_int32, c_int32, c_int32, c_void_p, c_void_p]
    L.si_topk_from_scores.restype = c_int32
    L.si_topk_from_scores.argtypes = [c_void_p, c_int32, c_int32, c_void_p, c_int32, c_int32,
                                      c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]
    L.si_materialize_bytes.restype = c_uint64
    L.si_materialize_bytes.argtypes = [POINTER(si_dims)]
    L.si_profile_enable.restype = c_int32
    L.si_profile_enable.argtypes = [c_int32]
    L.si_profile_reset.restype = c_int32
    L.si_profile_reset.argtypes = []
    L.si_profile_read.restype = c_int32
    L.si_profile_read.argtypes = [POINTER(c_double), POINTER(c_int64)]
    L.si_profile_phases.restype = c_int32
    L.si_profile_phases.argtypes = [c_void_p, c_int32]
    L.si_wall_clock_khz.restype = c_int32
    L.si_wall_clock_khz.argtypes = []
    L.si_strerror.restype = c_char_p
    L.si_strerror.argtypes = [c_int32]
    L.si_last_hip_error.restype = c_int32
    L.si_last_hip_error.argtypes = []
    L.si_version.restype = c_int32
    L.si_version.argtypes = []
    _lib = L
    return L


def _check(status: int, where: str):
    if status != SI_OK:
        raise StreamIndexError(status, where)


def _dev_ptr(t: torch.Tensor, dtype, name: str) -> int:
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name} must be a GPU tensor")
    if t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t.data_ptr()


def _stream_handle(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream)


def _dims_of(q, K, w) -> si_dims:
    if q.dim() != 4 or K.dim() != 3 or w.dim() != 3:
        raise ValueError("q must be [B,S,H_I,D], K [B,T,D], w [B,S,H_I]")
    B, S, H, D = q.shape
    if K.shape[0] != B or K.shape[2] != D or tuple(w.shape) != (B, S, H):
        raise ValueError(f"shape mismatch: q {tuple(q.shape)}, K {tuple(K.shape)}, w {tuple(w.shape)}")
    return si_dims(B, S, H, D, K.shape[1])


def si_strerror(status: int) -> str:
    return load().si_strerror(status).decode()


def si_last_hip_error() -> int:
    return int(load().si_last_hip_error())


def si_version() -> int:
    return int(load().si_version())


def si_materialize_bytes(B: int, S: int, H_I: int, D: int, T: int) -> int:
    return int(load().si_materialize_bytes(byref(si_dims(B, S, H_I, D, T))))


def si_workspace_bytes(B, S, H_I, D, T, k, c_S, c_T) -> int:
    return int(load().si_workspace_bytes(byref(si_dims(B, S, H_I, D, T)), k, c_S, c_T))


def si_plan_tiles(B, S, H_I, D, T, m, k, mask_mode, hbm_budget_bytes):
    """Returns (c_S, c_T, workspace_bytes)."""
    plan = si_plan()
    _check(load().si_plan_tiles(byref(si_dims(B, S, H_I, D, T)), m, k, mask_mode,
                                int(hbm_budget_bytes), byref(plan)), "si_plan_tiles")
    return int(plan.c_S), int(plan.c_T), int(plan.workspace_bytes)


def si_indexer_topk(q, K, w, m, k, mask_mode, out_idx, out_score, workspace, stream=None):
    """workspace: uint8 GPU tensor; its size is the HBM budget the tiling is planned against."""
    dims = _dims_of(q, K, w)
    _expect_out(out_idx, out_score, (dims.B, dims.S, k))
    _check(load().si_indexer_topk(
        _dev_ptr(q, torch.bfloat16, "q"), _dev_ptr(K, torch.bfloat16, "K"),
        _dev_ptr(w, torch.float32, "w"), byref(dims), m, k, mask_mode,
        _dev_ptr(out_idx, torch.int32, "out_idx"), _dev_ptr(out_score, torch.float32, "out_score"),
        _dev_ptr(workspace, torch.uint8, "workspace"), workspace.numel(),
        _stream_handle(stream)), "si_indexer_topk")


def si_indexer_topk_tiled(q, K, w, m, k, mask_mode, c_S, c_T, out_idx, out_score, workspace,
                          stream=None):
    dims = _dims_of(q, K, w)
    _expect_out(out_idx, out_score, (dims.B, dims.S, k))
    _check(load().si_indexer_topk_tiled(
        _dev_ptr(q, torch.bfloat16, "q"), _dev_ptr(K, torch.bfloat16, "K"),
        _dev_ptr(w, torch.float32, "w"), byref(dims), m, k, mask_mode, c_S, c_T,
        _dev_ptr(out_idx, torch.int32, "out_idx"), _dev_ptr(out_score, torch.float32, "out_score"),
        _dev_ptr(workspace, torch.uint8, "workspace"), workspace.numel(),
        _stream_handle(stream)), "si_indexer_topk_tiled")


def si_fused_workspace_bytes(B, S, H_I, D, T, k, c_S=0) -> int:
    return int(load().si_fused_workspace_bytes(byref(si_dims(B, S, H_I, D, T)), k, c_S))


def si_indexer_topk_fused(q, K, w, m, k, mask_mode, c_S, out_idx, out_score, workspace, stream=None):
    dims = _dims_of(q, K, w)
    _expect_out(out_idx, out_score, (dims.B, dims.S, k))
    _check(load().si_indexer_topk_fused(
        _dev_ptr(q, torch.bfloat16, "q"), _dev_ptr(K, torch.bfloat16, "K"),
        _dev_ptr(w, torch.float32, "w"), byref(dims), m, k, mask_mode, c_S,
        _dev_ptr(out_idx, torch.int32, "out_idx"), _dev_ptr(out_score, torch.float32, "out_score"),
        _dev_ptr(workspace, torch.uint8, "workspace"), workspace.numel(),
        _stream_handle(stream)), "si_indexer_topk_fused")


def si_fused_shape_for(B, S, H_I, D, T, m, k, mask_mode) -> int:
    """Queries per workgroup (8 or 4) si_indexer_topk_fused picks for this problem; 0 = not applicable."""
    return int(load().si_fused_shape_for(byref(si_dims(B, S, H_I, D, T)), m, k, mask_mode))


def si_indexer_topk_fused_shape(q, K, w, m, k, mask_mode, c_S, queries_per_workgroup, out_idx, out_score,
                                workspace, stream=None):
    dims = _dims_of(q, K, w)
    _expect_out(out_idx, out_score, (dims.B, dims.S, k))
    _check(load().si_indexer_topk_fused_shape(
        _dev_ptr(q, torch.bfloat16, "q"), _dev_ptr(K, torch.bfloat16, "K"),
        _dev_ptr(w, torch.float32, "w"), byref(dims), m, k, mask_mode, c_S, queries_per_workgroup,
        _dev_ptr(out_idx, torch.int32, "out_idx"), _dev_ptr(out_score, torch.float32, "out_score"),
        _dev_ptr(workspace, torch.uint8, "workspace"), workspace.numel(),
        _stream_handle(stream)), "si_indexer_topk_fused_shape")


def si_indexer_topk_static(q, K, w, m, k, mask_mode, out_idx, out_score, stream=None):
    """No workspace argument: the library's static scratch array is used (k <= 1024)."""
    dims = _dims_of(q, K, w)
    _expect_out(out_idx, out_score, (dims.B, dims.S, k))
    _check(load().si_indexer_topk_static(
        _dev_ptr(q, torch.bfloat16, "q"), _dev_ptr(K, torch.bfloat16, "K"),
        _dev_ptr(w, torch.float32, "w"), byref(dims), m, k, mask_mode,
        _dev_ptr(out_idx, torch.int32, "out_idx"), _dev_ptr(out_score, torch.float32, "out_score"),
        _stream_handle(stream)), "si_indexer_topk_static")


def si_sparse_attention(qa, Kc, idx, m, mask_mode, n_win, scale, out, stream=None):
    """Attention over TopK(t) U Window(t): qa [B,S,H_A,D] bf16, Kc [B,T,D] bf16, idx [B,S,k] int32,
    out [B,S,H_A,D] f32."""
    if qa.dim() != 4 or Kc.dim() != 3 or idx.dim() != 3:
        raise ValueError("qa must be [B,S,H_A,D], Kc [B,T,D], idx [B,S,k]")
    B, S, H, D = qa.shape
    if Kc.shape[0] != B or Kc.shape[2] != D or tuple(idx.shape[:2]) != (B, S):
        raise ValueError(f"shape mismatch: qa {tuple(qa.shape)}, Kc {tuple(Kc.shape)}, idx {tuple(idx.shape)}")
    if tuple(out.shape) != (B, S, H, D):
        raise ValueError(f"out must be {(B, S, H, D)}")
    dims = si_dims(B, S, H, D, Kc.shape[1])
    _check(load().si_sparse_attention(
        _dev_ptr(qa, torch.bfloat16, "qa"), _dev_ptr(Kc, torch.bfloat16, "Kc"),
        _dev_ptr(idx, torch.int32, "idx"), byref(dims), m, idx.shape[2], mask_mode, n_win, float(scale),
        _dev_ptr(out, torch.float32, "out"), _stream_handle(stream)), "si_sparse_attention")


def si_score_tile(q, K, w, m, mask_mode, s0, t0, c_S, c_T, tile, stream=None):
    dims = _dims_of(q, K, w)
    if tuple(tile.shape) != (dims.B, c_S, c_T):
        raise ValueError(f"tile must be [B, c_S, c_T] = {(dims.B, c_S, c_T)}")
    _check(load().si_score_tile(
        _dev_ptr(q, torch.bfloat16, "q"), _dev_ptr(K, torch.bfloat16, "K"),
        _dev_ptr(w, torch.float32, "w"), byref(dims), m, mask_mode, s0, t0, c_S, c_T,
        _dev_ptr(tile, torch.float32, "tile"), _stream_handle(stream)), "si_score_tile")


def si_topk_from_scores(scores, legal, k, c_T, out_idx, out_score, workspace, stream=None):
    if scores.dim() != 2:
        raise ValueError("scores must be [R, n_cols]")
    R, n_cols = scores.shape
    _expect_out(out_idx, out_score, (R, k))
    legal_ptr = None
    if legal is not None:
        if tuple(legal.shape) != (R,):
            raise ValueError("legal must be [R]")
        legal_ptr = _dev_ptr(legal, torch.int32, "legal")
    _check(load().si_topk_from_scores(
        _dev_ptr(scores, torch.float32, "scores"), R, n_cols, legal_ptr, k, c_T,
        _dev_ptr(out_idx, torch.int32, "out_idx"), _dev_ptr(out_score, torch.float32, "out_score"),
        _dev_ptr(workspace, torch.uint8, "workspace"), workspace.numel(),
        _stream_handle(stream)), "si_topk_from_scores")


def _expect_out(out_idx, out_score, shape):
    if tuple(out_idx.shape) != tuple(shape) or tuple(out_score.shape) != tuple(shape):
        raise ValueError(f"out_idx/out_score must be {tuple(shape)}")


def si_profile_enable(on: bool):
    _check(load().si_profile_enable(1 if on else 0), "si_profile_enable")


def si_profile_reset():
    _check(load().si_profile_reset(), "si_profile_reset")


PHASE_WORDS = 32
PHASE_TRACE_EVENTS = 2048
PHASE_NAMES = ("setup", "sweep", "merge", "final", "final_wait", "resident",
               "items", "sweeps", "steps", "merges", "launches",
               "merge_sync", "merge_load", "merge_radix", "merge_keep",
               "final_load", "final_radix", "final_keep", "final_sort", "final_write",
               "hw_id", "xcc_id", "start_tick")
PHASE_TIME_WORDS = (0, 1, 2, 3, 4, 5, 11, 12, 13, 14, 15, 16, 17, 18, 19)


def si_profile_phases(device_words, n_workgroups: int = 0):
    """device_words: int64 GPU tensor of n_workgroups*16 zeros, or None to switch the clock off."""
    if device_words is None:
        _check(load().si_profile_phases(None, 0), "si_profile_phases")
        return
    if device_words.numel() < n_workgroups * PHASE_WORDS + 2 * PHASE_TRACE_EVENTS:
        raise ValueError("device_words must hold n_workgroups * 32 + 4096 words")
    _check(load().si_profile_phases(_dev_ptr(device_words, torch.int64, "device_words"), n_workgroups),
           "si_profile_phases")


def si_wall_clock_khz() -> int:
    return int(load().si_wall_clock_khz())


def si_profile_read():
    """Returns {class name: (milliseconds, launches)} since the last reset."""
    ms = (c_double * SI_PROFILE_CLASSES)()
    n = (c_int64 * SI_PROFILE_CLASSES)()
    _check(load().si_profile_read(ms, n), "si_profile_read")
    return {name: (float(ms[i]), int(n[i])) for i, name in enumerate(PROFILE_CLASS_NAMES)}
