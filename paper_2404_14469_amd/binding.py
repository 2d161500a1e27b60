"""ctypes binding of libsnapkv.so: argument marshalling only, same names as include/snapkv.h.

Every step of the path runs in the HIP kernels behind the C ABI.  PyTorch appears here only as
the owner of device memory and of the stream the work is enqueued on.  There is no fallback:
if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libsnapkv.so")

POOL_MAX, POOL_AVG = 0, 1
DTYPE_BF16, DTYPE_F32, DTYPE_F16 = 0, 1, 2

SYMBOLS = ("snapkv_version", "snapkv_strerror", "snapkv_compress", "snapkv_compress_f32",
           "snapkv_pooled_scores", "snapkv_pooled_scores_f32", "snapkv_workspace_bytes",
           "snapkv_compress_ws", "snapkv_select_topk", "snapkv_release", "snapkv_profile_start",
           "snapkv_profile_stop", "snapkv_num_stages", "snapkv_stage_name", "snapkv_set_scoring_scheme",
           "snapkv_sync_timeouts", "snapkv_compress_lse", "snapkv_pooled_scores_lse",
           "snapkv_compress_strided", "snapkv_compress_f16", "snapkv_pooled_scores_f16",
           "snapkv_decode_attention", "snapkv_compress_per_query_head",
           "snapkv_capacity_for_rate", "snapkv_hit_rate", "snapkv_compress_paged",
           "snapkv_compress_varlen", "snapkv_compress_layers", "snapkv_compress_static",
           "snapkv_compress_ws_status", "snapkv_debug_set_wait_limit")

_lib = None


class SnapKVError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"snapkv error {code}: {text}")
        self.code = code


def load():
    """Load libsnapkv.so (built in-tree by paper_2404_14469_amd/build.py); raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2404_14469_amd.build` "
            "(there is no CPU fallback)")
    L = ctypes.CDLL(LIB_PATH)
    vp, i64, i32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_size_t
    L.snapkv_version.restype = i32
    L.snapkv_version.argtypes = []
    L.snapkv_strerror.restype = ctypes.c_char_p
    L.snapkv_strerror.argtypes = [i32]
    for name in ("snapkv_compress", "snapkv_compress_f32", "snapkv_compress_f16"):
        f = getattr(L, name)
        f.restype = i64
        f.argtypes = [vp, vp, vp, i64, i32, i32, i32, i32, i32, i32, i64, vp, vp, vp, vp]
    for name in ("snapkv_pooled_scores", "snapkv_pooled_scores_f32", "snapkv_pooled_scores_f16"):
        f = getattr(L, name)
        f.restype = i32
        f.argtypes = [vp, vp, i64, i32, i32, i32, i32, i32, i32, vp, vp]
    L.snapkv_compress_lse.restype = i64
    L.snapkv_compress_lse.argtypes = [i32, vp, vp, vp, vp, i64, i32, i32, i32, i32, i32, i32, i64, vp, vp, vp, vp]
    L.snapkv_pooled_scores_lse.restype = i32
    L.snapkv_pooled_scores_lse.argtypes = [i32, vp, vp, vp, i64, i32, i32, i32, i32, i32, i32, vp, vp]
    L.snapkv_compress_strided.restype = i64
    L.snapkv_compress_strided.argtypes = [i32, vp, vp, vp, i64, i32, i32, i32, i32, i64, i64, i64, i64, i32, i32,
                                          i64, vp, vp, vp, vp]
    L.snapkv_workspace_bytes.restype = sz
    L.snapkv_workspace_bytes.argtypes = [i64, i32, i32, i32, i32]
    L.snapkv_compress_ws.restype = i64
    L.snapkv_compress_ws.argtypes = [i32, vp, vp, vp, i64, i32, i32, i32, i32, i32, i32, i64, vp, vp,
                                     vp, vp, sz, vp]
    L.snapkv_compress_static.restype = i64
    L.snapkv_compress_static.argtypes = [i32, vp, vp, vp, i64, i32, i32, i32, i32, i32, i32, i64, vp, vp, vp, vp]
    L.snapkv_compress_ws_status.restype = i64
    L.snapkv_compress_ws_status.argtypes = [i32, vp, vp, vp, i64, i32, i32, i32, i32, i32, i32, i64, vp, vp,
                                            vp, vp, sz, vp, vp]
    L.snapkv_debug_set_wait_limit.restype = i32
    L.snapkv_debug_set_wait_limit.argtypes = [ctypes.c_longlong]
    L.snapkv_select_topk.restype = i32
    L.snapkv_select_topk.argtypes = [vp, i32, i64, i64, vp, vp]
    L.snapkv_compress_per_query_head.restype = i64
    L.snapkv_compress_per_query_head.argtypes = [i32, vp, vp, vp, i64, i32, i32, i32, i32, i32, i32, i64, vp, vp, vp, vp]
    L.snapkv_capacity_for_rate.restype = i64
    L.snapkv_capacity_for_rate.argtypes = [i64, i32, ctypes.c_double]
    L.snapkv_compress_paged.restype = i64
    L.snapkv_compress_paged.argtypes = [i32, vp, vp, vp, vp, i64, i32, i64, i32, i32, i32, i32, i32, i32, i64, vp, vp, vp, vp]
    L.snapkv_compress_layers.restype = i32
    L.snapkv_compress_layers.argtypes = [i32, i32, vp, vp, vp, i64, i32, i32, i32, i32, i32, i32, i64, vp, vp, vp, vp]
    L.snapkv_compress_varlen.restype = i32
    L.snapkv_compress_varlen.argtypes = [i32, i32, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, i64, vp, vp, vp, vp, vp]
    L.snapkv_hit_rate.restype = i32
    L.snapkv_hit_rate.argtypes = [i32, vp, vp, i64, i64, i32, i32, i32, vp, i32, i64, i64, ctypes.c_float, vp, vp]
    L.snapkv_decode_attention.restype = i32
    L.snapkv_decode_attention.argtypes = [i32, vp, vp, vp, vp, i32, i32, i32, i32, i64, i64, vp, vp, vp]
    L.snapkv_release.restype = None
    L.snapkv_release.argtypes = []
    L.snapkv_profile_start.restype = i32
    L.snapkv_profile_start.argtypes = [i32]
    L.snapkv_profile_stop.restype = i32
    L.snapkv_profile_stop.argtypes = [vp, vp]
    L.snapkv_set_scoring_scheme.restype = i32
    L.snapkv_set_scoring_scheme.argtypes = [i32]
    L.snapkv_sync_timeouts.restype = i64
    L.snapkv_sync_timeouts.argtypes = []
    L.snapkv_num_stages.restype = i32
    L.snapkv_num_stages.argtypes = []
    L.snapkv_stage_name.restype = ctypes.c_char_p
    L.snapkv_stage_name.argtypes = [i32]
    _lib = L
    return L


def _check(code: int) -> int:
    if code < 0:
        raise SnapKVError(int(code), load().snapkv_strerror(int(code)).decode())
    return int(code)


def _stream(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream) if hasattr(stream, "cuda_stream") else int(stream)


def _dev(t: torch.Tensor, name: str, dtype=None) -> int:
    if not t.is_cuda:
        raise ValueError(f"{name} must be a GPU tensor")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"{name} must be {dtype}, got {t.dtype}")
    return t.data_ptr()


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return DTYPE_BF16
    if t.dtype == torch.float32:
        return DTYPE_F32
    if t.dtype == torch.float16:
        return DTYPE_F16
    raise ValueError(f"q/k/v must be bfloat16, float16 or float32, got {t.dtype}")


def snapkv_version() -> int:
    return int(load().snapkv_version())


def snapkv_strerror(code: int) -> str:
    return load().snapkv_strerror(int(code)).decode()


def snapkv_workspace_bytes(L: int, Hq: int, Hkv: int, D: int, W: int) -> int:
    return int(load().snapkv_workspace_bytes(L, Hq, Hkv, D, W))


def snapkv_release() -> None:
    load().snapkv_release()


def snapkv_set_scoring_scheme(scheme: int) -> None:
    """Bit 0: always the two-pass scoring kernels; bit 1: always separate pooling and selection kernels;
    bit 2 (test hook): the single-read kernel plans with 16 resident workgroups."""
    _check(load().snapkv_set_scoring_scheme(int(scheme)))


def snapkv_sync_timeouts() -> int:
    return _check(load().snapkv_sync_timeouts())


def snapkv_profile_start(max_calls: int) -> None:
    _check(load().snapkv_profile_start(int(max_calls)))


def snapkv_profile_stop():
    """Returns ({stage name: mean ms}, calls averaged)."""
    lib = load()
    ns = int(lib.snapkv_num_stages())
    ms = (ctypes.c_double * ns)()
    calls = ctypes.c_int(0)
    _check(lib.snapkv_profile_stop(ctypes.cast(ms, ctypes.c_void_p), ctypes.cast(ctypes.byref(calls), ctypes.c_void_p)))
    return {lib.snapkv_stage_name(i).decode(): float(ms[i]) for i in range(ns)}, int(calls.value)


def _shapes(q_win, k):
    Hq, W, D = q_win.shape
    Hkv, L, D2 = k.shape
    if D != D2:
        raise ValueError("q_win and k disagree on head dim")
    return Hq, Hkv, L, D, W


def snapkv_compress(q_win: torch.Tensor, k: torch.Tensor, v: torch.Tensor, pool_kind: int, p: int,
                    C: int, out_k: torch.Tensor, out_v: torch.Tensor, out_idx: torch.Tensor,
                    stream=None, workspace: Optional[torch.Tensor] = None) -> int:
    """q_win [Hq,W,D], k/v [Hkv,L,D] -> out_k/out_v [Hkv,C,D], out_idx [Hkv,C] int32; returns rows kept.

    bf16 tensors go to snapkv_compress, fp32 tensors to snapkv_compress_f32; with `workspace`
    (a uint8 GPU tensor) the call goes to snapkv_compress_ws and never allocates.
    """
    lib = load()
    Hq, Hkv, L, D, W = _shapes(q_win, k)
    code = _dtype_code(k)
    if v.shape != k.shape:
        raise ValueError("k and v must have the same shape")
    if tuple(out_k.shape) != (Hkv, C, D) or tuple(out_v.shape) != (Hkv, C, D):
        raise ValueError("out_k/out_v must be [Hkv, C, D]")
    if tuple(out_idx.shape) != (Hkv, C):
        raise ValueError("out_idx must be [Hkv, C]")
    ptrs = (_dev(q_win, "q_win", k.dtype), _dev(k, "k"), _dev(v, "v", k.dtype))
    outs = (_dev(out_k, "out_k", k.dtype), _dev(out_v, "out_v", k.dtype),
            _dev(out_idx, "out_idx", torch.int32))
    if workspace is not None:
        wp = _dev(workspace, "workspace", torch.uint8)
        return _check(lib.snapkv_compress_ws(code, *ptrs, L, Hq, Hkv, D, W, pool_kind, p, C, *outs, wp,
                                             workspace.numel(), _stream(stream)))
    fn = {DTYPE_BF16: lib.snapkv_compress, DTYPE_F32: lib.snapkv_compress_f32, DTYPE_F16: lib.snapkv_compress_f16}[code]
    return _check(fn(*ptrs, L, Hq, Hkv, D, W, pool_kind, p, C, *outs, _stream(stream)))


STATIC_SCRATCH_BYTES = 32 << 20
ERR_TIMEOUT = -6


def snapkv_compress_ws_status(q_win: torch.Tensor, k: torch.Tensor, v: torch.Tensor, pool_kind: int, p: int, C: int,
                              out_k: torch.Tensor, out_v: torch.Tensor, out_idx: torch.Tensor, workspace: torch.Tensor,
                              status: torch.Tensor, stream=None) -> int:
    """snapkv_compress_ws plus `status` (an int32 GPU tensor of one element): rows kept, or ERR_TIMEOUT."""
    lib = load()
    Hq, Hkv, L, D, W = _shapes(q_win, k)
    if v.shape != k.shape:
        raise ValueError("k and v must have the same shape")
    if tuple(out_k.shape) != (Hkv, C, D) or tuple(out_v.shape) != (Hkv, C, D) or tuple(out_idx.shape) != (Hkv, C):
        raise ValueError("out_k/out_v must be [Hkv, C, D] and out_idx [Hkv, C]")
    return _check(lib.snapkv_compress_ws_status(
        _dtype_code(k), _dev(q_win, "q_win", k.dtype), _dev(k, "k"), _dev(v, "v", k.dtype), L, Hq, Hkv, D, W, pool_kind, p, C,
        _dev(out_k, "out_k", k.dtype), _dev(out_v, "out_v", k.dtype), _dev(out_idx, "out_idx", torch.int32),
        _dev(workspace, "workspace", torch.uint8), workspace.numel(), _dev(status, "status", torch.int32), _stream(stream)))


def snapkv_debug_set_wait_limit(polls: int) -> None:
    """Test hook: bound of every wait inside the kernels, in polls (negative = the kernels' own bounds)."""
    _check(load().snapkv_debug_set_wait_limit(int(polls)))



def snapkv_compress_static(q_win: torch.Tensor, k: torch.Tensor, v: torch.Tensor, pool_kind: int, p: int,
                           C: int, out_k: torch.Tensor, out_v: torch.Tensor, out_idx: torch.Tensor, stream=None) -> int:
    """snapkv_compress on the library's fixed scratch array: allocates nothing, takes no workspace."""
    lib = load()
    Hq, Hkv, L, D, W = _shapes(q_win, k)
    if v.shape != k.shape:
        raise ValueError("k and v must have the same shape")
    if tuple(out_k.shape) != (Hkv, C, D) or tuple(out_v.shape) != (Hkv, C, D) or tuple(out_idx.shape) != (Hkv, C):
        raise ValueError("out_k/out_v must be [Hkv, C, D] and out_idx [Hkv, C]")
    return _check(lib.snapkv_compress_static(
        _dtype_code(k), _dev(q_win, "q_win", k.dtype), _dev(k, "k"), _dev(v, "v", k.dtype), L, Hq, Hkv, D, W, pool_kind, p, C,
        _dev(out_k, "out_k", k.dtype), _dev(out_v, "out_v", k.dtype), _dev(out_idx, "out_idx", torch.int32), _stream(stream)))


def snapkv_compress_strided(q_win: torch.Tensor, k: torch.Tensor, v: torch.Tensor, pool_kind: int, p: int,
                            C: int, out_k: torch.Tensor, out_v: torch.Tensor, out_idx: torch.Tensor,
                            stream=None) -> int:
    """snapkv_compress for k/v given as [Hkv, L, D] *views* of any storage order with contiguous rows
    (e.g. kv_token_major.permute(1, 0, 2)); the strides of dims 0 and 1 are passed on as they are."""
    lib = load()
    Hq, Hkv, L, D, W = _shapes(q_win, k)
    code = _dtype_code(k)
    if v.shape != k.shape or v.dtype != k.dtype:
        raise ValueError("k and v must have the same shape and dtype")
    for t, name in ((k, "k"), (v, "v")):
        if not t.is_cuda:
            raise ValueError(f"{name} must be a GPU tensor")
        if t.stride(2) != 1:
            raise ValueError(f"the rows of {name} must be contiguous")
    if tuple(out_k.shape) != (Hkv, C, D) or tuple(out_v.shape) != (Hkv, C, D):
        raise ValueError("out_k/out_v must be [Hkv, C, D]")
    if tuple(out_idx.shape) != (Hkv, C):
        raise ValueError("out_idx must be [Hkv, C]")
    return _check(lib.snapkv_compress_strided(
        code, _dev(q_win, "q_win", k.dtype), k.data_ptr(), v.data_ptr(), L, Hq, Hkv, D, W,
        k.stride(0), k.stride(1), v.stride(0), v.stride(1), pool_kind, p, C,
        _dev(out_k, "out_k", k.dtype), _dev(out_v, "out_v", k.dtype), _dev(out_idx, "out_idx", torch.int32),
        _stream(stream)))


def _lse_ptr(lse: torch.Tensor, Hq: int, W: int) -> int:
    if tuple(lse.shape) != (Hq, W):
        raise ValueError("lse must be [Hq, W]")
    return _dev(lse, "lse", torch.float32)


def snapkv_compress_lse(q_win: torch.Tensor, k: torch.Tensor, v: torch.Tensor, lse: torch.Tensor,
                        pool_kind: int, p: int, C: int, out_k: torch.Tensor, out_v: torch.Tensor,
                        out_idx: torch.Tensor, stream=None) -> int:
    """snapkv_compress with the window rows' log-sum-exp handed in (lse [Hq, W] float32)."""
    lib = load()
    Hq, Hkv, L, D, W = _shapes(q_win, k)
    code = _dtype_code(k)
    if v.shape != k.shape:
        raise ValueError("k and v must have the same shape")
    if tuple(out_k.shape) != (Hkv, C, D) or tuple(out_v.shape) != (Hkv, C, D):
        raise ValueError("out_k/out_v must be [Hkv, C, D]")
    if tuple(out_idx.shape) != (Hkv, C):
        raise ValueError("out_idx must be [Hkv, C]")
    return _check(lib.snapkv_compress_lse(
        code, _dev(q_win, "q_win", k.dtype), _dev(k, "k"), _dev(v, "v", k.dtype), _lse_ptr(lse, Hq, W),
        L, Hq, Hkv, D, W, pool_kind, p, C, _dev(out_k, "out_k", k.dtype), _dev(out_v, "out_v", k.dtype),
        _dev(out_idx, "out_idx", torch.int32), _stream(stream)))


def snapkv_pooled_scores_lse(q_win: torch.Tensor, k: torch.Tensor, lse: torch.Tensor, pool_kind: int,
                             p: int, out_scores: torch.Tensor, stream=None) -> None:
    """snapkv_pooled_scores with the window rows' log-sum-exp handed in."""
    lib = load()
    Hq, Hkv, L, D, W = _shapes(q_win, k)
    code = _dtype_code(k)
    if tuple(out_scores.shape) != (Hkv, L - W):
        raise ValueError("out_scores must be [Hkv, L-W]")
    _check(lib.snapkv_pooled_scores_lse(code, _dev(q_win, "q_win", k.dtype), _dev(k, "k"), _lse_ptr(lse, Hq, W),
                                        L, Hq, Hkv, D, W, pool_kind, p,
                                        _dev(out_scores, "out_scores", torch.float32), _stream(stream)))


def snapkv_pooled_scores(q_win: torch.Tensor, k: torch.Tensor, pool_kind: int, p: int,
                         out_scores: torch.Tensor, stream=None) -> None:
    """out_scores [Hkv, L-W] float32."""
    lib = load()
    Hq, Hkv, L, D, W = _shapes(q_win, k)
    code = _dtype_code(k)
    if tuple(out_scores.shape) != (Hkv, L - W):
        raise ValueError("out_scores must be [Hkv, L-W]")
    fn = {DTYPE_BF16: lib.snapkv_pooled_scores, DTYPE_F32: lib.snapkv_pooled_scores_f32,
          DTYPE_F16: lib.snapkv_pooled_scores_f16}[code]
    _check(fn(_dev(q_win, "q_win", k.dtype), _dev(k, "k"), L, Hq, Hkv, D, W, pool_kind, p,
              _dev(out_scores, "out_scores", torch.float32), _stream(stream)))


def snapkv_select_topk(scores: torch.Tensor, kcount: int, out_idx: torch.Tensor, stream=None) -> None:
    """scores [H, n] float32 (>= +0) -> out_idx [H, kcount] int32, ascending positions."""
    lib = load()
    H, n = scores.shape
    if tuple(out_idx.shape) != (H, kcount):
        raise ValueError("out_idx must be [H, kcount]")
    _check(lib.snapkv_select_topk(_dev(scores, "scores", torch.float32), H, n, kcount,
                                  _dev(out_idx, "out_idx", torch.int32), _stream(stream)))


def snapkv_compress_per_query_head(q_win: torch.Tensor, k: torch.Tensor, v: torch.Tensor, pool_kind: int, p: int,
                                   C: int, out_k: torch.Tensor, out_v: torch.Tensor, out_idx: torch.Tensor,
                                   stream=None) -> int:
    """One cache per query head: q_win [Hq,W,D], k/v [Hkv,L,D] -> out_k/out_v [Hq,C,D], out_idx [Hq,C]."""
    lib = load()
    Hq, Hkv, L, D, W = _shapes(q_win, k)
    if tuple(out_k.shape) != (Hq, C, D) or tuple(out_v.shape) != (Hq, C, D) or tuple(out_idx.shape) != (Hq, C):
        raise ValueError("out_k/out_v must be [Hq, C, D] and out_idx [Hq, C]")
    code = _dtype_code(q_win)
    kept = lib.snapkv_compress_per_query_head(
        code, _dev(q_win, "q_win"), _dev(k, "k", q_win.dtype), _dev(v, "v", q_win.dtype), L, Hq, Hkv, D, W,
        int(pool_kind), int(p), int(C), _dev(out_k, "out_k", q_win.dtype), _dev(out_v, "out_v", q_win.dtype),
        _dev(out_idx, "out_idx", torch.int32), _stream(stream))
    return _check(kept)


def snapkv_compress_paged(q_win: torch.Tensor, k_pages: torch.Tensor, v_pages: torch.Tensor, block_table: torch.Tensor,
                          L: int, pool_kind: int, p: int, C: int, out_k: torch.Tensor, out_v: torch.Tensor,
                          out_idx: torch.Tensor, stream=None) -> int:
    """q_win [Hq,W,D]; k_pages/v_pages [num_pages, page_size, Hkv, D]; block_table [ceil(L/page_size)] int32
    -> out_k/out_v [Hkv,C,D], out_idx [Hkv,C] (logical positions); returns rows kept."""
    lib = load()
    Hq, W, D = q_win.shape
    num_pages, page_size, Hkv, D2 = k_pages.shape
    if D != D2 or tuple(v_pages.shape) != tuple(k_pages.shape):
        raise ValueError("q_win, k_pages and v_pages disagree on their shapes")
    if block_table.dim() != 1 or block_table.numel() < (L + page_size - 1) // page_size:
        raise ValueError("block_table must hold ceil(L / page_size) entries")
    if tuple(out_k.shape) != (Hkv, C, D) or tuple(out_v.shape) != (Hkv, C, D) or tuple(out_idx.shape) != (Hkv, C):
        raise ValueError("out_k/out_v must be [Hkv, C, D] and out_idx [Hkv, C]")
    return _check(lib.snapkv_compress_paged(
        _dtype_code(q_win), _dev(q_win, "q_win"), _dev(k_pages, "k_pages", q_win.dtype),
        _dev(v_pages, "v_pages", q_win.dtype), _dev(block_table, "block_table", torch.int32), num_pages, page_size,
        int(L), Hq, Hkv, D, W, int(pool_kind), int(p), int(C), _dev(out_k, "out_k", q_win.dtype),
        _dev(out_v, "out_v", q_win.dtype), _dev(out_idx, "out_idx", torch.int32), _stream(stream)))


def snapkv_compress_varlen(q_wins, ks, vs, pool_kind: int, p: int, C: int, out_ks, out_vs, out_idxs, stream=None):
    """A batch of prompts of one model: lists of tensors shaped as for snapkv_compress (k [Hkv, L_i, D], ...).
    Returns the rows kept per head of every prompt."""
    lib = load()
    n = len(q_wins)
    if not (len(ks) == len(vs) == len(out_ks) == len(out_vs) == len(out_idxs) == n):
        raise ValueError("all lists must have one entry per prompt")
    if n == 0:
        return []
    Hq, Hkv, _, D, W = _shapes(q_wins[0], ks[0])
    code = _dtype_code(q_wins[0])
    Ls = []
    for i in range(n):
        hq, hkv, L, d, w = _shapes(q_wins[i], ks[i])
        if (hq, hkv, d, w) != (Hq, Hkv, D, W) or _dtype_code(q_wins[i]) != code:
            raise ValueError("the prompts of a batch share heads, head dim, window and dtype")
        if tuple(vs[i].shape) != tuple(ks[i].shape):
            raise ValueError("k and v must have the same shape")
        if tuple(out_ks[i].shape) != (Hkv, C, D) or tuple(out_vs[i].shape) != (Hkv, C, D) or \
                tuple(out_idxs[i].shape) != (Hkv, C):
            raise ValueError("out_k/out_v must be [Hkv, C, D] and out_idx [Hkv, C]")
        Ls.append(L)
    dt = q_wins[0].dtype
    arr = lambda ts, name, dtype: (ctypes.c_void_p * n)(*[_dev(t, name, dtype) for t in ts])
    kept = (ctypes.c_int64 * n)()
    _check(lib.snapkv_compress_varlen(
        code, n, arr(q_wins, "q_win", dt), arr(ks, "k", dt), arr(vs, "v", dt), (ctypes.c_int64 * n)(*Ls), Hq, Hkv, D, W,
        int(pool_kind), int(p), int(C), arr(out_ks, "out_k", dt), arr(out_vs, "out_v", dt),
        arr(out_idxs, "out_idx", torch.int32), kept, _stream(stream)))
    return [int(x) for x in kept]


def snapkv_compress_layers(q_wins, ks, vs, pool_kind: int, p: int, C: int, out_ks, out_vs, out_idxs, stream=None) -> None:
    """Several layers of one prompt: lists of tensors shaped as for snapkv_compress, all of one shape.  Slices of
    stacked [layers, heads, ...] tensors (for all six lists) take the fast form of the step."""
    lib = load()
    n = len(q_wins)
    if not (len(ks) == len(vs) == len(out_ks) == len(out_vs) == len(out_idxs) == n):
        raise ValueError("all lists must have one entry per layer")
    if n == 0:
        return
    Hq, Hkv, L, D, W = _shapes(q_wins[0], ks[0])
    code = _dtype_code(q_wins[0])
    for i in range(n):
        if _shapes(q_wins[i], ks[i]) != (Hq, Hkv, L, D, W) or _dtype_code(q_wins[i]) != code:
            raise ValueError("the layers of a call share heads, length, head dim, window and dtype")
        if tuple(vs[i].shape) != tuple(ks[i].shape):
            raise ValueError("k and v must have the same shape")
        if tuple(out_ks[i].shape) != (Hkv, C, D) or tuple(out_vs[i].shape) != (Hkv, C, D) or \
                tuple(out_idxs[i].shape) != (Hkv, C):
            raise ValueError("out_k/out_v must be [Hkv, C, D] and out_idx [Hkv, C]")
    dt = q_wins[0].dtype
    arr = lambda ts, name, dtype: (ctypes.c_void_p * n)(*[_dev(t, name, dtype) for t in ts])
    _check(lib.snapkv_compress_layers(
        code, n, arr(q_wins, "q_win", dt), arr(ks, "k", dt), arr(vs, "v", dt), L, Hq, Hkv, D, W, int(pool_kind), int(p),
        int(C), arr(out_ks, "out_k", dt), arr(out_vs, "out_v", dt), arr(out_idxs, "out_idx", torch.int32), _stream(stream)))


def snapkv_capacity_for_rate(L: int, W: int, rate: float) -> int:
    """C = W + floor(rate * (L - W)): the capacity that keeps the given share of the prefix."""
    return _check(load().snapkv_capacity_for_rate(int(L), int(W), float(rate)))


def snapkv_hit_rate(q_cur: torch.Tensor, k: torch.Tensor, n: int, idx: torch.Tensor, kcount: int, theta: float,
                    out_counts: torch.Tensor, stream=None) -> None:
    """q_cur [Hq,D], k [Hkv,Lk,D] (bf16 or fp16), idx [Hidx, stride] int32 whose first kcount entries per row
    are the selected prefix positions (ascending) -> out_counts [Hq,2] int32: (important, hits) per query head."""
    lib = load()
    Hq, D = q_cur.shape
    Hkv, Lk, D2 = k.shape
    if D != D2:
        raise ValueError("q_cur and k disagree on head dim")
    if idx.dim() != 2 or tuple(out_counts.shape) != (Hq, 2):
        raise ValueError("idx must be [Hidx, stride] and out_counts [Hq, 2]")
    _check(lib.snapkv_hit_rate(_dtype_code(q_cur), _dev(q_cur, "q_cur"), _dev(k, "k", q_cur.dtype), Lk, int(n), Hq, Hkv, D,
                               _dev(idx, "idx", torch.int32), idx.shape[0], int(kcount), idx.shape[1], float(theta),
                               _dev(out_counts, "out_counts", torch.int32), _stream(stream)))


def snapkv_decode_attention(q: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor, S: int,
                            out: torch.Tensor, out_lse: Optional[torch.Tensor] = None,
                            lens: Optional[torch.Tensor] = None, stream=None) -> None:
    """q [B,Hq,D], k_cache/v_cache [B,Hkv,cap,D] (bf16 or fp16) -> out [B,Hq,D] float32 and, if given,
    out_lse [B,Hq] float32; S valid rows per sequence, or lens [B] int32 on the GPU."""
    lib = load()
    B, Hq, D = q.shape
    Bk, Hkv, cap, Dk = k_cache.shape
    if (Bk, Dk) != (B, D) or tuple(v_cache.shape) != tuple(k_cache.shape):
        raise ValueError("q, k_cache and v_cache disagree on their shapes")
    if tuple(out.shape) != (B, Hq, D) or (out_lse is not None and tuple(out_lse.shape) != (B, Hq)):
        raise ValueError("out must be [B, Hq, D] and out_lse [B, Hq]")
    if lens is not None and tuple(lens.shape) != (B,):
        raise ValueError("lens must be [B]")
    code = _dtype_code(q)
    _check(lib.snapkv_decode_attention(
        code, _dev(q, "q"), _dev(k_cache, "k_cache", q.dtype), _dev(v_cache, "v_cache", q.dtype),
        _dev(lens, "lens", torch.int32) if lens is not None else None, B, Hq, Hkv, D, int(S), cap,
        _dev(out, "out", torch.float32), _dev(out_lse, "out_lse", torch.float32) if out_lse is not None else None,
        _stream(stream)))


def compress(q_win, k, v, pool_kind: int, p: int, C: int, stream=None
             ) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor, int]:
    """Convenience wrapper: allocates the outputs with torch and returns (out_k, out_v, out_idx, kept)."""
    Hkv, L, D = k.shape
    out_k = torch.empty((Hkv, C, D), dtype=k.dtype, device=k.device)
    out_v = torch.empty((Hkv, C, D), dtype=k.dtype, device=k.device)
    out_idx = torch.empty((Hkv, C), dtype=torch.int32, device=k.device)
    kept = snapkv_compress(q_win, k, v, pool_kind, p, C, out_k, out_v, out_idx, stream=stream)
    return out_k, out_v, out_idx, kept
