"""Thin ctypes binding of libspecext (argument marshalling only).

Every function has the name and argument order of its C entry point in
include/specext.h.  Tensors are torch tensors living on the GPU; the binding
passes their data pointers and the current HIP stream and checks the returned
status.  No arithmetic of the method happens in Python.  If the shared library
is missing, loading raises: there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

# SPECEXT_LIBRARY may name another build of the same library (e.g. one compiled with other flags)
_LIB_PATH = os.environ.get("SPECEXT_LIBRARY") or os.path.join(os.path.dirname(os.path.abspath(__file__)),
                                                              "libspecext.so")

SPECEXT_F32 = 0
SPECEXT_BF16 = 1
SPECEXT_MAX_TREE = 128
SPECEXT_MAX_SPLITS = 256
SPECEXT_FLAG_VALU_PREFIX = 1
SPECEXT_FLAG_PREFIX_ONLY = 2
SPECEXT_FLAG_FUSED_MERGE = 4
SPECEXT_FLAG_SHORT_WAIT = 8
WORKSPACE_HEADER_BYTES = 82176

STATUS_NAMES = {0: "SPECEXT_OK", -1: "SPECEXT_ERR_INVALID_ARG", -2: "SPECEXT_ERR_UNSUPPORTED",
                -3: "SPECEXT_ERR_WORKSPACE_TOO_SMALL", -4: "SPECEXT_ERR_LAUNCH_FAILED"}

EXPORTED = ("specext_strerror", "specext_workspace_bytes", "specext_num_splits", "specext_verify_attn",
            "specext_chunk_scores", "specext_select_chunks", "specext_gather_draft_kv", "specext_accept_greedy",
            "specext_commit_tree_kv", "specext_chunk_scores_accepted", "specext_materialized_bytes",
            "specext_materialized_ld", "specext_attn_materialized", "specext_chunk_scores_materialized",
            "specext_prefill_attn", "specext_verify_attn_static", "specext_workspace_init",
            "specext_calib_stream_read", "specext_calib_mfma", "specext_calib_issue_mix", "specext_chunk_scores_select")


class SpecextError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {STATUS_NAMES.get(status, status)} ({strerror(status)})")


class specext_desc(ctypes.Structure):
    _fields_ = [
        ("struct_size", ctypes.c_uint32), ("dtype", ctypes.c_int32), ("out_dtype", ctypes.c_int32),
        ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
        ("prefix_len", ctypes.c_int32), ("n_tree", ctypes.c_int32), ("chunk_size", ctypes.c_int32),
        ("want_scores", ctypes.c_int32), ("num_splits", ctypes.c_int32), ("softmax_scale", ctypes.c_float),
        ("flags", ctypes.c_uint32), ("reserved", ctypes.c_uint32),
        ("q_stride_t", ctypes.c_int64), ("q_stride_h", ctypes.c_int64),
        ("kp_stride_h", ctypes.c_int64), ("kp_stride_l", ctypes.c_int64),
        ("kt_stride_h", ctypes.c_int64), ("kt_stride_t", ctypes.c_int64),
        ("o_stride_t", ctypes.c_int64), ("o_stride_h", ctypes.c_int64),
    ]


_lib = None


def load_library() -> ctypes.CDLL:
    """Load libspecext.so from the package directory; raises if it was not built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2505_20776_amd.build` "
                          "(there is no fallback implementation)")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    dp = ctypes.POINTER(specext_desc)
    lib.specext_strerror.restype = ctypes.c_char_p
    lib.specext_strerror.argtypes = [ctypes.c_int]
    lib.specext_workspace_bytes.restype = sz
    lib.specext_workspace_bytes.argtypes = [dp]
    lib.specext_num_splits.restype = ctypes.c_int
    lib.specext_num_splits.argtypes = [dp]
    lib.specext_verify_attn.restype = ctypes.c_int
    lib.specext_verify_attn.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.specext_workspace_init.restype = ctypes.c_int
    lib.specext_workspace_init.argtypes = [vp, sz, vp]
    lib.specext_verify_attn_static.restype = ctypes.c_int
    lib.specext_verify_attn_static.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.specext_chunk_scores.restype = ctypes.c_int
    lib.specext_chunk_scores.argtypes = [dp, vp, sz, i32, vp, vp]
    lib.specext_select_chunks.restype = ctypes.c_int
    lib.specext_select_chunks.argtypes = [vp, i32, i32, vp, vp, vp]
    lib.specext_gather_draft_kv.restype = ctypes.c_int
    lib.specext_gather_draft_kv.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, i32, i32, vp, vp, vp]
    i64 = ctypes.c_int64
    lib.specext_accept_greedy.restype = ctypes.c_int
    lib.specext_accept_greedy.argtypes = [vp, vp, vp, vp, i32, vp, vp, vp, vp]
    lib.specext_commit_tree_kv.restype = ctypes.c_int
    lib.specext_commit_tree_kv.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, i32,
                                           i64, i64, i64, i64, i64, i64, vp]
    lib.specext_chunk_scores_accepted.restype = ctypes.c_int
    lib.specext_chunk_scores_accepted.argtypes = [dp, vp, sz, vp, vp, vp, vp]
    lib.specext_materialized_bytes.restype = sz
    lib.specext_materialized_bytes.argtypes = [dp]
    lib.specext_materialized_ld.restype = ctypes.c_int
    lib.specext_materialized_ld.argtypes = [dp]
    lib.specext_attn_materialized.restype = ctypes.c_int
    lib.specext_attn_materialized.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.specext_chunk_scores_materialized.restype = ctypes.c_int
    lib.specext_chunk_scores_materialized.argtypes = [dp, vp, sz, i32, vp, vp, vp, vp]
    lib.specext_prefill_attn.restype = ctypes.c_int
    lib.specext_prefill_attn.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, ctypes.c_float,
                                         i64, i64, i64, i64, i64, i64, vp]
    lib.specext_chunk_scores_select.restype = ctypes.c_int
    lib.specext_chunk_scores_select.argtypes = [dp, vp, sz, i32, vp, vp, i32, vp, vp, vp, vp]
    lib.specext_calib_stream_read.restype = ctypes.c_int
    lib.specext_calib_stream_read.argtypes = [vp, sz, vp, vp]
    lib.specext_calib_mfma.restype = ctypes.c_int64
    lib.specext_calib_mfma.argtypes = [i32, i32, i32, vp, vp]
    lib.specext_calib_issue_mix.restype = ctypes.c_int
    lib.specext_calib_issue_mix.argtypes = [i32, i32, i32, i32, vp, vp]
    _lib = lib
    return lib


def make_desc(*, dtype: int, n_q_heads: int, n_kv_heads: int, head_dim: int, prefix_len: int, n_tree: int,
              out_dtype: Optional[int] = None, chunk_size: int = 0, want_scores: bool = False,
              num_splits: int = 0, softmax_scale: float = 0.0, flags: int = 0, **strides) -> specext_desc:
    d = specext_desc()
    d.struct_size = ctypes.sizeof(specext_desc)
    d.dtype = dtype
    d.out_dtype = dtype if out_dtype is None else out_dtype
    d.n_q_heads, d.n_kv_heads, d.head_dim = n_q_heads, n_kv_heads, head_dim
    d.prefix_len, d.n_tree = prefix_len, n_tree
    d.chunk_size, d.want_scores, d.num_splits = chunk_size, int(bool(want_scores)), num_splits
    d.softmax_scale = softmax_scale
    d.flags = flags
    for name, val in strides.items():
        if not hasattr(d, name):
            raise TypeError(f"unknown descriptor field {name}")
        setattr(d, name, val)
    return d


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def _check(status: int, where: str) -> None:
    if status != 0:
        raise SpecextError(status, where)


def strerror(status: int) -> str:
    return load_library().specext_strerror(int(status)).decode()


def workspace_bytes(desc: specext_desc) -> int:
    return int(load_library().specext_workspace_bytes(ctypes.byref(desc)))


def num_splits(desc: specext_desc) -> int:
    return int(load_library().specext_num_splits(ctypes.byref(desc)))


def workspace_init(workspace, workspace_nbytes: Optional[int] = None, stream=None, check: bool = True) -> int:
    if workspace_nbytes is None:
        workspace_nbytes = workspace.numel() * workspace.element_size()
    rc = load_library().specext_workspace_init(_ptr(workspace), workspace_nbytes, _stream(stream))
    if check:
        _check(rc, "specext_workspace_init")
    return rc


def verify_attn(desc, q, k_prefix, v_prefix, k_tree, v_tree, parent, out, lse, workspace,
                workspace_nbytes: Optional[int] = None, stream=None, check: bool = True) -> int:
    if workspace_nbytes is None:
        workspace_nbytes = workspace.numel() * workspace.element_size()
    rc = load_library().specext_verify_attn(ctypes.byref(desc), _ptr(q), _ptr(k_prefix), _ptr(v_prefix),
                                            _ptr(k_tree), _ptr(v_tree), _ptr(parent), _ptr(out), _ptr(lse),
                                            _ptr(workspace), workspace_nbytes, _stream(stream))
    if check:
        _check(rc, "specext_verify_attn")
    return rc


def verify_attn_static(desc, q, k_prefix, v_prefix, k_tree, v_tree, parent, out, lse, status_out=None,
                       stream=None, check: bool = True) -> int:
    rc = load_library().specext_verify_attn_static(ctypes.byref(desc), _ptr(q), _ptr(k_prefix), _ptr(v_prefix),
                                                   _ptr(k_tree), _ptr(v_tree), _ptr(parent), _ptr(out), _ptr(lse),
                                                   _ptr(status_out), _stream(stream))
    if check:
        _check(rc, "specext_verify_attn_static")
    return rc


def chunk_scores(desc, workspace, score_row: int, scores, workspace_nbytes: Optional[int] = None,
                 stream=None, check: bool = True) -> int:
    if workspace_nbytes is None:
        workspace_nbytes = workspace.numel() * workspace.element_size()
    rc = load_library().specext_chunk_scores(ctypes.byref(desc), _ptr(workspace), workspace_nbytes,
                                             int(score_row), _ptr(scores), _stream(stream))
    if check:
        _check(rc, "specext_chunk_scores")
    return rc


def select_chunks(scores, n_chunks: int, k: int, idx_out, n_out, stream=None, check: bool = True) -> int:
    rc = load_library().specext_select_chunks(_ptr(scores), int(n_chunks), int(k), _ptr(idx_out), _ptr(n_out),
                                              _stream(stream))
    if check:
        _check(rc, "specext_select_chunks")
    return rc


def gather_draft_kv(k_src, v_src, k_dst, v_dst, idx, n_idx, max_idx: int, n_layers: int, n_kv_heads: int,
                    src_len: int, dst_cap: int, head_dim: int, chunk_size: int, elem_bytes: int,
                    pos_out=None, len_out=None, stream=None, check: bool = True, src_cap: int = 0) -> int:
    rc = load_library().specext_gather_draft_kv(_ptr(k_src), _ptr(v_src), _ptr(k_dst), _ptr(v_dst), _ptr(idx),
                                                _ptr(n_idx), int(max_idx), int(n_layers), int(n_kv_heads),
                                                int(src_len), int(src_cap), int(dst_cap), int(head_dim),
                                                int(chunk_size), int(elem_bytes), _ptr(pos_out), _ptr(len_out), _stream(stream))
    if check:
        _check(rc, "specext_gather_draft_kv")
    return rc


def accept_greedy(parent, draft_token, target_token, first_target, n_tree: int, path_out, n_accept_out,
                  next_token_out, stream=None, check: bool = True) -> int:
    rc = load_library().specext_accept_greedy(_ptr(parent), _ptr(draft_token), _ptr(target_token), _ptr(first_target),
                                              int(n_tree), _ptr(path_out), _ptr(n_accept_out), _ptr(next_token_out),
                                              _stream(stream))
    if check:
        _check(rc, "specext_accept_greedy")
    return rc


def commit_tree_kv(k_tree, v_tree, k_cache, v_cache, path, n_accept, max_accept: int, n_tree: int, n_layers: int,
                   n_kv_heads: int, head_dim: int, elem_bytes: int, prefix_len: int, cache_capacity: int,
                   tree_stride_layer: int = 0, tree_stride_h: int = 0, tree_stride_t: int = 0,
                   cache_stride_layer: int = 0, cache_stride_h: int = 0, cache_stride_l: int = 0, stream=None,
                   check: bool = True) -> int:
    rc = load_library().specext_commit_tree_kv(_ptr(k_tree), _ptr(v_tree), _ptr(k_cache), _ptr(v_cache), _ptr(path),
                                               _ptr(n_accept), int(max_accept), int(n_tree), int(n_layers),
                                               int(n_kv_heads), int(head_dim), int(elem_bytes), int(prefix_len),
                                               int(cache_capacity), int(tree_stride_layer), int(tree_stride_h),
                                               int(tree_stride_t), int(cache_stride_layer), int(cache_stride_h),
                                               int(cache_stride_l), _stream(stream))
    if check:
        _check(rc, "specext_commit_tree_kv")
    return rc


def chunk_scores_accepted(desc, workspace, path, n_accept, scores, workspace_nbytes: Optional[int] = None,
                          stream=None, check: bool = True) -> int:
    if workspace_nbytes is None:
        workspace_nbytes = workspace.numel() * workspace.element_size()
    rc = load_library().specext_chunk_scores_accepted(ctypes.byref(desc), _ptr(workspace), workspace_nbytes,
                                                      _ptr(path), _ptr(n_accept), _ptr(scores), _stream(stream))
    if check:
        _check(rc, "specext_chunk_scores_accepted")
    return rc


def materialized_bytes(desc: specext_desc) -> int:
    return int(load_library().specext_materialized_bytes(ctypes.byref(desc)))


def materialized_ld(desc: specext_desc) -> int:
    return int(load_library().specext_materialized_ld(ctypes.byref(desc)))


def attn_materialized(desc, q, k_prefix, v_prefix, k_tree, v_tree, parent, out, lse, workspace,
                      workspace_nbytes: Optional[int] = None, stream=None, check: bool = True) -> int:
    if workspace_nbytes is None:
        workspace_nbytes = workspace.numel() * workspace.element_size()
    rc = load_library().specext_attn_materialized(ctypes.byref(desc), _ptr(q), _ptr(k_prefix), _ptr(v_prefix),
                                                  _ptr(k_tree), _ptr(v_tree), _ptr(parent), _ptr(out), _ptr(lse),
                                                  _ptr(workspace), workspace_nbytes, _stream(stream))
    if check:
        _check(rc, "specext_attn_materialized")
    return rc


def chunk_scores_materialized(desc, workspace, score_row: int, scores, path=None, n_accept=None,
                              workspace_nbytes: Optional[int] = None, stream=None, check: bool = True) -> int:
    if workspace_nbytes is None:
        workspace_nbytes = workspace.numel() * workspace.element_size()
    rc = load_library().specext_chunk_scores_materialized(ctypes.byref(desc), _ptr(workspace), workspace_nbytes,
                                                          int(score_row), _ptr(path), _ptr(n_accept), _ptr(scores),
                                                          _stream(stream))
    if check:
        _check(rc, "specext_chunk_scores_materialized")
    return rc


def prefill_attn(q, k, v, out, lse, n_q_heads: int, n_kv_heads: int, head_dim: int, q_len: int, kv_len: int,
                 dtype: int = SPECEXT_BF16, out_dtype: int = SPECEXT_BF16, softmax_scale: float = 0.0,
                 q_stride_t: int = 0, q_stride_h: int = 0, kv_stride_h: int = 0, kv_stride_l: int = 0,
                 o_stride_t: int = 0, o_stride_h: int = 0, stream=None, check: bool = True) -> int:
    rc = load_library().specext_prefill_attn(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), int(n_q_heads),
                                             int(n_kv_heads), int(head_dim), int(q_len), int(kv_len), int(dtype),
                                             int(out_dtype), float(softmax_scale), int(q_stride_t), int(q_stride_h),
                                             int(kv_stride_h), int(kv_stride_l), int(o_stride_t), int(o_stride_h),
                                             _stream(stream))
    if check:
        _check(rc, "specext_prefill_attn")
    return rc


def calib_stream_read(src, nbytes: int, sink=None, stream=None, check: bool = True) -> int:
    rc = load_library().specext_calib_stream_read(_ptr(src), int(nbytes), _ptr(sink), _stream(stream))
    if check:
        _check(rc, "specext_calib_stream_read")
    return rc


def calib_mfma(iters: int, tile: int = 32, workgroups: int = 512, sink=None, stream=None,
                    check: bool = True) -> int:
    """Returns the floating-point operations of the launch."""
    rc = int(load_library().specext_calib_mfma(int(iters), int(tile), int(workgroups), _ptr(sink),
                                                    _stream(stream)))
    if check and rc < 0:
        _check(rc, "specext_calib_mfma")
    return rc


def calib_issue_mix(mode: int, vector_per_matrix: int, iters: int, workgroups: int = 256, sink=None, stream=None,
                    check: bool = True) -> int:
    rc = int(load_library().specext_calib_issue_mix(int(mode), int(vector_per_matrix), int(iters), int(workgroups),
                                                    _ptr(sink), _stream(stream)))
    if check:
        _check(rc, "specext_calib_issue_mix")
    return rc


def chunk_scores_select(desc, workspace, score_row: int, k: int, idx_out, n_out, scores=None, path=None, n_accept=None,
                        workspace_nbytes: Optional[int] = None, stream=None, check: bool = True) -> int:
    if workspace_nbytes is None:
        workspace_nbytes = workspace.numel() * workspace.element_size()
    rc = load_library().specext_chunk_scores_select(ctypes.byref(desc), _ptr(workspace), workspace_nbytes,
                                                    int(score_row), _ptr(path), _ptr(n_accept), int(k), _ptr(scores),
                                                    _ptr(idx_out), _ptr(n_out), _stream(stream))
    if check:
        _check(rc, "specext_chunk_scores_select")
    return rc
