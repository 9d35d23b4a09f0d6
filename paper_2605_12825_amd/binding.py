"""Thin ctypes binding of liborthrus.so: same names as the C ABI, argument marshalling only.

Every step of the path runs in the library's HIP kernels; nothing here computes.  Device
buffers are torch tensors (torch is used for device memory and streams only); the functions
pass their data pointers straight through.  There is no CPU fallback: if the library cannot be
loaded the import of this module fails.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

from . import build as _build

ORTHRUS_OK = 0
ORTHRUS_EINVAL = -1
ORTHRUS_EUNSUPPORTED = -2
ORTHRUS_EWORKSPACE = -3
ORTHRUS_ECAPACITY = -4
ORTHRUS_EHIP = -5

ORTHRUS_VIEW_DIFFUSION = 0
ORTHRUS_VIEW_AR_VERIFY = 1

EXPORTED = [
    "orthrus_create", "orthrus_destroy", "orthrus_status_string", "orthrus_attn_workspace_bytes",
    "orthrus_consensus_workspace_bytes", "orthrus_sampling_workspace_bytes", "orthrus_attn_num_splits",
    "orthrus_dual_view_attn", "orthrus_consensus_commit", "orthrus_sampling_consensus_commit",
    "orthrus_prefill_workspace_bytes", "orthrus_prefill_attn",
    "orthrus_graph_begin", "orthrus_graph_end", "orthrus_graph_launch", "orthrus_graph_destroy",
    "orthrus_attn_timing", "orthrus_attn_timing_read", "orthrus_attn_timing_samples", "orthrus_last_device_error",
    "orthrus_attn_num_splits_on", "orthrus_attn_workspace_bytes_on", "orthrus_build_id", "orthrus_kv_stream_probe",
    "orthrus_noalloc_scratch_bytes", "orthrus_consensus_commit_noalloc",
]


class orthrus_params(ctypes.Structure):
    """Mirror of the C struct orthrus_params."""
    _fields_ = [
        ("batch", ctypes.c_int32), ("num_q_heads", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("block_k", ctypes.c_int32), ("page_size", ctypes.c_int32),
        ("max_pages_per_seq", ctypes.c_int32), ("max_seq_len", ctypes.c_int32),
        ("num_splits", ctypes.c_int32), ("num_layers", ctypes.c_int32), ("vocab", ctypes.c_int32),
        ("sm_scale", ctypes.c_float), ("num_pages", ctypes.c_int64),
        ("pool_stride_layer", ctypes.c_int64), ("pool_stride_page", ctypes.c_int64),
        ("pool_stride_head", ctypes.c_int64), ("pool_stride_tok", ctypes.c_int64),
        ("q_stride_row", ctypes.c_int64), ("q_stride_head", ctypes.c_int64), ("blk_stride_row", ctypes.c_int64),
        ("blk_stride_head", ctypes.c_int64), ("blk_stride_layer", ctypes.c_int64),
    ]


class OrthrusError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: %s (%d)" % (where, orthrus_status_string(status), status))


def _library_file() -> str:
    """The built library; ORTHRUS_LIBRARY selects another build of the same sources (the host-UBSan one)."""
    return os.environ.get("ORTHRUS_LIBRARY") or _build.LIB


def _load() -> ctypes.CDLL:
    if not os.path.exists(_library_file()):
        if os.environ.get("ORTHRUS_LIBRARY"):
            raise ImportError("ORTHRUS_LIBRARY=%s does not exist" % _library_file())
        _build.build_library()   # nothing built yet: build once
    # PyTorch ships its own HIP runtime; load it first so that this library binds to that one.  Two
    # HIP runtimes in one process do not share the GPU: whichever initialises second sees no device.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = ctypes.CDLL(_library_file())
    # A library older than the sources next to it would silently test yesterday's kernels: its build id is
    # the digest of the sources and flags it was compiled from, so a mismatch means "rebuild".
    lib.orthrus_build_id.restype = ctypes.c_char_p
    lib.orthrus_build_id.argtypes = []
    built, now = lib.orthrus_build_id().decode(), _build.source_digest()
    if built != now:
        raise ImportError("%s was built from other sources (build id %s, sources %s): rebuild it with "
                          "`python -m paper_2605_12825_amd.build`" % (_library_file(), built, now))
    vp, i32p = ctypes.c_void_p, ctypes.c_void_p
    pp = ctypes.POINTER(orthrus_params)
    lib.orthrus_create.restype = ctypes.c_int
    lib.orthrus_create.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_int]
    lib.orthrus_destroy.restype = ctypes.c_int
    lib.orthrus_destroy.argtypes = [vp]
    lib.orthrus_status_string.restype = ctypes.c_char_p
    lib.orthrus_status_string.argtypes = [ctypes.c_int]
    lib.orthrus_attn_workspace_bytes.restype = ctypes.c_int64
    lib.orthrus_attn_workspace_bytes.argtypes = [pp]
    lib.orthrus_consensus_workspace_bytes.restype = ctypes.c_int64
    lib.orthrus_consensus_workspace_bytes.argtypes = [pp]
    lib.orthrus_attn_num_splits.restype = ctypes.c_int32
    lib.orthrus_attn_num_splits.argtypes = [pp]
    lib.orthrus_dual_view_attn.restype = ctypes.c_int
    lib.orthrus_dual_view_attn.argtypes = [vp, pp, ctypes.c_int, vp, vp, vp, vp, vp, i32p, i32p, vp, vp, vp,
                                           ctypes.c_size_t, vp]
    lib.orthrus_consensus_commit.restype = ctypes.c_int
    lib.orthrus_consensus_commit.argtypes = [vp, pp, vp, i32p, vp, vp, vp, vp, i32p, i32p, i32p, i32p, i32p, i32p,
                                             vp, ctypes.c_size_t, vp]
    lib.orthrus_sampling_workspace_bytes.restype = ctypes.c_int64
    lib.orthrus_sampling_workspace_bytes.argtypes = [pp]
    lib.orthrus_sampling_consensus_commit.restype = ctypes.c_int
    lib.orthrus_sampling_consensus_commit.argtypes = [vp, pp, ctypes.c_float, vp, vp, i32p, vp, vp, vp, vp, vp, vp,
                                                      i32p, i32p, i32p, i32p, i32p, i32p, vp, ctypes.c_size_t, vp]
    lib.orthrus_prefill_workspace_bytes.restype = ctypes.c_int64
    lib.orthrus_prefill_workspace_bytes.argtypes = [pp, ctypes.c_int32]
    lib.orthrus_prefill_attn.restype = ctypes.c_int
    lib.orthrus_prefill_attn.argtypes = [vp, pp, ctypes.c_int32, vp, vp, vp, i32p, vp, vp, i32p, i32p, vp, vp,
                                         ctypes.c_size_t, vp]
    lib.orthrus_graph_begin.restype = ctypes.c_int
    lib.orthrus_graph_begin.argtypes = [vp, vp]
    lib.orthrus_graph_end.restype = ctypes.c_int
    lib.orthrus_graph_end.argtypes = [vp, vp, ctypes.POINTER(ctypes.c_void_p)]
    lib.orthrus_graph_launch.restype = ctypes.c_int
    lib.orthrus_graph_launch.argtypes = [vp, vp]
    lib.orthrus_graph_destroy.restype = ctypes.c_int
    lib.orthrus_graph_destroy.argtypes = [vp]
    lib.orthrus_attn_timing.restype = ctypes.c_int
    lib.orthrus_attn_timing.argtypes = [vp, ctypes.c_int]
    lib.orthrus_attn_timing_read.restype = ctypes.c_int
    lib.orthrus_attn_timing_read.argtypes = [vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64),
                                             ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64)]
    lib.orthrus_last_device_error.restype = ctypes.c_int
    lib.orthrus_last_device_error.argtypes = [vp, vp, ctypes.POINTER(ctypes.c_int32)]
    lib.orthrus_attn_timing_samples.restype = ctypes.c_int
    lib.orthrus_attn_timing_samples.argtypes = [vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double),
                                                ctypes.c_int64, ctypes.POINTER(ctypes.c_int64)]
    lib.orthrus_attn_num_splits_on.restype = ctypes.c_int32
    lib.orthrus_attn_num_splits_on.argtypes = [vp, pp]
    lib.orthrus_attn_workspace_bytes_on.restype = ctypes.c_int64
    lib.orthrus_attn_workspace_bytes_on.argtypes = [vp, pp]
    lib.orthrus_noalloc_scratch_bytes.restype = ctypes.c_int64
    lib.orthrus_noalloc_scratch_bytes.argtypes = []
    lib.orthrus_consensus_commit_noalloc.restype = ctypes.c_int
    lib.orthrus_consensus_commit_noalloc.argtypes = [vp, pp, vp, i32p, vp, vp, vp, vp, i32p, i32p, i32p, i32p, i32p,
                                                     i32p, vp]
    lib.orthrus_kv_stream_probe.restype = ctypes.c_int
    lib.orthrus_kv_stream_probe.argtypes = [vp, pp, vp, vp, i32p, i32p, vp]
    return lib


_lib = _load()


def library_path() -> str:
    return _library_file()


def _ptr(t) -> Optional[int]:
    """Device (or host) address of a torch tensor, an int address, or None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return int(t.data_ptr())


def _nbytes(t) -> int:
    return 0 if t is None else int(t.numel() * t.element_size())


def _stream_handle(stream) -> Optional[int]:
    if stream is None:
        import torch
        return int(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return stream
    return int(stream.cuda_stream)


def orthrus_status_string(status: int) -> str:
    return _lib.orthrus_status_string(int(status)).decode()


def orthrus_create(device: int = 0) -> int:
    h = ctypes.c_void_p()
    st = _lib.orthrus_create(ctypes.byref(h), int(device))
    if st != ORTHRUS_OK:
        raise OrthrusError(st, "orthrus_create")
    return h.value


def orthrus_destroy(ctx: int) -> None:
    st = _lib.orthrus_destroy(ctx)
    if st != ORTHRUS_OK:
        raise OrthrusError(st, "orthrus_destroy")


def orthrus_attn_workspace_bytes(p: orthrus_params) -> int:
    n = _lib.orthrus_attn_workspace_bytes(ctypes.byref(p))
    if n < 0:
        raise OrthrusError(int(n), "orthrus_attn_workspace_bytes")
    return int(n)


def orthrus_consensus_workspace_bytes(p: orthrus_params) -> int:
    n = _lib.orthrus_consensus_workspace_bytes(ctypes.byref(p))
    if n < 0:
        raise OrthrusError(int(n), "orthrus_consensus_workspace_bytes")
    return int(n)


def orthrus_attn_num_splits(p: orthrus_params) -> int:
    n = _lib.orthrus_attn_num_splits(ctypes.byref(p))
    if n < 0:
        raise OrthrusError(int(n), "orthrus_attn_num_splits")
    return int(n)


def orthrus_attn_num_splits_on(ctx, p: orthrus_params) -> int:
    n = _lib.orthrus_attn_num_splits_on(ctx, ctypes.byref(p))
    if n < 0:
        raise OrthrusError(int(n), "orthrus_attn_num_splits_on")
    return int(n)


def orthrus_attn_workspace_bytes_on(ctx, p: orthrus_params) -> int:
    n = _lib.orthrus_attn_workspace_bytes_on(ctx, ctypes.byref(p))
    if n < 0:
        raise OrthrusError(int(n), "orthrus_attn_workspace_bytes_on")
    return int(n)


def orthrus_build_id() -> str:
    return _lib.orthrus_build_id().decode()


def orthrus_kv_stream_probe(ctx, p: orthrus_params, k_pool, v_pool, page_table, seq_lens, stream=None) -> None:
    st = _lib.orthrus_kv_stream_probe(ctx, ctypes.byref(p), _ptr(k_pool), _ptr(v_pool), _ptr(page_table),
                                      _ptr(seq_lens), _stream_handle(stream))
    if st != ORTHRUS_OK:
        raise OrthrusError(st, "orthrus_kv_stream_probe")


def orthrus_dual_view_attn(ctx, p: orthrus_params, view: int, q, k_blk, v_blk, k_pool, v_pool, page_table,
                           seq_lens, out, lse=None, workspace=None, stream=None, check: bool = True) -> int:
    st = _lib.orthrus_dual_view_attn(ctx, ctypes.byref(p), int(view), _ptr(q), _ptr(k_blk), _ptr(v_blk),
                                     _ptr(k_pool), _ptr(v_pool), _ptr(page_table), _ptr(seq_lens), _ptr(out),
                                     _ptr(lse), _ptr(workspace), _nbytes(workspace), _stream_handle(stream))
    if check and st != ORTHRUS_OK:
        raise OrthrusError(st, "orthrus_dual_view_attn")
    return st


def orthrus_consensus_commit(ctx, p: orthrus_params, ar_logits, draft_tokens, k_blk_ar, v_blk_ar, k_pool, v_pool,
                             page_table, seq_lens, accept_len, num_committed, out_tokens, next_anchor,
                             workspace=None, stream=None, check: bool = True) -> int:
    st = _lib.orthrus_consensus_commit(ctx, ctypes.byref(p), _ptr(ar_logits), _ptr(draft_tokens), _ptr(k_blk_ar),
                                       _ptr(v_blk_ar), _ptr(k_pool), _ptr(v_pool), _ptr(page_table),
                                       _ptr(seq_lens), _ptr(accept_len), _ptr(num_committed), _ptr(out_tokens),
                                       _ptr(next_anchor), _ptr(workspace), _nbytes(workspace),
                                       _stream_handle(stream))
    if check and st != ORTHRUS_OK:
        raise OrthrusError(st, "orthrus_consensus_commit")
    return st


def orthrus_noalloc_scratch_bytes() -> int:
    return int(_lib.orthrus_noalloc_scratch_bytes())


def orthrus_consensus_commit_noalloc(ctx, p: orthrus_params, ar_logits, draft_tokens, k_blk_ar, v_blk_ar, k_pool,
                                     v_pool, page_table, seq_lens, accept_len, num_committed, out_tokens,
                                     next_anchor, stream=None, check: bool = True) -> int:
    st = _lib.orthrus_consensus_commit_noalloc(ctx, ctypes.byref(p), _ptr(ar_logits), _ptr(draft_tokens),
                                               _ptr(k_blk_ar), _ptr(v_blk_ar), _ptr(k_pool), _ptr(v_pool),
                                               _ptr(page_table), _ptr(seq_lens), _ptr(accept_len),
                                               _ptr(num_committed), _ptr(out_tokens), _ptr(next_anchor),
                                               _stream_handle(stream))
    if check and st != ORTHRUS_OK:
        raise OrthrusError(st, "orthrus_consensus_commit_noalloc")
    return st


def orthrus_sampling_workspace_bytes(p: orthrus_params) -> int:
    n = _lib.orthrus_sampling_workspace_bytes(ctypes.byref(p))
    if n < 0:
        raise OrthrusError(int(n), "orthrus_sampling_workspace_bytes")
    return int(n)


def orthrus_sampling_consensus_commit(ctx, p: orthrus_params, temperature: float, ar_logits, diff_logits,
                                      draft_tokens, accept_u, gumbel, k_blk_ar, v_blk_ar, k_pool, v_pool,
                                      page_table, seq_lens, accept_len, num_committed, out_tokens, next_anchor,
                                      workspace=None, stream=None, check: bool = True) -> int:
    st = _lib.orthrus_sampling_consensus_commit(
        ctx, ctypes.byref(p), float(temperature), _ptr(ar_logits), _ptr(diff_logits), _ptr(draft_tokens),
        _ptr(accept_u), _ptr(gumbel), _ptr(k_blk_ar), _ptr(v_blk_ar), _ptr(k_pool), _ptr(v_pool), _ptr(page_table),
        _ptr(seq_lens), _ptr(accept_len), _ptr(num_committed), _ptr(out_tokens), _ptr(next_anchor),
        _ptr(workspace), _nbytes(workspace), _stream_handle(stream))
    if check and st != ORTHRUS_OK:
        raise OrthrusError(st, "orthrus_sampling_consensus_commit")
    return st


def orthrus_prefill_workspace_bytes(p: orthrus_params, max_new_tokens: int) -> int:
    n = _lib.orthrus_prefill_workspace_bytes(ctypes.byref(p), int(max_new_tokens))
    if n < 0:
        raise OrthrusError(int(n), "orthrus_prefill_workspace_bytes")
    return int(n)


def orthrus_prefill_attn(ctx, p: orthrus_params, max_new_tokens: int, q, k_new, v_new, new_lens, k_pool, v_pool,
                         page_table, seq_lens, out, workspace, stream=None) -> None:
    st = _lib.orthrus_prefill_attn(ctx, ctypes.byref(p), int(max_new_tokens), _ptr(q), _ptr(k_new), _ptr(v_new),
                                   _ptr(new_lens), _ptr(k_pool), _ptr(v_pool), _ptr(page_table), _ptr(seq_lens),
                                   _ptr(out), _ptr(workspace), _nbytes(workspace), _stream_handle(stream))
    if st != ORTHRUS_OK:
        raise OrthrusError(st, "orthrus_prefill_attn")


def orthrus_graph_begin(ctx, stream) -> None:
    st = _lib.orthrus_graph_begin(ctx, _stream_handle(stream))
    if st != ORTHRUS_OK:
        raise OrthrusError(st, "orthrus_graph_begin")


def orthrus_graph_end(ctx, stream) -> int:
    g = ctypes.c_void_p()
    st = _lib.orthrus_graph_end(ctx, _stream_handle(stream), ctypes.byref(g))
    if st != ORTHRUS_OK:
        raise OrthrusError(st, "orthrus_graph_end")
    return g.value


def orthrus_graph_launch(graph, stream=None) -> None:
    st = _lib.orthrus_graph_launch(graph, _stream_handle(stream))
    if st != ORTHRUS_OK:
        raise OrthrusError(st, "orthrus_graph_launch")


def orthrus_graph_destroy(graph) -> None:
    st = _lib.orthrus_graph_destroy(graph)
    if st != ORTHRUS_OK:
        raise OrthrusError(st, "orthrus_graph_destroy")


def orthrus_attn_timing(ctx, enable: bool) -> None:
    st = _lib.orthrus_attn_timing(ctx, 1 if enable else 0)
    if st != ORTHRUS_OK:
        raise OrthrusError(st, "orthrus_attn_timing")


def orthrus_attn_timing_read(ctx):
    """(split kernel microseconds, launches, combine kernel microseconds, launches) since the last read."""
    su, cu = ctypes.c_double(0.0), ctypes.c_double(0.0)
    sn, cn = ctypes.c_int64(0), ctypes.c_int64(0)
    st = _lib.orthrus_attn_timing_read(ctx, ctypes.byref(su), ctypes.byref(sn), ctypes.byref(cu), ctypes.byref(cn))
    if st != ORTHRUS_OK:
        raise OrthrusError(st, "orthrus_attn_timing_read")
    return su.value, sn.value, cu.value, cn.value


def orthrus_attn_timing_samples(ctx, capacity: int = 4096):
    """Per-call (split kernel us, combine kernel us) of the timed calls since the last read, in launch order."""
    su = (ctypes.c_double * capacity)()
    cu = (ctypes.c_double * capacity)()
    n = ctypes.c_int64(0)
    st = _lib.orthrus_attn_timing_samples(ctx, su, cu, capacity, ctypes.byref(n))
    if st != ORTHRUS_OK:
        raise OrthrusError(st, "orthrus_attn_timing_samples")
    k = min(int(n.value), capacity)
    return [(su[i], cu[i]) for i in range(k)]


def orthrus_last_device_error(ctx, stream=None) -> int:
    code = ctypes.c_int32(0)
    st = _lib.orthrus_last_device_error(ctx, _stream_handle(stream), ctypes.byref(code))
    if st != ORTHRUS_OK:
        raise OrthrusError(st, "orthrus_last_device_error")
    return int(code.value)


def make_params(*, batch, num_q_heads, num_kv_heads, head_dim, block_k, page_size, max_pages_per_seq, max_seq_len,
                num_pages, num_splits=0, num_layers=1, vocab=0, sm_scale=None, pool_stride_layer=None,
                pool_stride_page=None, pool_stride_head=None, pool_stride_tok=None, q_stride_row=0, q_stride_head=0,
                blk_stride_row=0, blk_stride_head=0, blk_stride_layer=0) -> orthrus_params:
    """Fills orthrus_params; pool strides default to the [pages, H_kv, P, d] layout, block inputs to dense."""
    p = orthrus_params()
    p.batch, p.num_q_heads, p.num_kv_heads, p.head_dim = batch, num_q_heads, num_kv_heads, head_dim
    p.block_k, p.page_size, p.max_pages_per_seq, p.max_seq_len = block_k, page_size, max_pages_per_seq, max_seq_len
    p.num_splits, p.num_layers, p.vocab = num_splits, num_layers, vocab
    p.sm_scale = float(sm_scale) if sm_scale is not None else (1.0 / float(head_dim) ** 0.5 if head_dim > 0 else 0.0)
    p.num_pages = num_pages
    p.pool_stride_tok = head_dim if pool_stride_tok is None else pool_stride_tok
    p.pool_stride_head = page_size * head_dim if pool_stride_head is None else pool_stride_head
    p.pool_stride_page = num_kv_heads * page_size * head_dim if pool_stride_page is None else pool_stride_page
    p.pool_stride_layer = num_pages * p.pool_stride_page if pool_stride_layer is None else pool_stride_layer
    p.q_stride_row, p.q_stride_head = q_stride_row, q_stride_head
    p.blk_stride_row, p.blk_stride_head, p.blk_stride_layer = blk_stride_row, blk_stride_head, blk_stride_layer
    return p
