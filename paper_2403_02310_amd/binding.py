"""ctypes binding of libsarathi (include/sarathi.h).  Argument marshalling only.

Device tensors are torch tensors used purely as device memory; their ``data_ptr()`` and the
current HIP stream handle are what crosses the boundary.  There is no fallback: if the
library has not been built, importing this module raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("SARATHI_LIB", os.path.join(_HERE, "libsarathi.so"))  # override: A/B builds of the same sources

OK, EINVAL, ESHAPE, ECAPACITY, EWORKSPACE, EHIP = 0, -1, -2, -3, -4, -5
STATUS_NAMES = {0: "SARATHI_OK", -1: "SARATHI_EINVAL", -2: "SARATHI_ESHAPE", -3: "SARATHI_ECAPACITY",
                -4: "SARATHI_EWORKSPACE", -5: "SARATHI_EHIP"}


class SarathiError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("%s: %s" % (STATUS_NAMES.get(status, status), message))
        self.status = status


class Config(ctypes.Structure):
    _fields_ = [("num_q_heads", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("page_size", ctypes.c_int32), ("dtype", ctypes.c_int32), ("max_tokens", ctypes.c_int32),
                ("max_seqs", ctypes.c_int32), ("max_blocks_per_seq", ctypes.c_int32)]


class WorkItem(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("seq", "col_begin", "n_cols", "key_begin", "key_end", "part_row", "kind", "reserved")]


class PlanInfo(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("num_items", "num_reduce_items", "num_part_rows", "split_keys",
                                              "num_tile_items", "tile_split_keys")]


class Request(ctypes.Structure):
    _fields_ = [("id", ctypes.c_int64), ("prompt_len", ctypes.c_int32), ("num_prefilled", ctypes.c_int32),
                ("num_decoded", ctypes.c_int32), ("reserved", ctypes.c_int32)]


class Batch(ctypes.Structure):
    _fields_ = [("num_seqs", ctypes.c_int32), ("num_tokens", ctypes.c_int32), ("num_decodes", ctypes.c_int32),
                ("num_prefill_chunks", ctypes.c_int32), ("num_admitted", ctypes.c_int32), ("reserved", ctypes.c_int32),
                ("free_pages_left", ctypes.c_int64),
                ("seq_id", ctypes.POINTER(ctypes.c_int64)), ("q_start", ctypes.POINTER(ctypes.c_int32)),
                ("q_len", ctypes.POINTER(ctypes.c_int32)), ("ctx_len", ctypes.POINTER(ctypes.c_int32))]


class KernelTimes(ctypes.Structure):
    _fields_ = [("append_ms", ctypes.c_double), ("attention_ms", ctypes.c_double), ("merge_ms", ctypes.c_double),
                ("append_launches", ctypes.c_int64), ("attention_launches", ctypes.c_int64),
                ("merge_launches", ctypes.c_int64)]


EXPORTED = ["sarathi_create", "sarathi_destroy", "sarathi_workspace_bytes", "sarathi_last_error",
            "sarathi_set_option", "sarathi_kv_append", "sarathi_hybrid_attention",
            "sarathi_plan_hybrid_attention", "sarathi_build_stall_free_batch", "sarathi_get_kernel_times",
            "sarathi_linear", "sarathi_linear_workspace_bytes", "sarathi_hybrid_attention_noalloc"]

if not os.path.exists(LIB_PATH):
    raise ImportError("libsarathi.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                      "(or python -m paper_2403_02310_amd.build) first; there is no fallback path")

lib = ctypes.CDLL(LIB_PATH)
_i32p = ctypes.POINTER(ctypes.c_int32)
_vp = ctypes.c_void_p
lib.sarathi_create.restype = ctypes.c_int
lib.sarathi_create.argtypes = [ctypes.POINTER(Config), ctypes.POINTER(_vp)]
lib.sarathi_destroy.restype = ctypes.c_int
lib.sarathi_destroy.argtypes = [_vp]
lib.sarathi_workspace_bytes.restype = ctypes.c_size_t
lib.sarathi_workspace_bytes.argtypes = [_vp]
lib.sarathi_last_error.restype = ctypes.c_char_p
lib.sarathi_last_error.argtypes = [_vp]
lib.sarathi_set_option.restype = ctypes.c_int
lib.sarathi_set_option.argtypes = [_vp, ctypes.c_char_p, ctypes.c_int64]
lib.sarathi_get_kernel_times.restype = ctypes.c_int
lib.sarathi_get_kernel_times.argtypes = [_vp, ctypes.POINTER(KernelTimes)]
lib.sarathi_kv_append.restype = ctypes.c_int
lib.sarathi_kv_append.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _i32p, _i32p, _i32p,
                                  ctypes.c_int32, ctypes.c_int32, ctypes.c_int64, _vp, _vp]
lib.sarathi_hybrid_attention.restype = ctypes.c_int
lib.sarathi_hybrid_attention.argtypes = [_vp, _vp, _vp, _vp, _vp, _i32p, _i32p, _i32p,
                                         ctypes.c_int32, ctypes.c_int32, ctypes.c_int64, ctypes.c_float, _vp, _vp, _vp]
lib.sarathi_hybrid_attention_noalloc.restype = ctypes.c_int
lib.sarathi_hybrid_attention_noalloc.argtypes = [_vp, _vp, _vp, _vp, _vp, _i32p, _i32p, _i32p,
                                                 ctypes.c_int32, ctypes.c_int32, ctypes.c_int64, ctypes.c_float, _vp, _vp]
lib.sarathi_plan_hybrid_attention.restype = ctypes.c_int
lib.sarathi_plan_hybrid_attention.argtypes = [_vp, _i32p, _i32p, _i32p, ctypes.c_int32, ctypes.c_int32,
                                              ctypes.POINTER(PlanInfo), ctypes.POINTER(WorkItem), ctypes.c_int32]
lib.sarathi_build_stall_free_batch.restype = ctypes.c_int
lib.sarathi_build_stall_free_batch.argtypes = [ctypes.c_int32, ctypes.c_int32,
                                               ctypes.POINTER(Request), ctypes.c_int32,
                                               ctypes.POINTER(Request), ctypes.c_int32,
                                               ctypes.POINTER(Request), ctypes.c_int32,
                                               ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.POINTER(Batch)]
lib.sarathi_linear_workspace_bytes.restype = ctypes.c_size_t
lib.sarathi_linear_workspace_bytes.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32]
lib.sarathi_linear.restype = ctypes.c_int
lib.sarathi_linear.argtypes = [_vp, _vp, _vp, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, _vp, ctypes.c_size_t, _vp]


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(_i32p)


def _dev(t) -> Optional[int]:
    """Device address of a torch tensor (must be contiguous); None passes a null pointer."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_contiguous():
        raise ValueError("device tensors must be contiguous")
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


class Handle:
    """One ``sarathi_handle``: attention shape, capacity bounds, and the caller-side workspace."""

    def __init__(self, num_q_heads: int, num_kv_heads: int, head_dim: int, max_tokens: int, max_seqs: int,
                 max_blocks_per_seq: int, page_size: int = 16, dtype: int = 0):
        self.config = Config(num_q_heads, num_kv_heads, head_dim, page_size, dtype, max_tokens, max_seqs,
                             max_blocks_per_seq)
        h = _vp()
        st = lib.sarathi_create(ctypes.byref(self.config), ctypes.byref(h))
        if st != OK:
            raise SarathiError(st, "sarathi_create rejected the configuration")
        self._h = h
        self.workspace = None

    def close(self):
        if getattr(self, "_h", None):
            lib.sarathi_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- plain accessors -------------------------------------------------
    def workspace_bytes(self) -> int:
        return int(lib.sarathi_workspace_bytes(self._h))

    def last_error(self) -> str:
        return lib.sarathi_last_error(self._h).decode()

    def set_option(self, name: str, value: int) -> None:
        self._check(lib.sarathi_set_option(self._h, name.encode(), int(value)))

    def kernel_times(self) -> KernelTimes:
        kt = KernelTimes()
        self._check(lib.sarathi_get_kernel_times(self._h, ctypes.byref(kt)))
        return kt

    def _check(self, st: int) -> None:
        if st != OK:
            raise SarathiError(st, self.last_error())

    def ensure_workspace(self, device="cuda"):
        """Allocates the device scratch once (torch is only the allocator here)."""
        if self.workspace is None:
            import torch
            self.workspace = torch.empty(self.workspace_bytes(), dtype=torch.uint8, device=device)
        return self.workspace

    # ---- entry points ----------------------------------------------------
    def plan(self, q_start, q_len, ctx_len, num_tokens: Optional[int] = None, with_items: bool = True):
        qs, ql, cl = _i32(q_start), _i32(q_len), _i32(ctx_len)
        n = int(ql.sum()) if num_tokens is None else num_tokens
        info = PlanInfo()
        self._check(lib.sarathi_plan_hybrid_attention(self._h, _ptr(qs), _ptr(ql), _ptr(cl), len(ql), n,
                                                      ctypes.byref(info), None, 0))
        items = None
        if with_items:
            items = (WorkItem * max(1, info.num_items))()
            self._check(lib.sarathi_plan_hybrid_attention(self._h, _ptr(qs), _ptr(ql), _ptr(cl), len(ql), n,
                                                          ctypes.byref(info), items, info.num_items))
            items = list(items)[: info.num_items]
        return info, items

    def _check_block_table(self, block_table, num_seqs: int) -> None:
        """The C ABI takes a bare pointer and walks it with the handle's row width; a tensor of another width
        would be read with the wrong stride, so the marshalling layer, which still sees the shape, refuses it."""
        shape = getattr(block_table, "shape", None)
        if shape is None:
            return
        if len(shape) != 2 or int(shape[1]) != int(self.config.max_blocks_per_seq) or int(shape[0]) < num_seqs:
            raise ValueError("block_table must be [>= %d, %d] (the handle's max_blocks_per_seq), got %s"
                             % (num_seqs, self.config.max_blocks_per_seq, tuple(shape)))
        if hasattr(block_table, "is_contiguous") and not block_table.is_contiguous():
            raise ValueError("block_table must be contiguous")

    def kv_append(self, k_new, v_new, k_cache, v_cache, block_table, q_start, q_len, ctx_len,
                  num_pages: Optional[int] = None, num_tokens: Optional[int] = None, workspace=None, stream=None):
        qs, ql, cl = _i32(q_start), _i32(q_len), _i32(ctx_len)
        n = int(ql.sum()) if num_tokens is None else num_tokens
        pages = int(k_cache.shape[0]) if num_pages is None else num_pages
        ws = workspace if workspace is not None else self.ensure_workspace()
        self._check_block_table(block_table, len(ql))
        self._check(lib.sarathi_kv_append(self._h, _dev(k_new), _dev(v_new), _dev(k_cache), _dev(v_cache),
                                          _dev(block_table), _ptr(qs), _ptr(ql), _ptr(cl), len(ql), n, pages,
                                          _dev(ws), _stream(stream)))

    def hybrid_attention(self, q, k_cache, v_cache, block_table, q_start, q_len, ctx_len, sm_scale: float, out,
                         num_pages: Optional[int] = None, num_tokens: Optional[int] = None, workspace=None,
                         stream=None):
        qs, ql, cl = _i32(q_start), _i32(q_len), _i32(ctx_len)
        n = int(ql.sum()) if num_tokens is None else num_tokens
        pages = int(k_cache.shape[0]) if num_pages is None else num_pages
        ws = workspace if workspace is not None else self.ensure_workspace()
        self._check_block_table(block_table, len(ql))
        self._check(lib.sarathi_hybrid_attention(self._h, _dev(q), _dev(k_cache), _dev(v_cache), _dev(block_table),
                                                 _ptr(qs), _ptr(ql), _ptr(cl), len(ql), n, pages, float(sm_scale),
                                                 _dev(out), _dev(ws), _stream(stream)))
        return out

    def hybrid_attention_noalloc(self, q, k_cache, v_cache, block_table, q_start, q_len, ctx_len, sm_scale: float, out,
                                 num_pages: Optional[int] = None, num_tokens: Optional[int] = None, stream=None):
        """``sarathi_hybrid_attention_noalloc``: no workspace, the library's built-in scratch."""
        qs, ql, cl = _i32(q_start), _i32(q_len), _i32(ctx_len)
        n = int(ql.sum()) if num_tokens is None else num_tokens
        pages = int(k_cache.shape[0]) if num_pages is None else num_pages
        self._check_block_table(block_table, len(ql))
        self._check(lib.sarathi_hybrid_attention_noalloc(self._h, _dev(q), _dev(k_cache), _dev(v_cache), _dev(block_table),
                                                         _ptr(qs), _ptr(ql), _ptr(cl), len(ql), n, pages, float(sm_scale),
                                                         _dev(out), _stream(stream)))
        return out


class PreparedBatch:
    """Host length arrays converted once, for callers that time repeated iterations."""

    def __init__(self, q_start, q_len, ctx_len):
        self.q_start, self.q_len, self.ctx_len = _i32(q_start), _i32(q_len), _i32(ctx_len)
        self.num_seqs = len(self.q_len)
        self.num_tokens = int(self.q_len.sum())
        self.p_q_start, self.p_q_len, self.p_ctx_len = _ptr(self.q_start), _ptr(self.q_len), _ptr(self.ctx_len)


def raw_kv_append(handle: Handle, pb: PreparedBatch, k_new_ptr, v_new_ptr, k_cache_ptr, v_cache_ptr, bt_ptr,
                  num_pages, ws_ptr, stream_ptr) -> int:
    return lib.sarathi_kv_append(handle._h, k_new_ptr, v_new_ptr, k_cache_ptr, v_cache_ptr, bt_ptr,
                                 pb.p_q_start, pb.p_q_len, pb.p_ctx_len, pb.num_seqs, pb.num_tokens, num_pages,
                                 ws_ptr, stream_ptr)


def raw_hybrid_attention(handle: Handle, pb: PreparedBatch, q_ptr, k_cache_ptr, v_cache_ptr, bt_ptr, num_pages,
                         sm_scale, out_ptr, ws_ptr, stream_ptr) -> int:
    return lib.sarathi_hybrid_attention(handle._h, q_ptr, k_cache_ptr, v_cache_ptr, bt_ptr,
                                        pb.p_q_start, pb.p_q_len, pb.p_ctx_len, pb.num_seqs, pb.num_tokens,
                                        num_pages, sm_scale, out_ptr, ws_ptr, stream_ptr)


def build_stall_free_batch(token_budget: int, chunk_size: int, running_decodes: Sequence, running_prefills: Sequence,
                           waiting_prefills: Sequence, free_pages: int, page_size: int = 16,
                           max_batch_size: int = 128):
    """One pass of stall-free batching; requests are (id, prompt_len, num_prefilled, num_decoded) tuples."""
    def arr(reqs):
        a = (Request * max(1, len(reqs)))()
        for i, r in enumerate(reqs):
            a[i] = Request(int(r[0]), int(r[1]), int(r[2]), int(r[3]), 0)
        return a
    cap = max(1, max_batch_size)
    seq_id = np.zeros(cap, np.int64); q_start = np.zeros(cap, np.int32)
    q_len = np.zeros(cap, np.int32); ctx_len = np.zeros(cap, np.int32)
    b = Batch()
    b.seq_id = seq_id.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))
    b.q_start, b.q_len, b.ctx_len = _ptr(q_start), _ptr(q_len), _ptr(ctx_len)
    st = lib.sarathi_build_stall_free_batch(token_budget, chunk_size, arr(running_decodes), len(running_decodes),
                                            arr(running_prefills), len(running_prefills),
                                            arr(waiting_prefills), len(waiting_prefills),
                                            free_pages, page_size, max_batch_size, ctypes.byref(b))
    if st != OK:
        raise SarathiError(st, "sarathi_build_stall_free_batch")
    n = b.num_seqs
    return {"seq_id": seq_id[:n].tolist(), "q_start": q_start[:n].tolist(), "q_len": q_len[:n].tolist(),
            "ctx_len": ctx_len[:n].tolist(), "num_tokens": b.num_tokens, "num_decodes": b.num_decodes,
            "num_prefill_chunks": b.num_prefill_chunks, "num_admitted": b.num_admitted,
            "free_pages_left": int(b.free_pages_left)}


def linear_workspace_bytes(num_tokens: int, out_features: int, in_features: int) -> int:
    return int(lib.sarathi_linear_workspace_bytes(num_tokens, out_features, in_features))


def linear(x, w, y, workspace=None, stream=None) -> None:
    """``y[t, n] = sum_k x[t, k] * w[n, k]`` on the GPU (``sarathi_linear``): x [T, K], w [N, K], y [T, N], bf16
    device tensors; ``workspace`` an optional device byte tensor for split-K partial tiles."""
    T, K = x.shape
    N = w.shape[0]
    if w.shape[1] != K or tuple(y.shape) != (T, N):
        raise ValueError("x [T, K], w [N, K], y [T, N] expected")
    for t in (x, w, y):
        if not t.is_contiguous():
            raise ValueError("tensors must be contiguous")
    ws_ptr, ws_bytes = (None, 0) if workspace is None else (_dev(workspace), workspace.numel() * workspace.element_size())
    st = lib.sarathi_linear(_dev(x), _dev(w), _dev(y), T, N, K, ws_ptr, ws_bytes, _stream(stream))
    if st != 0:
        raise SarathiError(st, "sarathi_linear(T=%d, N=%d, K=%d) failed" % (T, N, K))
