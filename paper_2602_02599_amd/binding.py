"""ctypes binding of librap.so (argument marshalling only; see include/rap.h for the contract)."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))


def library_path() -> str:
    return os.path.join(_HERE, "librap.so")


class RapError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__("librap: %s (status %d)" % (text, status))
        self.status = status


class RapShape(C.Structure):
    """Mirror of rap_shape_t."""
    _fields_ = [
        ("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("d_head", C.c_int32),
        ("n_pairs", C.c_int32), ("d_v", C.c_int32), ("cache_cap", C.c_int64), ("rope_theta", C.c_double),
        ("pair_inv_freq", C.c_void_p),
    ]


class RapPaging(C.Structure):
    """Mirror of rap_paging_t."""
    _fields_ = [
        ("page_rows", C.c_int32), ("n_pages", C.c_int32), ("max_pages", C.c_int32), ("reserved", C.c_int32),
        ("block_table", C.c_void_p),
    ]


class RapKvCache(C.Structure):
    """Mirror of rap_kv_cache_t."""
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p), ("k_scale", C.c_void_p), ("v_scale", C.c_void_p),
                ("paging", C.POINTER(RapPaging))]


class RapTuning(C.Structure):
    """Mirror of rap_tuning_t."""
    _fields_ = [
        ("kernel", C.c_int32), ("rows_per_split", C.c_int32), ("reserved0", C.c_int32), ("reserved1", C.c_int32),
        ("ev_main_start", C.c_void_p), ("ev_main_stop", C.c_void_p),
    ]


KERNEL_AUTO, KERNEL_VALU, KERNEL_MFMA = 0, 1, 2

STATUS = {0: "RAP_OK", 1: "RAP_ERR_NULL", 2: "RAP_ERR_SHAPE", 3: "RAP_ERR_UNSUPPORTED", 4: "RAP_ERR_CAPACITY",
          5: "RAP_ERR_WORKSPACE", 6: "RAP_ERR_HIP", 7: "RAP_ERR_STATIC_LIMIT"}


def _ptr(t: Optional[torch.Tensor], dtype=None, name="tensor") -> C.c_void_p:
    if t is None:
        return C.c_void_p(0)
    if not t.is_cuda:
        raise ValueError("%s must live on the GPU" % name)
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    if dtype is not None and t.dtype != dtype:
        raise ValueError("%s must be %s, got %s" % (name, dtype, t.dtype))
    return C.c_void_p(t.data_ptr())


def _stream(stream) -> C.c_void_p:
    if stream is None:
        if not torch.cuda.is_available():     # host-only argument checks: nothing will be launched
            return C.c_void_p(0)
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


class Rap:
    """The loaded library.  Method names are the C entry points."""

    def __init__(self, path: Optional[str] = None):
        path = path or library_path()
        if not os.path.exists(path):
            raise RapError(-1, "%s is missing: build it with `python -m paper_2602_02599_amd.build` "
                               "(or __graft_entry__.build()); there is no fallback path" % path)
        self.path = path
        self.lib = C.CDLL(path)
        L = self.lib
        L.rap_rope_append.restype = C.c_int
        L.rap_rope_append.argtypes = [C.POINTER(RapShape), C.c_int32] + [C.c_void_p] * 7
        L.rap_decode_attn_workspace_bytes.restype = C.c_size_t
        L.rap_decode_attn_workspace_bytes.argtypes = [C.POINTER(RapShape), C.c_int64, C.POINTER(RapTuning)]
        L.rap_decode_attn.restype = C.c_int
        L.rap_decode_attn.argtypes = [C.POINTER(RapShape), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64,
                                      C.c_void_p, C.c_float, C.c_void_p, C.c_size_t, C.POINTER(RapTuning), C.c_void_p]
        if hasattr(L, "rap_decode_attn_static"):
            L.rap_decode_attn_static.restype = C.c_int
            L.rap_decode_attn_static.argtypes = [C.POINTER(RapShape), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64,
                                                 C.c_void_p, C.c_float, C.POINTER(RapTuning), C.c_void_p]
        if hasattr(L, "rap_rope_append_mx4"):
            L.rap_rope_append_mx4.restype = C.c_int
            L.rap_rope_append_mx4.argtypes = [C.POINTER(RapShape), C.c_int32] + [C.c_void_p] * 9
            L.rap_decode_attn_mx4.restype = C.c_int
            L.rap_decode_attn_mx4.argtypes = [C.POINTER(RapShape)] + [C.c_void_p] * 6 + [C.c_int64, C.c_void_p, C.c_float,
                                               C.c_void_p, C.c_size_t, C.POINTER(RapTuning), C.c_void_p]
        L.rap_decode_attn_rope.restype = C.c_int
        L.rap_decode_attn_rope.argtypes = [C.POINTER(RapShape), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                           C.c_void_p, C.c_int64, C.c_void_p, C.c_float, C.c_void_p, C.c_size_t,
                                           C.POINTER(RapTuning), C.c_void_p]
        if hasattr(L, "rap_decode_step"):
            L.rap_decode_step.restype = C.c_int
            L.rap_decode_step.argtypes = [C.POINTER(RapShape), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                          C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_float, C.c_void_p,
                                          C.c_size_t, C.POINTER(RapTuning), C.c_void_p]
        L.rap_rope_queries.restype = C.c_int
        L.rap_rope_queries.argtypes = [C.POINTER(RapShape), C.c_int32] + [C.c_void_p] * 5
        L.rap_prefill_attn.restype = C.c_int
        L.rap_prefill_attn.argtypes = [C.POINTER(RapShape), C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                       C.c_int64, C.c_void_p, C.c_float, C.c_void_p]
        L.rap_prefill_attn_paged.restype = C.c_int
        L.rap_prefill_attn_paged.argtypes = [C.POINTER(RapShape), C.POINTER(RapPaging), C.c_int32, C.c_void_p, C.c_void_p,
                                             C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_float, C.c_void_p]
        L.rap_rope_append_paged.restype = C.c_int
        L.rap_rope_append_paged.argtypes = [C.POINTER(RapShape), C.POINTER(RapPaging), C.c_int32] + [C.c_void_p] * 7
        L.rap_decode_attn_paged.restype = C.c_int
        L.rap_decode_attn_paged.argtypes = [C.POINTER(RapShape), C.POINTER(RapPaging), C.c_void_p, C.c_void_p, C.c_void_p,
                                            C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_float,
                                            C.c_void_p, C.c_size_t, C.POINTER(RapTuning), C.c_void_p]
        L.rap_rope_append_q8.restype = C.c_int
        L.rap_rope_append_q8.argtypes = [C.POINTER(RapShape), C.c_int32] + [C.c_void_p] * 9
        L.rap_decode_attn_q8.restype = C.c_int
        L.rap_decode_attn_q8.argtypes = [C.POINTER(RapShape), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                         C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_float,
                                         C.c_void_p, C.c_size_t, C.POINTER(RapTuning), C.c_void_p]
        L.rap_rope_append_paged_q8.restype = C.c_int
        L.rap_rope_append_paged_q8.argtypes = [C.POINTER(RapShape), C.POINTER(RapPaging), C.c_int32] + [C.c_void_p] * 9
        L.rap_decode_attn_paged_q8.restype = C.c_int
        L.rap_decode_attn_paged_q8.argtypes = [C.POINTER(RapShape), C.POINTER(RapPaging)] + [C.c_void_p] * 8 + [
            C.c_int64, C.c_void_p, C.c_float, C.c_void_p, C.c_size_t, C.POINTER(RapTuning), C.c_void_p]
        L.rap_decode_step_ex.restype = C.c_int
        L.rap_decode_step_ex.argtypes = [C.POINTER(RapShape), C.POINTER(RapKvCache)] + [C.c_void_p] * 5 + [
            C.c_int32, C.c_void_p, C.c_int64, C.c_void_p, C.c_float, C.c_void_p, C.c_size_t, C.POINTER(RapTuning), C.c_void_p]
        L.rap_prefill_attn_ex.restype = C.c_int
        L.rap_prefill_attn_ex.argtypes = [C.POINTER(RapShape), C.POINTER(RapKvCache), C.c_int32, C.c_void_p, C.c_void_p,
                                          C.c_int64, C.c_void_p, C.c_float, C.c_void_p]
        L.rap_prefill_attn_split_workspace_bytes.restype = C.c_size_t
        L.rap_prefill_attn_split_workspace_bytes.argtypes = [C.POINTER(RapShape), C.c_int32, C.c_int64]
        L.rap_prefill_attn_split.restype = C.c_int
        L.rap_prefill_attn_split.argtypes = [C.POINTER(RapShape), C.POINTER(RapKvCache), C.c_int32, C.c_void_p, C.c_void_p,
                                             C.c_int64, C.c_void_p, C.c_float, C.c_void_p, C.c_size_t, C.c_void_p]
        L.rap_decode_attn_multi.restype = C.c_int
        L.rap_decode_attn_multi.argtypes = [C.POINTER(RapShape), C.POINTER(RapKvCache), C.c_int32, C.c_void_p, C.c_void_p,
                                            C.c_int64, C.c_void_p, C.c_float, C.c_void_p, C.c_size_t,
                                            C.POINTER(RapTuning), C.c_void_p]
        L.rap_check_inputs.restype = C.c_int
        L.rap_check_inputs.argtypes = [C.POINTER(RapShape), C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64,
                                       C.c_void_p, C.c_void_p]
        L.rap_stream_read.restype = C.c_int
        L.rap_stream_read.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
        L.rap_stream_copy.restype = C.c_int
        L.rap_stream_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.rap_status_str.restype = C.c_char_p
        L.rap_status_str.argtypes = [C.c_int]
        L.rap_version.restype = C.c_int32
        L.rap_version.argtypes = []

    # -- helpers
    def _check(self, status: int):
        if status != 0:
            raise RapError(status, self.lib.rap_status_str(status).decode())

    def rap_status_str(self, status: int) -> str:
        return self.lib.rap_status_str(status).decode()

    def rap_version(self) -> int:
        return int(self.lib.rap_version())

    @staticmethod
    def shape(batch, n_q_heads, n_kv_heads, d_head, n_pairs, d_v, cache_cap, rope_theta, pair_inv_freq=None) -> RapShape:
        """pair_inv_freq: optional float64 GPU tensor [n_kv_heads, n_pairs] (see rap_shape_t); the
        returned object keeps a reference to it."""
        if pair_inv_freq is not None and tuple(pair_inv_freq.shape) != (n_kv_heads, n_pairs):
            raise ValueError("pair_inv_freq must be [n_kv_heads, n_pairs]")
        shp = RapShape(batch, n_q_heads, n_kv_heads, d_head, n_pairs, d_v, cache_cap, rope_theta,
                       _ptr(pair_inv_freq, torch.float64, "pair_inv_freq"))
        shp._keep_alive = pair_inv_freq
        return shp

    @staticmethod
    def paging(page_rows: int, n_pages: int, block_table) -> RapPaging:
        """block_table: int32 GPU tensor [batch, max_pages]; the returned object keeps a reference."""
        pg = RapPaging(page_rows, n_pages, int(block_table.shape[1]), 0, _ptr(block_table, torch.int32, "block_table"))
        pg._keep_alive = block_table
        return pg

    @staticmethod
    def tuning(kernel=0, rows_per_split=0, ev_main_start=None, ev_main_stop=None) -> RapTuning:
        return RapTuning(kernel, rows_per_split, 0, 0, ev_main_start, ev_main_stop)

    # -- entry points
    def rap_rope_append(self, shape: RapShape, n_new: int, k_new, v_new, pos, keep_pair_idx, k_cache, v_cache,
                        stream=None, check=True) -> int:
        st = self.lib.rap_rope_append(C.byref(shape), n_new, _ptr(k_new, torch.bfloat16, "k_new"),
                                      _ptr(v_new, torch.bfloat16, "v_new"), _ptr(pos, torch.int32, "pos"),
                                      _ptr(keep_pair_idx, torch.int32, "keep_pair_idx"),
                                      _ptr(k_cache, torch.bfloat16, "k_cache"), _ptr(v_cache, torch.bfloat16, "v_cache"),
                                      _stream(stream))
        if check:
            self._check(st)
        return st

    def rap_decode_attn_workspace_bytes(self, shape: RapShape, max_seq_len: int, tuning: Optional[RapTuning] = None) -> int:
        return int(self.lib.rap_decode_attn_workspace_bytes(C.byref(shape), max_seq_len,
                                                            C.byref(tuning) if tuning is not None else None))

    def rap_decode_attn(self, shape: RapShape, q, k_cache, v_cache, seq_lens, max_seq_len: int, out, scale: float,
                        workspace=None, tuning: Optional[RapTuning] = None, stream=None, check=True) -> int:
        st = self.lib.rap_decode_attn(C.byref(shape), _ptr(q, torch.bfloat16, "q"), _ptr(k_cache, torch.bfloat16, "k_cache"),
                                      _ptr(v_cache, torch.bfloat16, "v_cache"), _ptr(seq_lens, torch.int32, "seq_lens"),
                                      max_seq_len, _ptr(out, torch.float32, "out"), scale,
                                      _ptr(workspace, None, "workspace"),
                                      0 if workspace is None else workspace.numel() * workspace.element_size(),
                                      C.byref(tuning) if tuning is not None else None, _stream(stream))
        if check:
            self._check(st)
        return st

    def rap_decode_attn_static(self, shape: RapShape, q, k_cache, v_cache, seq_lens, max_seq_len: int, out, scale: float,
                               tuning: Optional[RapTuning] = None, stream=None, check=True) -> int:
        st = self.lib.rap_decode_attn_static(C.byref(shape), _ptr(q, torch.bfloat16, "q"), _ptr(k_cache, torch.bfloat16, "k_cache"),
                                             _ptr(v_cache, torch.bfloat16, "v_cache"), _ptr(seq_lens, torch.int32, "seq_lens"),
                                             max_seq_len, _ptr(out, torch.float32, "out"), scale,
                                             C.byref(tuning) if tuning is not None else None, _stream(stream))
        if check:
            self._check(st)
        return st

    def rap_decode_attn_rope(self, shape: RapShape, q, q_pos, keep_pair_idx, k_cache, v_cache, seq_lens, max_seq_len: int,
                             out, scale: float, workspace=None, tuning: Optional[RapTuning] = None, stream=None,
                             check=True) -> int:
        st = self.lib.rap_decode_attn_rope(C.byref(shape), _ptr(q, torch.bfloat16, "q"), _ptr(q_pos, torch.int32, "q_pos"),
                                           _ptr(keep_pair_idx, torch.int32, "keep_pair_idx"),
                                           _ptr(k_cache, torch.bfloat16, "k_cache"), _ptr(v_cache, torch.bfloat16, "v_cache"),
                                           _ptr(seq_lens, torch.int32, "seq_lens"), max_seq_len,
                                           _ptr(out, torch.float32, "out"), scale, _ptr(workspace, None, "workspace"),
                                           0 if workspace is None else workspace.numel() * workspace.element_size(),
                                           C.byref(tuning) if tuning is not None else None, _stream(stream))
        if check:
            self._check(st)
        return st

    def rap_decode_step(self, shape: RapShape, k_new, v_new, pos, keep_pair_idx, q, q_is_rotated: bool, k_cache, v_cache,
                        seq_lens, max_seq_len: int, out, scale: float, workspace=None, tuning: Optional[RapTuning] = None,
                        stream=None, check=True) -> int:
        st = self.lib.rap_decode_step(C.byref(shape), _ptr(k_new, torch.bfloat16, "k_new"), _ptr(v_new, torch.bfloat16, "v_new"),
                                      _ptr(pos, torch.int32, "pos"), _ptr(keep_pair_idx, torch.int32, "keep_pair_idx"),
                                      _ptr(q, torch.bfloat16, "q"), 1 if q_is_rotated else 0,
                                      _ptr(k_cache, torch.bfloat16, "k_cache"), _ptr(v_cache, torch.bfloat16, "v_cache"),
                                      _ptr(seq_lens, torch.int32, "seq_lens"), max_seq_len, _ptr(out, torch.float32, "out"),
                                      scale, _ptr(workspace, None, "workspace"),
                                      0 if workspace is None else workspace.numel() * workspace.element_size(),
                                      C.byref(tuning) if tuning is not None else None, _stream(stream))
        if check:
            self._check(st)
        return st

    def rap_rope_queries(self, shape: RapShape, n_new: int, q, pos, keep_pair_idx, q_out, stream=None, check=True) -> int:
        st = self.lib.rap_rope_queries(C.byref(shape), n_new, _ptr(q, torch.bfloat16, "q"), _ptr(pos, torch.int32, "pos"),
                                       _ptr(keep_pair_idx, torch.int32, "keep_pair_idx"), _ptr(q_out, torch.bfloat16, "q_out"),
                                       _stream(stream))
        if check:
            self._check(st)
        return st

    def rap_prefill_attn(self, shape: RapShape, n_new: int, q, k_cache, v_cache, seq_lens, max_seq_len: int, out,
                         scale: float, stream=None, check=True) -> int:
        st = self.lib.rap_prefill_attn(C.byref(shape), n_new, _ptr(q, torch.bfloat16, "q"),
                                       _ptr(k_cache, torch.bfloat16, "k_cache"), _ptr(v_cache, torch.bfloat16, "v_cache"),
                                       _ptr(seq_lens, torch.int32, "seq_lens"), max_seq_len, _ptr(out, torch.float32, "out"),
                                       scale, _stream(stream))
        if check:
            self._check(st)
        return st

    def rap_prefill_attn_paged(self, shape: RapShape, paging: RapPaging, n_new: int, q, k_pool, v_pool, seq_lens,
                               max_seq_len: int, out, scale: float, stream=None, check=True) -> int:
        st = self.lib.rap_prefill_attn_paged(C.byref(shape), C.byref(paging), n_new, _ptr(q, torch.bfloat16, "q"),
                                             _ptr(k_pool, torch.bfloat16, "k_pool"), _ptr(v_pool, torch.bfloat16, "v_pool"),
                                             _ptr(seq_lens, torch.int32, "seq_lens"), max_seq_len,
                                             _ptr(out, torch.float32, "out"), scale, _stream(stream))
        if check:
            self._check(st)
        return st

    def rap_rope_append_paged(self, shape: RapShape, paging: RapPaging, n_new: int, k_new, v_new, pos, keep_pair_idx,
                              k_pool, v_pool, stream=None, check=True) -> int:
        st = self.lib.rap_rope_append_paged(C.byref(shape), C.byref(paging), n_new, _ptr(k_new, torch.bfloat16, "k_new"),
                                            _ptr(v_new, torch.bfloat16, "v_new"), _ptr(pos, torch.int32, "pos"),
                                            _ptr(keep_pair_idx, torch.int32, "keep_pair_idx"),
                                            _ptr(k_pool, torch.bfloat16, "k_pool"), _ptr(v_pool, torch.bfloat16, "v_pool"),
                                            _stream(stream))
        if check:
            self._check(st)
        return st

    def rap_decode_attn_paged(self, shape: RapShape, paging: RapPaging, q, q_pos, keep_pair_idx, k_pool, v_pool, seq_lens,
                              max_seq_len: int, out, scale: float, workspace=None, tuning: Optional[RapTuning] = None,
                              stream=None, check=True) -> int:
        st = self.lib.rap_decode_attn_paged(C.byref(shape), C.byref(paging), _ptr(q, torch.bfloat16, "q"),
                                            _ptr(q_pos, torch.int32, "q_pos"), _ptr(keep_pair_idx, torch.int32, "keep_pair_idx"),
                                            _ptr(k_pool, torch.bfloat16, "k_pool"), _ptr(v_pool, torch.bfloat16, "v_pool"),
                                            _ptr(seq_lens, torch.int32, "seq_lens"), max_seq_len, _ptr(out, torch.float32, "out"),
                                            scale, _ptr(workspace, None, "workspace"),
                                            0 if workspace is None else workspace.numel() * workspace.element_size(),
                                            C.byref(tuning) if tuning is not None else None, _stream(stream))
        if check:
            self._check(st)
        return st

    def rap_rope_append_q8(self, shape: RapShape, n_new: int, k_new, v_new, pos, keep_pair_idx, k_cache8, v_cache8,
                           k_scale, v_scale, stream=None, check=True) -> int:
        st = self.lib.rap_rope_append_q8(C.byref(shape), n_new, _ptr(k_new, torch.bfloat16, "k_new"),
                                         _ptr(v_new, torch.bfloat16, "v_new"), _ptr(pos, torch.int32, "pos"),
                                         _ptr(keep_pair_idx, torch.int32, "keep_pair_idx"),
                                         _ptr(k_cache8, torch.uint8, "k_cache8"), _ptr(v_cache8, torch.uint8, "v_cache8"),
                                         _ptr(k_scale, torch.float32, "k_scale"), _ptr(v_scale, torch.float32, "v_scale"),
                                         _stream(stream))
        if check:
            self._check(st)
        return st

    def rap_decode_attn_q8(self, shape: RapShape, q, q_pos, keep_pair_idx, k_cache8, v_cache8, k_scale, v_scale, seq_lens,
                           max_seq_len: int, out, scale: float, workspace=None, tuning: Optional[RapTuning] = None,
                           stream=None, check=True) -> int:
        st = self.lib.rap_decode_attn_q8(C.byref(shape), _ptr(q, torch.bfloat16, "q"), _ptr(q_pos, torch.int32, "q_pos"),
                                         _ptr(keep_pair_idx, torch.int32, "keep_pair_idx"),
                                         _ptr(k_cache8, torch.uint8, "k_cache8"), _ptr(v_cache8, torch.uint8, "v_cache8"),
                                         _ptr(k_scale, torch.float32, "k_scale"), _ptr(v_scale, torch.float32, "v_scale"),
                                         _ptr(seq_lens, torch.int32, "seq_lens"), max_seq_len, _ptr(out, torch.float32, "out"),
                                         scale, _ptr(workspace, None, "workspace"),
                                         0 if workspace is None else workspace.numel() * workspace.element_size(),
                                         C.byref(tuning) if tuning is not None else None, _stream(stream))
        if check:
            self._check(st)
        return st

    def rap_rope_append_mx4(self, shape: RapShape, n_new: int, k_new, v_new, pos, keep_pair_idx, k_codes, k_scales,
                            v_codes, v_scales, stream=None, check=True) -> int:
        st = self.lib.rap_rope_append_mx4(C.byref(shape), n_new, _ptr(k_new, torch.bfloat16, "k_new"),
                                          _ptr(v_new, torch.bfloat16, "v_new"), _ptr(pos, torch.int32, "pos"),
                                          _ptr(keep_pair_idx, torch.int32, "keep_pair_idx"),
                                          _ptr(k_codes, torch.uint8, "k_codes"), _ptr(k_scales, torch.uint8, "k_scales"),
                                          _ptr(v_codes, torch.uint8, "v_codes"), _ptr(v_scales, torch.uint8, "v_scales"),
                                          _stream(stream))
        if check:
            self._check(st)
        return st

    def rap_decode_attn_mx4(self, shape: RapShape, q, k_codes, k_scales, v_codes, v_scales, seq_lens, max_seq_len: int, out,
                            scale: float, workspace=None, tuning: Optional[RapTuning] = None, stream=None, check=True) -> int:
        st = self.lib.rap_decode_attn_mx4(C.byref(shape), _ptr(q, torch.bfloat16, "q"),
                                          _ptr(k_codes, torch.uint8, "k_codes"), _ptr(k_scales, torch.uint8, "k_scales"),
                                          _ptr(v_codes, torch.uint8, "v_codes"), _ptr(v_scales, torch.uint8, "v_scales"),
                                          _ptr(seq_lens, torch.int32, "seq_lens"), max_seq_len, _ptr(out, torch.float32, "out"),
                                          scale, _ptr(workspace, None, "workspace"),
                                          0 if workspace is None else workspace.numel() * workspace.element_size(),
                                          C.byref(tuning) if tuning is not None else None, _stream(stream))
        if check:
            self._check(st)
        return st

    def rap_rope_append_paged_q8(self, shape: RapShape, paging: RapPaging, n_new: int, k_new, v_new, pos, keep_pair_idx,
                                 k_pool8, v_pool8, k_scale, v_scale, stream=None, check=True) -> int:
        st = self.lib.rap_rope_append_paged_q8(C.byref(shape), C.byref(paging), n_new, _ptr(k_new, torch.bfloat16, "k_new"),
                                               _ptr(v_new, torch.bfloat16, "v_new"), _ptr(pos, torch.int32, "pos"),
                                               _ptr(keep_pair_idx, torch.int32, "keep_pair_idx"),
                                               _ptr(k_pool8, torch.uint8, "k_pool8"), _ptr(v_pool8, torch.uint8, "v_pool8"),
                                               _ptr(k_scale, torch.float32, "k_scale"), _ptr(v_scale, torch.float32, "v_scale"),
                                               _stream(stream))
        if check:
            self._check(st)
        return st

    def rap_decode_attn_paged_q8(self, shape: RapShape, paging: RapPaging, q, q_pos, keep_pair_idx, k_pool8, v_pool8,
                                 k_scale, v_scale, seq_lens, max_seq_len: int, out, scale: float, workspace=None,
                                 tuning: Optional[RapTuning] = None, stream=None, check=True) -> int:
        st = self.lib.rap_decode_attn_paged_q8(C.byref(shape), C.byref(paging), _ptr(q, torch.bfloat16, "q"),
                                               _ptr(q_pos, torch.int32, "q_pos"), _ptr(keep_pair_idx, torch.int32, "keep_pair_idx"),
                                               _ptr(k_pool8, torch.uint8, "k_pool8"), _ptr(v_pool8, torch.uint8, "v_pool8"),
                                               _ptr(k_scale, torch.float32, "k_scale"), _ptr(v_scale, torch.float32, "v_scale"),
                                               _ptr(seq_lens, torch.int32, "seq_lens"), max_seq_len,
                                               _ptr(out, torch.float32, "out"), scale, _ptr(workspace, None, "workspace"),
                                               0 if workspace is None else workspace.numel() * workspace.element_size(),
                                               C.byref(tuning) if tuning is not None else None, _stream(stream))
        if check:
            self._check(st)
        return st

    def rap_decode_step_ex(self, shape: RapShape, k, v, k_scale, v_scale, paging: Optional[RapPaging], k_new, v_new, pos,
                           keep_pair_idx, q, q_is_rotated: bool, seq_lens, max_seq_len: int, out, scale: float,
                           workspace=None, tuning: Optional[RapTuning] = None, stream=None, check=True) -> int:
        """k, v: bf16 caches or pools, or uint8 ones with k_scale / v_scale; paging None for dense caches."""
        el = torch.uint8 if k_scale is not None else torch.bfloat16
        cache = RapKvCache(_ptr(k, el, "k"), _ptr(v, el, "v"), _ptr(k_scale, torch.float32, "k_scale"),
                           _ptr(v_scale, torch.float32, "v_scale"), C.pointer(paging) if paging is not None else None)
        st = self.lib.rap_decode_step_ex(C.byref(shape), C.byref(cache), _ptr(k_new, torch.bfloat16, "k_new"),
                                         _ptr(v_new, torch.bfloat16, "v_new"), _ptr(pos, torch.int32, "pos"),
                                         _ptr(keep_pair_idx, torch.int32, "keep_pair_idx"), _ptr(q, torch.bfloat16, "q"),
                                         1 if q_is_rotated else 0, _ptr(seq_lens, torch.int32, "seq_lens"), max_seq_len,
                                         _ptr(out, torch.float32, "out"), scale, _ptr(workspace, None, "workspace"),
                                         0 if workspace is None else workspace.numel() * workspace.element_size(),
                                         C.byref(tuning) if tuning is not None else None, _stream(stream))
        if check:
            self._check(st)
        return st

    def rap_prefill_attn_ex(self, shape: RapShape, k, v, k_scale, v_scale, paging: Optional[RapPaging], n_new: int, q,
                            seq_lens, max_seq_len: int, out, scale: float, stream=None, check=True) -> int:
        """k, v: bf16 caches or pools, or uint8 ones with k_scale / v_scale; paging None for dense caches."""
        el = torch.uint8 if k_scale is not None else torch.bfloat16
        cache = RapKvCache(_ptr(k, el, "k"), _ptr(v, el, "v"), _ptr(k_scale, torch.float32, "k_scale"),
                           _ptr(v_scale, torch.float32, "v_scale"), C.pointer(paging) if paging is not None else None)
        st = self.lib.rap_prefill_attn_ex(C.byref(shape), C.byref(cache), n_new, _ptr(q, torch.bfloat16, "q"),
                                          _ptr(seq_lens, torch.int32, "seq_lens"), max_seq_len,
                                          _ptr(out, torch.float32, "out"), scale, _stream(stream))
        if check:
            self._check(st)
        return st

    def rap_prefill_attn_split_workspace_bytes(self, shape: RapShape, n_new: int, max_seq_len: int) -> int:
        return int(self.lib.rap_prefill_attn_split_workspace_bytes(C.byref(shape), n_new, max_seq_len))

    def rap_prefill_attn_split(self, shape: RapShape, k, v, k_scale, v_scale, paging: Optional[RapPaging], n_new: int, q,
                               seq_lens, max_seq_len: int, out, scale: float, workspace, stream=None, check=True) -> int:
        """rap_prefill_attn_ex with a workspace (uint8 tensor of rap_prefill_attn_split_workspace_bytes, or None)."""
        el = torch.uint8 if k_scale is not None else torch.bfloat16
        cache = RapKvCache(_ptr(k, el, "k"), _ptr(v, el, "v"), _ptr(k_scale, torch.float32, "k_scale"),
                           _ptr(v_scale, torch.float32, "v_scale"), C.pointer(paging) if paging is not None else None)
        st = self.lib.rap_prefill_attn_split(C.byref(shape), C.byref(cache), n_new, _ptr(q, torch.bfloat16, "q"),
                                             _ptr(seq_lens, torch.int32, "seq_lens"), max_seq_len,
                                             _ptr(out, torch.float32, "out"), scale, _ptr(workspace, None, "workspace"),
                                             0 if workspace is None else workspace.numel() * workspace.element_size(),
                                             _stream(stream))
        if check:
            self._check(st)
        return st

    def rap_decode_attn_multi(self, shape: RapShape, k, v, k_scale, v_scale, paging: Optional[RapPaging], n_tok: int, q,
                              seq_lens, max_seq_len: int, out, scale: float, workspace, tuning=None, stream=None,
                              check=True) -> int:
        """k, v: bf16 caches or pools, or uint8 ones with k_scale / v_scale; paging None for dense caches."""
        el = torch.uint8 if k_scale is not None else torch.bfloat16
        cache = RapKvCache(_ptr(k, el, "k"), _ptr(v, el, "v"), _ptr(k_scale, torch.float32, "k_scale"),
                           _ptr(v_scale, torch.float32, "v_scale"), C.pointer(paging) if paging is not None else None)
        st = self.lib.rap_decode_attn_multi(C.byref(shape), C.byref(cache), n_tok, _ptr(q, torch.bfloat16, "q"),
                                            _ptr(seq_lens, torch.int32, "seq_lens"), max_seq_len,
                                            _ptr(out, torch.float32, "out"), scale, _ptr(workspace, None, "workspace"),
                                            0 if workspace is None else workspace.numel() * workspace.element_size(),
                                            C.byref(tuning) if tuning is not None else None, _stream(stream))
        if check:
            self._check(st)
        return st

    def rap_check_inputs(self, shape: RapShape, n_new: int, pos, keep_pair_idx, seq_lens, max_seq_len: int, flags,
                         stream=None, check=True) -> int:
        """flags: one int32/uint32 word on the device, zeroed by the caller; bits as RAP_FLAG_* in rap.h."""
        st = self.lib.rap_check_inputs(C.byref(shape), n_new, _ptr(pos, torch.int32, "pos"),
                                       _ptr(keep_pair_idx, torch.int32, "keep_pair_idx"),
                                       _ptr(seq_lens, torch.int32, "seq_lens"), max_seq_len, _ptr(flags, torch.int32, "flags"),
                                       _stream(stream))
        if check:
            self._check(st)
        return st

    def rap_stream_read(self, src, sink, stream=None):
        self._check(self.lib.rap_stream_read(_ptr(src), src.numel() * src.element_size(), _ptr(sink), _stream(stream)))

    def rap_stream_copy(self, dst, src, stream=None):
        self._check(self.lib.rap_stream_copy(_ptr(dst), _ptr(src), src.numel() * src.element_size(), _stream(stream)))

    # -- convenience on top of the entry points (allocation of scratch and output only)
    def new_workspace(self, shape: RapShape, max_seq_len: int, tuning=None, device="cuda", n_tok: int = 1) -> torch.Tensor:
        n = self.rap_decode_attn_workspace_bytes(shape, max_seq_len, tuning)
        if n == 0:
            raise RapError(2, "workspace query rejected the shape")
        return torch.empty(n * n_tok, dtype=torch.uint8, device=device)


_LOADED: Optional[Rap] = None


def load(path: Optional[str] = None) -> Rap:
    """Load librap.so (once).  Raises RapError if it has not been built."""
    global _LOADED
    if _LOADED is None or (path is not None and path != _LOADED.path):
        _LOADED = Rap(path)
    return _LOADED
