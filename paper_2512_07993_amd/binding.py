"""Thin ctypes binding of libskipkv.so: argument marshalling only.

Every function has the name and argument order of the C entry point in include/skipkv.h.
Tensors are torch tensors used purely as device-memory handles (data_ptr()); all work
runs in the library's HIP kernels on the current torch stream unless `stream` is given.
There is no fallback: if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import torch

F32, BF16 = 0, 1
OK, EINVAL, EBUDGET, ECAPACITY, EWORKSPACE, EHIP = 0, -1, -2, -3, -4, -5
DEV_BAD_OFFSETS, DEV_TOO_MANY_SENT, DEV_TIMEOUT, DEV_TOO_MANY_TOK, DEV_BAD_BLOCK_TABLE, DEV_BAD_BUDGET, DEV_BAD_SCORES = 1, 2, 4, 8, 16, 32, 64
FLAG_FORCE_TWO_PASS = 1
PROFILE_SLOTS = 16

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libskipkv.so")
_lib = None


class CCache(C.Structure):
    _fields_ = [
        ("k", C.c_void_p), ("v", C.c_void_p),
        ("stride_layer", C.c_int64), ("stride_head", C.c_int64), ("stride_tok", C.c_int64),
        ("dtype", C.c_int32), ("n_layers", C.c_int32), ("n_kv_heads", C.c_int32),
        ("n_q_heads", C.c_int32), ("head_dim", C.c_int32), ("batch", C.c_int32),
        ("total_tokens", C.c_int32), ("total_sentences", C.c_int32),
        ("seq_off", C.c_void_p), ("sent_ptr", C.c_void_p), ("sent_off", C.c_void_p),
    ]


class CRanges(C.Structure):
    _fields_ = [("len", C.c_void_p), ("sent_cnt", C.c_void_p), ("sent_off", C.c_void_p)]


class CPaging(C.Structure):
    _fields_ = [("block_table", C.c_void_p), ("table_stride", C.c_int32), ("block_size", C.c_int32),
                ("n_blocks", C.c_int32), ("stride_block", C.c_int64)]


class CParams(C.Structure):
    _fields_ = [
        ("obs_window", C.c_int32), ("protect_window", C.c_int32),
        ("sigma", C.c_float), ("tau", C.c_float),
        ("budget", C.c_void_p), ("budget_scalar", C.c_int32), ("max_budget", C.c_int32),
        ("dev_status", C.c_void_p), ("profile", C.c_void_p),
        ("flags", C.c_uint32), ("spin_limit", C.c_int32),
    ]


def lib() -> C.CDLL:
    """Load libskipkv.so (built by paper_2512_07993_amd.build); raise if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(
                "libskipkv.so is not built: run `python -m paper_2512_07993_amd.build` "
                "(there is no CPU fallback)")
        L = C.CDLL(_LIB_PATH)
        vp, i32, sz, fl = C.c_void_p, C.c_int32, C.c_size_t, C.c_float
        cp, pp = C.POINTER(CCache), C.POINTER(CParams)
        L.skipkv_workspace_bytes.argtypes = [cp, pp, C.POINTER(sz)]
        L.skipkv_score.argtypes = [cp, pp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.skipkv_select.argtypes = [cp, pp, vp, vp, vp, vp, vp, vp, i32, vp]
        L.skipkv_compact.argtypes = [cp, vp, vp, i32, vp]
        L.skipkv_step.argtypes = [cp, pp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, sz, vp]
        L.skipkv_step_static.argtypes = [cp, pp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp]
        L.skipkv_select_tokens.argtypes = [cp, pp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp]
        L.skipkv_redundancy_workspace_bytes.argtypes = [cp, C.POINTER(sz)]
        L.skipkv_token_redundancy.argtypes = [cp, vp, vp, sz, vp]
        L.skipkv_steer_add.argtypes = [vp, vp, vp, fl, vp, i32, i32, i32, vp]
        L.skipkv_similarity_workspace_bytes.argtypes = [cp, i32, C.POINTER(sz)]
        L.skipkv_sentence_similarity.argtypes = [cp, vp, i32, i32, vp, vp, sz, vp]
        L.skipkv_score_shared.argtypes = [cp, pp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.skipkv_steer_strength.argtypes = [vp, fl, fl, vp, i32, vp]
        rp = C.POINTER(CRanges)
        L.skipkv_ranges_workspace_bytes.argtypes = [cp, pp, C.POINTER(sz)]
        L.skipkv_ranges_append.argtypes = [cp, rp, vp, vp, vp, vp, vp]
        L.skipkv_token_redundancy_ranges.argtypes = [cp, rp, vp, vp, sz, vp]
        L.skipkv_score_ranges.argtypes = [cp, rp, pp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.skipkv_select_tokens_ranges.argtypes = [cp, rp, pp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, sz, vp]
        L.skipkv_select_ranges.argtypes = [cp, rp, pp, vp, vp, vp, vp, vp, vp, i32, vp, sz, vp]
        L.skipkv_ranges_ids_select.argtypes = [cp, rp, i32, vp, vp, vp, vp]
        L.skipkv_ranges_ids_append.argtypes = [cp, vp, vp, vp, vp]
        L.skipkv_score_shared_ranges.argtypes = [cp, rp, vp, vp, pp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.skipkv_step_ranges.argtypes = [cp, rp, pp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, sz, vp]
        gp = C.POINTER(CPaging)
        L.skipkv_paged_workspace_bytes.argtypes = [cp, gp, pp, C.POINTER(sz)]
        L.skipkv_step_paged.argtypes = [cp, gp, pp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, sz, vp]
        L.skipkv_score_paged.argtypes = [cp, gp, pp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.skipkv_score_shared_paged.argtypes = [cp, gp, pp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.skipkv_compact_paged_workspace_bytes.argtypes = [cp, gp, i32, C.POINTER(sz)]
        L.skipkv_compact_paged.argtypes = [cp, gp, vp, vp, i32, vp, vp, sz, vp]
        L.skipkv_redundancy_paged_workspace_bytes.argtypes = [cp, gp, C.POINTER(sz)]
        L.skipkv_token_redundancy_paged.argtypes = [cp, gp, vp, vp, vp, sz, vp]
        L.skipkv_score_ranges_paged.argtypes = [cp, rp, gp, vp, vp, vp, pp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.skipkv_token_redundancy_ranges_paged.argtypes = [cp, rp, gp, vp, vp, vp, sz, vp]
        L.skipkv_ranges_paged_workspace_bytes.argtypes = [cp, gp, pp, C.POINTER(sz)]
        L.skipkv_step_ranges_paged.argtypes = [cp, rp, gp, pp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, sz, vp]
        L.skipkv_profile_create.argtypes = [C.POINTER(vp)]
        L.skipkv_profile_read.argtypes = [vp, C.POINTER(i32), C.POINTER(C.c_char_p), C.POINTER(fl)]
        L.skipkv_profile_destroy.argtypes = [vp]
        L.skipkv_strerror.argtypes = [C.c_int]
        L.skipkv_strerror.restype = C.c_char_p
        L.skipkv_version.argtypes = []
        for name in ("skipkv_workspace_bytes", "skipkv_score", "skipkv_select", "skipkv_compact", "skipkv_step",
                     "skipkv_steer_add", "skipkv_redundancy_workspace_bytes", "skipkv_token_redundancy",
                     "skipkv_select_tokens", "skipkv_ranges_workspace_bytes", "skipkv_ranges_append", "skipkv_step_ranges",
                     "skipkv_similarity_workspace_bytes", "skipkv_sentence_similarity", "skipkv_score_shared", "skipkv_steer_strength",
                     "skipkv_paged_workspace_bytes", "skipkv_step_paged",
                     "skipkv_profile_create", "skipkv_profile_read", "skipkv_profile_destroy",
                     "skipkv_version"):
            getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


class SkipKVError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__("libskipkv: %s (%d)" % (lib().skipkv_strerror(status).decode(), status))


def _check(status: int) -> None:
    if status != OK:
        raise SkipKVError(status)


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else None
    return stream if isinstance(stream, int) else stream.cuda_stream


def dtype_code(t: torch.dtype) -> int:
    if t == torch.float32:
        return F32
    if t == torch.bfloat16:
        return BF16
    raise ValueError("unsupported dtype %s" % t)


@dataclass
class Cache:
    """Python mirror of skipkv_cache.  k, v: [L, Hk, T, D] tensors (any strides with D contiguous)."""
    k: torch.Tensor
    v: torch.Tensor
    n_q_heads: int
    seq_off: torch.Tensor      # int32 device [B+1]
    sent_ptr: torch.Tensor     # int32 device [B+1]
    sent_off: torch.Tensor     # int32 device [S_total + B]
    total_tokens: int
    total_sentences: int

    @property
    def batch(self) -> int:
        return int(self.seq_off.numel()) - 1

    def c(self) -> CCache:
        k = self.k
        assert k.dim() == 4 and k.stride(3) == 1 and self.v.stride() == k.stride() and self.v.shape == k.shape
        return CCache(k.data_ptr(), self.v.data_ptr(), k.stride(0), k.stride(1), k.stride(2), dtype_code(k.dtype),
                      k.shape[0], k.shape[1], self.n_q_heads, k.shape[3], self.batch,
                      self.total_tokens, self.total_sentences,
                      _ptr(self.seq_off), _ptr(self.sent_ptr), _ptr(self.sent_off))


@dataclass
class Params:
    """Python mirror of skipkv_params."""
    obs_window: int
    protect_window: int
    budget: "int | torch.Tensor"
    max_budget: int = -1
    sigma: float = 0.1
    tau: float = 0.95
    dev_status: Optional[torch.Tensor] = None
    profile: Optional[int] = None
    flags: int = 0
    spin_limit: int = 0

    def c(self) -> CParams:
        if isinstance(self.budget, int):
            bptr, bs = None, self.budget
            mb = self.budget if self.max_budget < 0 else self.max_budget
        else:
            bptr, bs, mb = self.budget.data_ptr(), 0, self.max_budget
        return CParams(self.obs_window, self.protect_window, self.sigma, self.tau, bptr, bs, mb,
                       _ptr(self.dev_status), self.profile, self.flags, self.spin_limit)


def skipkv_version() -> int:
    return lib().skipkv_version()


def skipkv_strerror(status: int) -> str:
    return lib().skipkv_strerror(status).decode()


def skipkv_workspace_bytes(cache: Cache, params: Params) -> int:
    out = C.c_size_t(0)
    _check(lib().skipkv_workspace_bytes(C.byref(cache.c()), C.byref(params.c()), C.byref(out)))
    return int(out.value)


def skipkv_score(cache: Cache, params: Params, q_obs, tok_redundancy, sent_score, sent_lambda, tok_importance,
                 ws, stream=None) -> None:
    _check(lib().skipkv_score(C.byref(cache.c()), C.byref(params.c()), _ptr(q_obs), _ptr(tok_redundancy),
                              _ptr(sent_score), _ptr(sent_lambda), _ptr(tok_importance), _ptr(ws),
                              ws.numel() * ws.element_size() if ws is not None else 0, _stream(stream)))


def skipkv_select(cache: Cache, params: Params, sent_score, sent_keep, kept_idx, new_len, new_sent_off,
                  new_sent_cnt, kept_stride: int, stream=None) -> None:
    _check(lib().skipkv_select(C.byref(cache.c()), C.byref(params.c()), _ptr(sent_score), _ptr(sent_keep),
                               _ptr(kept_idx), _ptr(new_len), _ptr(new_sent_off), _ptr(new_sent_cnt),
                               kept_stride, _stream(stream)))


def skipkv_select_tokens(cache: Cache, params: Params, tok_importance, tok_redundancy, sent_lambda, tok_score,
                         tok_keep, kept_idx, new_len, new_sent_off, new_sent_cnt, kept_stride: int, stream=None) -> None:
    _check(lib().skipkv_select_tokens(C.byref(cache.c()), C.byref(params.c()), _ptr(tok_importance),
                                      _ptr(tok_redundancy), _ptr(sent_lambda), _ptr(tok_score), _ptr(tok_keep),
                                      _ptr(kept_idx), _ptr(new_len), _ptr(new_sent_off), _ptr(new_sent_cnt),
                                      kept_stride, _stream(stream)))


def skipkv_compact(cache: Cache, kept_idx, new_len, kept_stride: int, stream=None) -> None:
    _check(lib().skipkv_compact(C.byref(cache.c()), _ptr(kept_idx), _ptr(new_len), kept_stride, _stream(stream)))


def skipkv_step(cache: Cache, params: Params, q_obs, tok_redundancy, sent_score, sent_lambda, tok_importance,
                sent_keep, kept_idx, new_len, new_sent_off, new_sent_cnt, kept_stride: int, ws, stream=None) -> None:
    _check(lib().skipkv_step(C.byref(cache.c()), C.byref(params.c()), _ptr(q_obs), _ptr(tok_redundancy),
                             _ptr(sent_score), _ptr(sent_lambda), _ptr(tok_importance), _ptr(sent_keep),
                             _ptr(kept_idx), _ptr(new_len), _ptr(new_sent_off), _ptr(new_sent_cnt), kept_stride,
                             _ptr(ws), ws.numel() * ws.element_size() if ws is not None else 0, _stream(stream)))


STATIC_WS_BYTES = 64 << 20  # SKIPKV_STATIC_WS_BYTES


def skipkv_step_static(cache: Cache, params: Params, q_obs, tok_redundancy, sent_score, sent_lambda, tok_importance,
                       sent_keep, kept_idx, new_len, new_sent_off, new_sent_cnt, kept_stride: int, stream=None) -> None:
    _check(lib().skipkv_step_static(C.byref(cache.c()), C.byref(params.c()), _ptr(q_obs), _ptr(tok_redundancy),
                                    _ptr(sent_score), _ptr(sent_lambda), _ptr(tok_importance), _ptr(sent_keep),
                                    _ptr(kept_idx), _ptr(new_len), _ptr(new_sent_off), _ptr(new_sent_cnt), kept_stride,
                                    _stream(stream)))


@dataclass
class Ranges:
    """Python mirror of skipkv_ranges: per-head lengths [L, Hk, B], sentence counts [L, Hk, B] and
    offsets [L, Hk, S_total + B] (int32 device tensors)."""
    len: torch.Tensor
    sent_cnt: torch.Tensor
    sent_off: torch.Tensor

    def c(self) -> CRanges:
        return CRanges(self.len.data_ptr(), self.sent_cnt.data_ptr(), self.sent_off.data_ptr())


def skipkv_ranges_workspace_bytes(cache: Cache, params: Params) -> int:
    out = C.c_size_t(0)
    _check(lib().skipkv_ranges_workspace_bytes(C.byref(cache.c()), C.byref(params.c()), C.byref(out)))
    return int(out.value)


def skipkv_ranges_append(cache: Cache, ranges: Ranges, n_new, bnd_ptr, bnd_off, dev_status=None, stream=None) -> None:
    _check(lib().skipkv_ranges_append(C.byref(cache.c()), C.byref(ranges.c()), _ptr(n_new), _ptr(bnd_ptr),
                                      _ptr(bnd_off), _ptr(dev_status), _stream(stream)))


def skipkv_step_ranges(cache: Cache, ranges: Ranges, params: Params, q_obs, tok_redundancy, sent_score, sent_lambda,
                       tok_importance, sent_keep, kept_idx, new_len, new_sent_off, new_sent_cnt, kept_stride: int, ws,
                       stream=None) -> None:
    _check(lib().skipkv_step_ranges(C.byref(cache.c()), C.byref(ranges.c()), C.byref(params.c()), _ptr(q_obs),
                                    _ptr(tok_redundancy), _ptr(sent_score), _ptr(sent_lambda), _ptr(tok_importance),
                                    _ptr(sent_keep), _ptr(kept_idx), _ptr(new_len), _ptr(new_sent_off),
                                    _ptr(new_sent_cnt), kept_stride, _ptr(ws),
                                    ws.numel() * ws.element_size() if ws is not None else 0, _stream(stream)))


def _nbytes(ws) -> int:
    return ws.numel() * ws.element_size() if ws is not None else 0


def skipkv_token_redundancy_ranges(cache: Cache, ranges: Ranges, tok_redundancy, ws, stream=None) -> None:
    _check(lib().skipkv_token_redundancy_ranges(C.byref(cache.c()), C.byref(ranges.c()), _ptr(tok_redundancy), _ptr(ws),
                                                _nbytes(ws), _stream(stream)))


def skipkv_score_ranges(cache: Cache, ranges: Ranges, params: Params, q_obs, tok_redundancy, sent_score, sent_lambda,
                        tok_importance, ws, stream=None) -> None:
    _check(lib().skipkv_score_ranges(C.byref(cache.c()), C.byref(ranges.c()), C.byref(params.c()), _ptr(q_obs),
                                     _ptr(tok_redundancy), _ptr(sent_score), _ptr(sent_lambda), _ptr(tok_importance),
                                     _ptr(ws), _nbytes(ws), _stream(stream)))


def skipkv_select_tokens_ranges(cache: Cache, ranges: Ranges, params: Params, tok_importance, tok_redundancy, sent_lambda,
                                tok_score, tok_keep, kept_idx, new_len, new_sent_off, new_sent_cnt, kept_stride: int, ws,
                                stream=None) -> None:
    _check(lib().skipkv_select_tokens_ranges(C.byref(cache.c()), C.byref(ranges.c()), C.byref(params.c()),
                                             _ptr(tok_importance), _ptr(tok_redundancy), _ptr(sent_lambda), _ptr(tok_score),
                                             _ptr(tok_keep), _ptr(kept_idx), _ptr(new_len), _ptr(new_sent_off),
                                             _ptr(new_sent_cnt), kept_stride, _ptr(ws), _nbytes(ws), _stream(stream)))


def skipkv_select_ranges(cache: Cache, ranges: Ranges, params: Params, sent_score, sent_keep, kept_idx, new_len, new_sent_off,
                         new_sent_cnt, kept_stride: int, ws, stream=None) -> None:
    _check(lib().skipkv_select_ranges(C.byref(cache.c()), C.byref(ranges.c()), C.byref(params.c()), _ptr(sent_score),
                                      _ptr(sent_keep), _ptr(kept_idx), _ptr(new_len), _ptr(new_sent_off), _ptr(new_sent_cnt),
                                      kept_stride, _ptr(ws), _nbytes(ws), _stream(stream)))


def skipkv_ranges_ids_select(cache: Cache, ranges, protect_window: int, sent_keep, sent_id_in, sent_id_out, stream=None) -> None:
    _check(lib().skipkv_ranges_ids_select(C.byref(cache.c()), C.byref(ranges.c()) if ranges is not None else None,
                                          protect_window, _ptr(sent_keep), _ptr(sent_id_in), _ptr(sent_id_out),
                                          _stream(stream)))


def skipkv_ranges_ids_append(cache: Cache, old_cnt, new_cnt, sent_id, stream=None) -> None:
    _check(lib().skipkv_ranges_ids_append(C.byref(cache.c()), _ptr(old_cnt), _ptr(new_cnt), _ptr(sent_id), _stream(stream)))


def skipkv_score_shared_ranges(cache: Cache, ranges: Ranges, sent_id, lambda_ptr, params: Params, q_obs, tok_redundancy,
                               shared_lambda, sent_score, sent_lambda, tok_importance, ws, stream=None) -> None:
    _check(lib().skipkv_score_shared_ranges(C.byref(cache.c()), C.byref(ranges.c()), _ptr(sent_id), _ptr(lambda_ptr),
                                            C.byref(params.c()), _ptr(q_obs), _ptr(tok_redundancy), _ptr(shared_lambda),
                                            _ptr(sent_score), _ptr(sent_lambda), _ptr(tok_importance), _ptr(ws), _nbytes(ws),
                                            _stream(stream)))


@dataclass
class PagedCache:
    """Python mirror of skipkv_cache + skipkv_paging for pools laid out [L, blocks, slots, Hk, D]
    (any strides with D contiguous); seq_off numbers the logical tokens."""
    k: torch.Tensor
    v: torch.Tensor
    block_table: torch.Tensor  # int32 device [B, table_stride]
    n_q_heads: int
    seq_off: torch.Tensor
    sent_ptr: torch.Tensor
    sent_off: torch.Tensor
    total_tokens: int
    total_sentences: int

    def c(self) -> CCache:
        k = self.k
        assert k.dim() == 5 and k.stride(4) == 1 and self.v.stride() == k.stride() and self.v.shape == k.shape
        return CCache(k.data_ptr(), self.v.data_ptr(), k.stride(0), k.stride(3), k.stride(2), dtype_code(k.dtype),
                      k.shape[0], k.shape[3], self.n_q_heads, k.shape[4], int(self.seq_off.numel()) - 1,
                      self.total_tokens, self.total_sentences,
                      _ptr(self.seq_off), _ptr(self.sent_ptr), _ptr(self.sent_off))

    def paging(self) -> CPaging:
        bt = self.block_table
        assert bt.dim() == 2 and bt.dtype == torch.int32 and bt.stride(1) == 1
        return CPaging(bt.data_ptr(), bt.stride(0), self.k.shape[2], self.k.shape[1], self.k.stride(1))


def skipkv_paged_workspace_bytes(cache: PagedCache, params: Params) -> int:
    out = C.c_size_t(0)
    _check(lib().skipkv_paged_workspace_bytes(C.byref(cache.c()), C.byref(cache.paging()), C.byref(params.c()), C.byref(out)))
    return int(out.value)


def skipkv_step_paged(cache: PagedCache, params: Params, q_obs, tok_redundancy, sent_score, sent_lambda, tok_importance,
                      sent_keep, kept_idx, new_len, new_sent_off, new_sent_cnt, kept_stride: int, ws, stream=None) -> None:
    _check(lib().skipkv_step_paged(C.byref(cache.c()), C.byref(cache.paging()), C.byref(params.c()), _ptr(q_obs),
                                   _ptr(tok_redundancy), _ptr(sent_score), _ptr(sent_lambda), _ptr(tok_importance),
                                   _ptr(sent_keep), _ptr(kept_idx), _ptr(new_len), _ptr(new_sent_off),
                                   _ptr(new_sent_cnt), kept_stride, _ptr(ws),
                                   ws.numel() * ws.element_size() if ws is not None else 0, _stream(stream)))


def skipkv_score_paged(cache: PagedCache, params: Params, q_obs, tok_redundancy, sent_score, sent_lambda, tok_importance,
                       ws, stream=None) -> None:
    _check(lib().skipkv_score_paged(C.byref(cache.c()), C.byref(cache.paging()), C.byref(params.c()), _ptr(q_obs),
                                    _ptr(tok_redundancy), _ptr(sent_score), _ptr(sent_lambda), _ptr(tok_importance),
                                    _ptr(ws), ws.numel() * ws.element_size() if ws is not None else 0, _stream(stream)))


def skipkv_score_shared_paged(cache: PagedCache, params: Params, q_obs, tok_redundancy, shared_lambda, sent_score, sent_lambda,
                              tok_importance, ws, stream=None) -> None:
    _check(lib().skipkv_score_shared_paged(C.byref(cache.c()), C.byref(cache.paging()), C.byref(params.c()), _ptr(q_obs),
                                           _ptr(tok_redundancy), _ptr(shared_lambda), _ptr(sent_score), _ptr(sent_lambda),
                                           _ptr(tok_importance), _ptr(ws), _nbytes(ws), _stream(stream)))


def skipkv_compact_paged_workspace_bytes(cache: PagedCache, kept_stride: int) -> int:
    out = C.c_size_t(0)
    _check(lib().skipkv_compact_paged_workspace_bytes(C.byref(cache.c()), C.byref(cache.paging()), kept_stride, C.byref(out)))
    return int(out.value)


def skipkv_compact_paged(cache: PagedCache, kept_idx, new_len, kept_stride: int, dev_status, ws, stream=None) -> None:
    _check(lib().skipkv_compact_paged(C.byref(cache.c()), C.byref(cache.paging()), _ptr(kept_idx), _ptr(new_len),
                                      kept_stride, _ptr(dev_status), _ptr(ws),
                                      ws.numel() * ws.element_size() if ws is not None else 0, _stream(stream)))


def skipkv_redundancy_paged_workspace_bytes(cache: PagedCache) -> int:
    out = C.c_size_t(0)
    _check(lib().skipkv_redundancy_paged_workspace_bytes(C.byref(cache.c()), C.byref(cache.paging()), C.byref(out)))
    return int(out.value)


def skipkv_token_redundancy_paged(cache: PagedCache, tok_redundancy, dev_status, ws, stream=None) -> None:
    _check(lib().skipkv_token_redundancy_paged(C.byref(cache.c()), C.byref(cache.paging()), _ptr(tok_redundancy),
                                               _ptr(dev_status), _ptr(ws),
                                               ws.numel() * ws.element_size() if ws is not None else 0, _stream(stream)))


def skipkv_score_ranges_paged(cache: PagedCache, ranges: Ranges, sent_id, lambda_ptr, shared_lambda, params: Params, q_obs,
                              tok_redundancy, sent_score, sent_lambda, tok_importance, ws, stream=None) -> None:
    _check(lib().skipkv_score_ranges_paged(C.byref(cache.c()), C.byref(ranges.c()), C.byref(cache.paging()), _ptr(sent_id),
                                           _ptr(lambda_ptr), _ptr(shared_lambda), C.byref(params.c()), _ptr(q_obs),
                                           _ptr(tok_redundancy), _ptr(sent_score), _ptr(sent_lambda), _ptr(tok_importance),
                                           _ptr(ws), _nbytes(ws), _stream(stream)))


def skipkv_token_redundancy_ranges_paged(cache: PagedCache, ranges: Ranges, tok_redundancy, dev_status, ws, stream=None) -> None:
    _check(lib().skipkv_token_redundancy_ranges_paged(C.byref(cache.c()), C.byref(ranges.c()), C.byref(cache.paging()),
                                                      _ptr(tok_redundancy), _ptr(dev_status), _ptr(ws), _nbytes(ws),
                                                      _stream(stream)))


def skipkv_ranges_paged_workspace_bytes(cache: PagedCache, params: Params) -> int:
    out = C.c_size_t(0)
    _check(lib().skipkv_ranges_paged_workspace_bytes(C.byref(cache.c()), C.byref(cache.paging()), C.byref(params.c()),
                                                     C.byref(out)))
    return int(out.value)


def skipkv_step_ranges_paged(cache: PagedCache, ranges: Ranges, params: Params, q_obs, tok_redundancy, sent_score,
                             sent_lambda, tok_importance, sent_keep, kept_idx, new_len, new_sent_off, new_sent_cnt,
                             kept_stride: int, ws, stream=None) -> None:
    _check(lib().skipkv_step_ranges_paged(C.byref(cache.c()), C.byref(ranges.c()), C.byref(cache.paging()),
                                          C.byref(params.c()), _ptr(q_obs), _ptr(tok_redundancy), _ptr(sent_score),
                                          _ptr(sent_lambda), _ptr(tok_importance), _ptr(sent_keep), _ptr(kept_idx),
                                          _ptr(new_len), _ptr(new_sent_off), _ptr(new_sent_cnt), kept_stride, _ptr(ws),
                                          ws.numel() * ws.element_size() if ws is not None else 0, _stream(stream)))


def skipkv_similarity_workspace_bytes(cache: Cache, d_model: int) -> int:
    out = C.c_size_t(0)
    _check(lib().skipkv_similarity_workspace_bytes(C.byref(cache.c()), d_model, C.byref(out)))
    return int(out.value)


def skipkv_sentence_similarity(cache: Cache, hidden, shared_lambda, ws, stream=None) -> None:
    assert hidden.dim() == 2 and hidden.is_contiguous()
    _check(lib().skipkv_sentence_similarity(C.byref(cache.c()), _ptr(hidden), hidden.shape[1], dtype_code(hidden.dtype),
                                            _ptr(shared_lambda), _ptr(ws),
                                            ws.numel() * ws.element_size() if ws is not None else 0, _stream(stream)))


def skipkv_score_shared(cache: Cache, params: Params, q_obs, tok_redundancy, shared_lambda, sent_score, sent_lambda,
                        tok_importance, ws, stream=None) -> None:
    _check(lib().skipkv_score_shared(C.byref(cache.c()), C.byref(params.c()), _ptr(q_obs), _ptr(tok_redundancy),
                                     _ptr(shared_lambda), _ptr(sent_score), _ptr(sent_lambda), _ptr(tok_importance),
                                     _ptr(ws), ws.numel() * ws.element_size() if ws is not None else 0, _stream(stream)))


def skipkv_redundancy_workspace_bytes(cache: Cache) -> int:
    out = C.c_size_t(0)
    _check(lib().skipkv_redundancy_workspace_bytes(C.byref(cache.c()), C.byref(out)))
    return int(out.value)


def skipkv_token_redundancy(cache: Cache, tok_redundancy, ws, stream=None) -> None:
    _check(lib().skipkv_token_redundancy(C.byref(cache.c()), _ptr(tok_redundancy), _ptr(ws),
                                         ws.numel() * ws.element_size() if ws is not None else 0, _stream(stream)))


def skipkv_steer_add(hidden, vec, coef, coef_scalar: float, row_mask, stream=None) -> None:
    rows, d_model = hidden.shape
    assert hidden.is_contiguous() and vec.is_contiguous() and vec.dtype == hidden.dtype
    _check(lib().skipkv_steer_add(_ptr(hidden), _ptr(vec), _ptr(coef), float(coef_scalar), _ptr(row_mask),
                                  rows, d_model, dtype_code(hidden.dtype), _stream(stream)))


def skipkv_steer_strength(n_nonexec, alpha0: float, gamma: float, coef, stream=None) -> None:
    _check(lib().skipkv_steer_strength(_ptr(n_nonexec), float(alpha0), float(gamma), _ptr(coef), n_nonexec.numel(), _stream(stream)))


def skipkv_profile_create() -> int:
    out = C.c_void_p(0)
    _check(lib().skipkv_profile_create(C.byref(out)))
    return int(out.value)


def skipkv_profile_read(profile: int) -> "list[tuple[str, float]]":
    n = C.c_int32(0)
    names = (C.c_char_p * PROFILE_SLOTS)()
    ms = (C.c_float * PROFILE_SLOTS)()
    _check(lib().skipkv_profile_read(profile, C.byref(n), names, ms))
    return [(names[i].decode(), float(ms[i])) for i in range(n.value)]


def skipkv_profile_destroy(profile: int) -> None:
    _check(lib().skipkv_profile_destroy(profile))
