"""Thin ctypes binding of the C-ABI library declared in include/tt_emb.h.

Argument marshalling only: every step of the path runs in the HIP kernels of
``libtt_emb.so``.  PyTorch supplies device memory (tensors) and the current HIP
stream; nothing here computes.  There is no CPU fallback: if the library has not
been built (``python -c "import __graft_entry__ as g; g.build()"``) loading
raises.
"""

from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtt_emb.so")

TT_OK = 0
ERR_NAMES = {0: "TT_OK", -1: "TT_ERR_NULL", -2: "TT_ERR_BAD_SHAPE", -3: "TT_ERR_BAD_ARG",
             -4: "TT_ERR_WORKSPACE", -5: "TT_ERR_HIP", -6: "TT_ERR_UNSUPPORTED"}

EXPORTS = ("tt_last_error", "tt_cache_table_capacity", "tt_emb_workspace_bytes",
           "tt_cache_build_workspace_bytes", "tt_emb_dedup_workspace_bytes",
           "tt_emb_bwd_sgd_workspace_bytes", "tt_cache_refill_workspace_bytes", "tt_cache_refill",
           "tt_emb_mean_weights", "tt_init_sampled_gaussian", "tt_embd_fwd", "tt_embd_bwd", "tt_embd_sgd_update", "tt_freq_reset", "tt_freq_update", "tt_freq_export", "tt_dense_bag_fwd", "tt_dense_bag_bwd_sgd", "tt_dense_bag_bwd_sgd_merged", "tt_dense_bag_bwd_workspace_bytes",
           "tt_emb_validate", "tt_emb_debug_launch_probe", "tt_emb_kept_bytes", "tt_emb_kept_has_lists", "tt_emb_kept_prepare", "tt_emb_fwd_keep", "tt_emb_bwd_kept", "tt_emb_bwd_sgd_kept", "tt_emb_debug_kept_lists", "tt_emb_bwd_sgd_static", "tt_emb_static_scratch_bytes", "tt_emb_fwd_keep_t0", "tt_emb_bwd_t0", "tt_emb_bwd_sgd_t0", "tt_emb_bwd_prepare", "tt_emb_fwd_prepared", "tt_emb_fwd_uses_lists", "tt_emb_bwd_sgd_prepared", "tt_emb_bwd_has_prepass", "tt_emb_bwd_two_calls_group_earlier",
           "tt_emb_fwd", "tt_emb_bwd", "tt_emb_bwd_sgd", "tt_emb_sgd_update", "tt_cache_build", "tt_cache_lookup",
           "tt_emb_debug_decode", "tt_emb_debug_decode_as", "tt_emb_debug_dedup", "tt_emb_debug_set_fast_path")


class TTShape(C.Structure):
    _fields_ = [("d", C.c_int32), ("num_rows", C.c_int64),
                ("m", C.c_int32 * 3), ("n", C.c_int32 * 3), ("r", C.c_int32 * 4)]


class TTCache(C.Structure):
    _fields_ = [("K", C.c_int64), ("capacity", C.c_int64),
                ("rows", C.c_void_p), ("keys", C.c_void_p), ("table", C.c_void_p)]


class TTError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__("%s (%d): %s" % (ERR_NAMES.get(code, "?"), code, text))
        self.code = code


_lib = None


def lib():
    """The loaded library.  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("HIP library %s is missing: run __graft_entry__.build() first" % LIB_PATH)
        l = C.CDLL(LIB_PATH)
        l.tt_last_error.restype = C.c_char_p
        l.tt_cache_table_capacity.restype = C.c_int64
        l.tt_cache_table_capacity.argtypes = [C.c_int64]
        for name in ("tt_emb_workspace_bytes", "tt_cache_build_workspace_bytes", "tt_emb_dedup_workspace_bytes",
                     "tt_emb_bwd_sgd_workspace_bytes", "tt_cache_refill_workspace_bytes"):
            getattr(l, name).restype = C.c_size_t
        l.tt_emb_workspace_bytes.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_int64]
        l.tt_emb_bwd_sgd_workspace_bytes.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_int64]
        l.tt_cache_build_workspace_bytes.argtypes = [C.c_void_p, C.c_int64, C.c_int64]
        l.tt_emb_dedup_workspace_bytes.argtypes = [C.c_int64]
        vp, i64, f32 = C.c_void_p, C.c_int64, C.c_float
        l.tt_emb_fwd.argtypes = [vp, vp, vp, i64, vp, i64, vp, vp, vp, vp, C.c_size_t, vp]
        l.tt_emb_bwd.argtypes = [vp, vp, vp, i64, vp, i64, vp, vp, vp, vp, vp, vp, C.c_size_t, vp]
        l.tt_emb_fwd_keep_t0.argtypes = [vp, vp, vp, i64, vp, i64, vp, vp, vp, vp, vp]
        l.tt_emb_bwd_t0.argtypes = [vp, vp, vp, i64, vp, i64, vp, vp, vp, vp, vp, vp, vp, C.c_size_t, vp]
        l.tt_emb_bwd_sgd_t0.argtypes = [vp, vp, vp, vp, i64, vp, i64, vp, vp, vp, vp, f32, vp, C.c_size_t, vp]
        l.tt_emb_bwd_sgd.argtypes = [vp, vp, vp, vp, i64, vp, i64, vp, vp, vp, f32, vp, C.c_size_t, vp]
        l.tt_emb_bwd_sgd_static.argtypes = [vp, vp, vp, vp, i64, vp, i64, vp, vp, vp, f32, vp]
        l.tt_emb_static_scratch_bytes.restype = C.c_size_t
        l.tt_emb_static_scratch_bytes.argtypes = []
        l.tt_emb_kept_bytes.restype = C.c_size_t
        l.tt_emb_validate.argtypes = [vp, vp, i64, vp, i64, vp, vp]
        l.tt_emb_debug_launch_probe.argtypes = [C.c_int32, vp, vp]
        l.tt_emb_kept_bytes.argtypes = [vp, i64]
        l.tt_emb_kept_has_lists.argtypes = [vp, i64]
        l.tt_emb_fwd_keep.argtypes = [vp, vp, vp, i64, vp, i64, vp, vp, vp, vp, C.c_size_t, C.c_int, vp]
        l.tt_emb_kept_prepare.argtypes = [vp, vp, i64, vp, vp, C.c_size_t, vp]
        l.tt_emb_bwd_kept.argtypes = [vp, vp, vp, i64, vp, i64, vp, vp, vp, vp, C.c_size_t, vp, vp, vp, vp, C.c_size_t, vp]
        l.tt_emb_bwd_sgd_kept.argtypes = [vp, vp, vp, vp, i64, vp, i64, vp, vp, vp, vp, C.c_size_t, f32, vp, vp, C.c_size_t, vp]
        l.tt_emb_debug_kept_lists.argtypes = [vp, vp, C.c_size_t, i64, vp, vp, vp, vp]
        l.tt_emb_bwd_prepare.argtypes = [vp, vp, i64, vp, i64, vp, C.c_int, vp, C.c_size_t, vp]
        l.tt_emb_fwd_uses_lists.argtypes = [vp, i64, i64, C.c_int]
        l.tt_emb_fwd_prepared.argtypes = [vp, vp, vp, i64, vp, i64, vp, vp, vp, vp, vp, C.c_size_t, vp]
        l.tt_emb_bwd_has_prepass.argtypes = [vp, i64, i64, C.c_int]
        l.tt_emb_bwd_two_calls_group_earlier.argtypes = [vp, i64, i64, C.c_int]
        l.tt_emb_bwd_sgd_prepared.argtypes = [vp, vp, vp, vp, i64, vp, i64, vp, vp, vp, vp, f32, vp, C.c_size_t, vp]
        l.tt_emb_sgd_update.argtypes = [vp, vp, vp, f32, vp, vp, C.c_int, vp]
        l.tt_cache_build.argtypes = [vp, vp, vp, vp, i64, vp, vp, C.c_size_t, vp]
        l.tt_cache_lookup.argtypes = [vp, vp, i64, vp, vp]
        l.tt_cache_refill.argtypes = [vp, vp, vp, vp, i64, vp, vp, C.c_size_t, vp]
        l.tt_cache_refill_workspace_bytes.argtypes = [vp, i64, i64]
        l.tt_dense_bag_fwd.argtypes = [vp, i64, C.c_int32, vp, i64, vp, i64, vp, vp, vp]
        l.tt_dense_bag_bwd_sgd.argtypes = [vp, i64, C.c_int32, vp, i64, vp, i64, vp, vp, f32, vp]
        l.tt_dense_bag_bwd_sgd_merged.argtypes = [vp, i64, C.c_int32, vp, i64, vp, i64, vp, vp, f32, vp, C.c_size_t, vp]
        l.tt_dense_bag_bwd_workspace_bytes.argtypes = [i64, C.c_int32]
        l.tt_dense_bag_bwd_workspace_bytes.restype = C.c_size_t
        l.tt_embd_fwd.argtypes = [vp, vp, vp, i64, vp, i64, vp, vp, vp]
        l.tt_embd_bwd.argtypes = [vp, vp, vp, i64, vp, i64, vp, vp, vp, vp]
        l.tt_embd_sgd_update.argtypes = [vp, vp, vp, f32, C.c_int, vp]
        l.tt_init_sampled_gaussian.argtypes = [vp, vp, C.c_uint64, vp]
        l.tt_emb_mean_weights.argtypes = [vp, i64, i64, vp, vp, vp]
        l.tt_freq_reset.argtypes = [vp, vp]
        l.tt_freq_update.argtypes = [vp, vp, i64, vp]
        l.tt_freq_export.argtypes = [vp, vp, vp, vp, vp]
        l.tt_emb_debug_decode.argtypes = [vp, vp, i64, vp, vp, vp, vp]
        l.tt_emb_debug_decode_as.argtypes = [vp, vp, i64, C.c_int, vp, vp, vp, vp]
        l.tt_emb_debug_dedup.argtypes = [vp, vp, i64, vp, C.c_int, vp, vp, vp, vp, vp, C.c_size_t, vp]
        l.tt_emb_debug_set_fast_path.argtypes = [C.c_int]
        _lib = l
    return _lib


def _check(rc: int):
    if rc != TT_OK:
        raise TTError(rc, lib().tt_last_error().decode())


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t: torch.Tensor, dtype) -> torch.Tensor:
    assert t.is_cuda and t.dtype == dtype and t.is_contiguous(), (t.device, t.dtype, t.is_contiguous())
    return t


def make_shape(num_rows: int, m: Sequence[int], n: Sequence[int], r: Sequence[int]) -> TTShape:
    s = TTShape()
    s.d = 3
    s.num_rows = int(num_rows)
    for k in range(3):
        s.m[k] = int(m[k])
        s.n[k] = int(n[k])
    for k in range(4):
        s.r[k] = int(r[k])
    return s


def shape_of(t) -> TTShape:
    """TTShape from any object with num_rows, m, n, r attributes."""
    return make_shape(t.num_rows, t.m, t.n, t.r)


def _ptr_array(ts: Sequence[torch.Tensor]):
    arr = (C.c_void_p * 3)()
    for k in range(3):
        arr[k] = _dev(ts[k], torch.float32).data_ptr()
    return arr


class Cache:
    """Device arrays of a cache plus the host struct that points at them."""

    def __init__(self, K: int, dim: int, device="cuda"):
        self.K = int(K)
        self.capacity = int(lib().tt_cache_table_capacity(self.K))
        self.rows = torch.zeros((max(self.K, 1), dim), dtype=torch.float32, device=device)
        self.keys = torch.zeros(max(self.K, 1), dtype=torch.int64, device=device)
        self.table = torch.zeros(self.capacity, dtype=torch.int64, device=device)
        self.c = TTCache(self.K, self.capacity, self.rows.data_ptr(), self.keys.data_ptr(), self.table.data_ptr())

    def ref(self):
        return C.byref(self.c)


def workspace_bytes(shape: TTShape, L: int, n_bags: int, cache_rows: int = 0) -> int:
    return int(lib().tt_emb_workspace_bytes(C.byref(shape), L, n_bags, int(cache_rows)))


def bwd_sgd_workspace_bytes(shape: TTShape, L: int, n_bags: int, cache_rows: int = 0) -> int:
    return int(lib().tt_emb_bwd_sgd_workspace_bytes(C.byref(shape), L, n_bags, int(cache_rows)))


def _ws(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def tt_emb_fwd(shape: TTShape, cores: Sequence[torch.Tensor], indices: torch.Tensor,
               offsets: Optional[torch.Tensor], n_bags: int, output: torch.Tensor,
               alpha: Optional[torch.Tensor] = None, cache: Optional[Cache] = None,
               workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    _dev(indices, torch.int64)
    if offsets is not None:
        _dev(offsets, torch.int64)
        assert offsets.numel() == n_bags + 1
    if alpha is not None:
        _dev(alpha, torch.float32)
    _dev(output, torch.float32)
    assert output.numel() == n_bags * shape.n[0] * shape.n[1] * shape.n[2]
    wsb = workspace.numel() if workspace is not None else 0
    _check(lib().tt_emb_fwd(C.byref(shape), _ptr_array(cores), _ptr(indices), indices.numel(), _ptr(offsets), n_bags,
                            _ptr(alpha), cache.ref() if cache else None, _ptr(output), _ptr(workspace), wsb, _stream()))
    return output


TT_BAD_INDEX, TT_BAD_OFFSETS_ORDER, TT_BAD_OFFSETS_RANGE = 1, 2, 4


def tt_emb_validate(shape: TTShape, indices: torch.Tensor, offsets: Optional[torch.Tensor], n_bags: int,
                    flag: torch.Tensor) -> torch.Tensor:
    """flag: int32 [1] on the device; 0 afterwards if the arguments are valid, else TT_BAD_* bits."""
    _dev(indices, torch.int64)
    _dev(flag, torch.int32)
    if offsets is not None:
        _dev(offsets, torch.int64)
        assert offsets.numel() == n_bags + 1
    _check(lib().tt_emb_validate(C.byref(shape), _ptr(indices), indices.numel(), _ptr(offsets), n_bags, _ptr(flag), _stream()))
    return flag


def tt_emb_debug_launch_probe(blocks: int, sink: Optional[torch.Tensor] = None) -> None:
    _check(lib().tt_emb_debug_launch_probe(int(blocks), _ptr(sink), _stream()))


def t0_floats(shape: TTShape) -> int:
    """fp32 values per position of the stored intermediate (n1 n2 r2)."""
    return shape.n[0] * shape.n[1] * shape.r[2]


def tt_emb_fwd_keep_t0(shape: TTShape, cores: Sequence[torch.Tensor], indices: torch.Tensor,
                       offsets: Optional[torch.Tensor], n_bags: int, output: torch.Tensor, t0: torch.Tensor,
                       alpha: Optional[torch.Tensor] = None, cache: Optional[Cache] = None) -> torch.Tensor:
    _dev(indices, torch.int64)
    if offsets is not None:
        _dev(offsets, torch.int64)
        assert offsets.numel() == n_bags + 1
    if alpha is not None:
        _dev(alpha, torch.float32)
    _dev(output, torch.float32)
    _dev(t0, torch.float32)
    assert t0.numel() >= indices.numel() * t0_floats(shape)
    _check(lib().tt_emb_fwd_keep_t0(C.byref(shape), _ptr_array(cores), _ptr(indices), indices.numel(), _ptr(offsets),
                                    n_bags, _ptr(alpha), cache.ref() if cache else None, _ptr(output), _ptr(t0), _stream()))
    return output


def fwd_uses_lists(shape: TTShape, L: int, cache_rows: int = 0, kept_t0: bool = False) -> bool:
    return bool(lib().tt_emb_fwd_uses_lists(C.byref(shape), int(L), int(cache_rows), int(kept_t0)))


def tt_emb_fwd_prepared(shape: TTShape, cores: Sequence[torch.Tensor], indices: torch.Tensor,
                        offsets: Optional[torch.Tensor], n_bags: int, output: torch.Tensor, workspace: torch.Tensor,
                        t0: Optional[torch.Tensor] = None, alpha: Optional[torch.Tensor] = None,
                        cache: Optional[Cache] = None) -> torch.Tensor:
    """The forward pass after tt_emb_bwd_prepare into the same workspace (t0: keep the intermediate there)."""
    _dev(indices, torch.int64)
    if offsets is not None:
        _dev(offsets, torch.int64)
        assert offsets.numel() == n_bags + 1
    if alpha is not None:
        _dev(alpha, torch.float32)
    _dev(output, torch.float32)
    _dev(workspace, torch.uint8)
    if t0 is not None:
        _dev(t0, torch.float32)
        assert t0.numel() >= indices.numel() * t0_floats(shape)
    assert output.numel() == n_bags * shape.n[0] * shape.n[1] * shape.n[2]
    _check(lib().tt_emb_fwd_prepared(C.byref(shape), _ptr_array(cores), _ptr(indices), indices.numel(), _ptr(offsets),
                                     n_bags, _ptr(alpha), cache.ref() if cache else None, _ptr(output), _ptr(t0),
                                     _ptr(workspace), workspace.numel(), _stream()))
    return output


def tt_emb_bwd(shape: TTShape, cores: Sequence[torch.Tensor], indices: torch.Tensor,
               offsets: Optional[torch.Tensor], n_bags: int, grad_output: torch.Tensor,
               grad_cores: Sequence[torch.Tensor], alpha: Optional[torch.Tensor] = None,
               cache: Optional[Cache] = None, grad_cache: Optional[torch.Tensor] = None,
               workspace: Optional[torch.Tensor] = None, t0: Optional[torch.Tensor] = None) -> None:
    _dev(indices, torch.int64)
    if offsets is not None:
        _dev(offsets, torch.int64)
        assert offsets.numel() == n_bags + 1
    if alpha is not None:
        _dev(alpha, torch.float32)
    _dev(grad_output, torch.float32)
    for k in range(3):
        assert grad_cores[k].numel() == cores[k].numel()
    if grad_cache is not None:
        _dev(grad_cache, torch.float32)
    wsb = workspace.numel() if workspace is not None else 0
    if t0 is not None:
        _dev(t0, torch.float32)
        _check(lib().tt_emb_bwd_t0(C.byref(shape), _ptr_array(cores), _ptr(indices), indices.numel(), _ptr(offsets),
                                   n_bags, _ptr(alpha), cache.ref() if cache else None, _ptr(grad_output), _ptr(t0),
                                   _ptr_array(grad_cores), _ptr(grad_cache), _ptr(workspace), wsb, _stream()))
        return
    _check(lib().tt_emb_bwd(C.byref(shape), _ptr_array(cores), _ptr(indices), indices.numel(), _ptr(offsets), n_bags,
                            _ptr(alpha), cache.ref() if cache else None, _ptr(grad_output), _ptr_array(grad_cores),
                            _ptr(grad_cache), _ptr(workspace), wsb, _stream()))


def bwd_has_prepass(shape: TTShape, L: int, cache_rows: int = 0, kept_t0: bool = False) -> bool:
    return bool(lib().tt_emb_bwd_has_prepass(C.byref(shape), L, cache_rows, int(kept_t0)))


def bwd_two_calls_group_earlier(shape: TTShape, L: int, cache_rows: int = 0, kept_t0: bool = False) -> bool:
    return bool(lib().tt_emb_bwd_two_calls_group_earlier(C.byref(shape), L, cache_rows, int(kept_t0)))


def tt_emb_bwd_prepare(shape: TTShape, indices: torch.Tensor, offsets: Optional[torch.Tensor], n_bags: int,
                       cache: Optional[Cache] = None, workspace: Optional[torch.Tensor] = None,
                       kept_t0: bool = False) -> None:
    """The index-only part of the fused step, on the current stream; tt_emb_bwd_sgd(..., prepared=True) does the rest."""
    _dev(indices, torch.int64)
    wsb = workspace.numel() if workspace is not None else 0
    _check(lib().tt_emb_bwd_prepare(C.byref(shape), _ptr(indices), indices.numel(), _ptr(offsets), n_bags,
                                    cache.ref() if cache else None, int(kept_t0), _ptr(workspace), wsb, _stream()))


def kept_bytes(shape: TTShape, L: int) -> int:
    return int(lib().tt_emb_kept_bytes(C.byref(shape), int(L)))


def kept_has_lists(shape: TTShape, L: int) -> bool:
    return bool(lib().tt_emb_kept_has_lists(C.byref(shape), int(L)))


class TTNextBatch(C.Structure):
    _fields_ = [("indices", C.c_void_p), ("L", C.c_int64), ("kept", C.c_void_p), ("kept_bytes", C.c_size_t)]


def _next(next_batch):
    """next_batch: None or (indices, kept) of the batch whose lists the call files as well."""
    if next_batch is None:
        return None
    indices, kept = next_batch
    _dev(indices, torch.int64)
    _dev(kept, torch.uint8)
    return C.byref(TTNextBatch(indices.data_ptr(), indices.numel(), kept.data_ptr(), kept.numel()))


def tt_emb_kept_prepare(shape: TTShape, indices: torch.Tensor, kept: torch.Tensor, cache: Optional["Cache"] = None) -> None:
    _dev(indices, torch.int64)
    _dev(kept, torch.uint8)
    _check(lib().tt_emb_kept_prepare(C.byref(shape), _ptr(indices), indices.numel(), cache.ref() if cache else None,
                                     _ptr(kept), kept.numel(), _stream()))


def tt_emb_fwd_keep(shape: TTShape, cores: Sequence[torch.Tensor], indices: torch.Tensor, offsets: Optional[torch.Tensor],
                    n_bags: int, output: torch.Tensor, kept: torch.Tensor, alpha: Optional[torch.Tensor] = None,
                    cache: Optional["Cache"] = None, lists_ready: bool = False) -> None:
    _dev(indices, torch.int64)
    if offsets is not None:
        _dev(offsets, torch.int64)
        assert offsets.numel() == n_bags + 1
    if alpha is not None:
        _dev(alpha, torch.float32)
    _dev(output, torch.float32)
    _dev(kept, torch.uint8)
    _check(lib().tt_emb_fwd_keep(C.byref(shape), _ptr_array(cores), _ptr(indices), indices.numel(), _ptr(offsets), n_bags,
                                 _ptr(alpha), cache.ref() if cache else None, _ptr(output), _ptr(kept), kept.numel(),
                                 1 if lists_ready else 0, _stream()))


def tt_emb_bwd_kept(shape: TTShape, cores: Sequence[torch.Tensor], indices: torch.Tensor, offsets: Optional[torch.Tensor],
                    n_bags: int, grad_output: torch.Tensor, kept: torch.Tensor, grad_cores: Sequence[torch.Tensor],
                    alpha: Optional[torch.Tensor] = None, cache: Optional["Cache"] = None,
                    grad_cache: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                    next_batch=None) -> None:
    _dev(indices, torch.int64)
    _dev(grad_output, torch.float32)
    _dev(kept, torch.uint8)
    wsb = workspace.numel() if workspace is not None else 0
    _check(lib().tt_emb_bwd_kept(C.byref(shape), _ptr_array(cores), _ptr(indices), indices.numel(), _ptr(offsets), n_bags,
                                 _ptr(alpha), cache.ref() if cache else None, _ptr(grad_output), _ptr(kept), kept.numel(),
                                 _ptr_array(grad_cores), _ptr(grad_cache), _next(next_batch), _ptr(workspace), wsb, _stream()))


def tt_emb_bwd_sgd_kept(shape: TTShape, cores: Sequence[torch.Tensor], cores_out: Sequence[torch.Tensor],
                        indices: torch.Tensor, offsets: Optional[torch.Tensor], n_bags: int, grad_output: torch.Tensor,
                        kept: torch.Tensor, lr: float, alpha: Optional[torch.Tensor] = None, cache: Optional["Cache"] = None,
                        workspace: Optional[torch.Tensor] = None, next_batch=None) -> None:
    _dev(indices, torch.int64)
    _dev(grad_output, torch.float32)
    _dev(kept, torch.uint8)
    for k in range(3):
        assert cores_out[k].numel() == cores[k].numel()
    wsb = workspace.numel() if workspace is not None else 0
    _check(lib().tt_emb_bwd_sgd_kept(C.byref(shape), _ptr_array(cores), _ptr_array(cores_out), _ptr(indices), indices.numel(),
                                     _ptr(offsets), n_bags, _ptr(alpha), cache.ref() if cache else None, _ptr(grad_output),
                                     _ptr(kept), kept.numel(), C.c_float(lr), _next(next_batch), _ptr(workspace), wsb,
                                     _stream()))


def tt_emb_debug_kept_lists(shape: TTShape, kept: torch.Tensor, L: int):
    """(slice, rep, times), each int32 [3][L]."""
    out = [torch.empty((3, L), dtype=torch.int32, device=kept.device) for _ in range(3)]
    _check(lib().tt_emb_debug_kept_lists(C.byref(shape), _ptr(kept), kept.numel(), int(L), _ptr(out[0]), _ptr(out[1]),
                                         _ptr(out[2]), _stream()))
    return out


def tt_emb_bwd_sgd_static(shape: TTShape, cores: Sequence[torch.Tensor], cores_out: Sequence[torch.Tensor],
                          indices: torch.Tensor, offsets: Optional[torch.Tensor], n_bags: int, grad_output: torch.Tensor,
                          lr: float, alpha: Optional[torch.Tensor] = None, cache: Optional[Cache] = None) -> None:
    """tt_emb_bwd_sgd with the library's own static scratch array instead of a workspace (allocates nothing)."""
    _dev(indices, torch.int64)
    if offsets is not None:
        _dev(offsets, torch.int64)
        assert offsets.numel() == n_bags + 1
    if alpha is not None:
        _dev(alpha, torch.float32)
    _dev(grad_output, torch.float32)
    for k in range(3):
        assert cores_out[k].numel() == cores[k].numel()
    _check(lib().tt_emb_bwd_sgd_static(C.byref(shape), _ptr_array(cores), _ptr_array(cores_out), _ptr(indices),
                                       indices.numel(), _ptr(offsets), n_bags, _ptr(alpha),
                                       cache.ref() if cache else None, _ptr(grad_output), C.c_float(lr), _stream()))


def static_scratch_bytes() -> int:
    return int(lib().tt_emb_static_scratch_bytes())


def tt_emb_bwd_sgd(shape: TTShape, cores: Sequence[torch.Tensor], cores_out: Sequence[torch.Tensor],
                   indices: torch.Tensor, offsets: Optional[torch.Tensor], n_bags: int, grad_output: torch.Tensor,
                   lr: float, alpha: Optional[torch.Tensor] = None, cache: Optional[Cache] = None,
                   workspace: Optional[torch.Tensor] = None, t0: Optional[torch.Tensor] = None,
                   prepared: bool = False) -> None:
    _dev(indices, torch.int64)
    if offsets is not None:
        _dev(offsets, torch.int64)
        assert offsets.numel() == n_bags + 1
    if alpha is not None:
        _dev(alpha, torch.float32)
    _dev(grad_output, torch.float32)
    for k in range(3):
        assert cores_out[k].numel() == cores[k].numel()
    wsb = workspace.numel() if workspace is not None else 0
    if prepared:
        if t0 is not None:
            _dev(t0, torch.float32)
        _check(lib().tt_emb_bwd_sgd_prepared(C.byref(shape), _ptr_array(cores), _ptr_array(cores_out), _ptr(indices),
                                             indices.numel(), _ptr(offsets), n_bags, _ptr(alpha),
                                             cache.ref() if cache else None, _ptr(grad_output), _ptr(t0), C.c_float(lr),
                                             _ptr(workspace), wsb, _stream()))
        return
    if t0 is not None:
        _dev(t0, torch.float32)
        _check(lib().tt_emb_bwd_sgd_t0(C.byref(shape), _ptr_array(cores), _ptr_array(cores_out), _ptr(indices),
                                       indices.numel(), _ptr(offsets), n_bags, _ptr(alpha),
                                       cache.ref() if cache else None, _ptr(grad_output), _ptr(t0), C.c_float(lr),
                                       _ptr(workspace), wsb, _stream()))
        return
    _check(lib().tt_emb_bwd_sgd(C.byref(shape), _ptr_array(cores), _ptr_array(cores_out), _ptr(indices), indices.numel(),
                                _ptr(offsets), n_bags, _ptr(alpha), cache.ref() if cache else None, _ptr(grad_output),
                                C.c_float(lr), _ptr(workspace), wsb, _stream()))


def tt_emb_sgd_update(shape: TTShape, cores: Sequence[torch.Tensor], grad_cores: Sequence[torch.Tensor], lr: float,
                      cache: Optional[Cache] = None, grad_cache: Optional[torch.Tensor] = None,
                      zero_grad: bool = False) -> None:
    _check(lib().tt_emb_sgd_update(C.byref(shape), _ptr_array(cores), _ptr_array(grad_cores), C.c_float(lr),
                                   cache.ref() if cache else None, _ptr(grad_cache), int(zero_grad), _stream()))


def tt_cache_build(shape: TTShape, cores: Sequence[torch.Tensor], cand_rows: torch.Tensor,
                   cand_counts: torch.Tensor, cache: Cache, workspace: Optional[torch.Tensor] = None) -> Cache:
    _dev(cand_rows, torch.int64)
    _dev(cand_counts, torch.int64)
    n = cand_rows.numel()
    assert cand_counts.numel() == n
    if workspace is None:
        workspace = _ws(lib().tt_cache_build_workspace_bytes(C.byref(shape), n, cache.K), cand_rows.device)
    _check(lib().tt_cache_build(C.byref(shape), _ptr_array(cores), _ptr(cand_rows), _ptr(cand_counts), n, cache.ref(),
                                _ptr(workspace), workspace.numel(), _stream()))
    return cache


def tt_cache_refill(shape: TTShape, cores: Sequence[torch.Tensor], cand_rows: torch.Tensor,
                    cand_counts: torch.Tensor, cache: Cache, workspace: Optional[torch.Tensor] = None) -> Cache:
    _dev(cand_rows, torch.int64)
    _dev(cand_counts, torch.int64)
    n = cand_rows.numel()
    assert cand_counts.numel() == n
    if workspace is None:
        workspace = _ws(lib().tt_cache_refill_workspace_bytes(C.byref(shape), n, cache.K), cand_rows.device)
    _check(lib().tt_cache_refill(C.byref(shape), _ptr_array(cores), _ptr(cand_rows), _ptr(cand_counts), n, cache.ref(),
                                 _ptr(workspace), workspace.numel(), _stream()))
    return cache


class TTFreq(C.Structure):
    _fields_ = [("capacity", C.c_int64), ("table", C.c_void_p), ("stats", C.c_void_p)]


class Freq:
    """Device arrays of an access-frequency tracker and the host struct that points at them."""

    def __init__(self, capacity: int, device):
        assert capacity >= 64 and capacity & (capacity - 1) == 0
        self.capacity = capacity
        self.table = torch.empty(capacity, dtype=torch.int64, device=device)
        self.stats = torch.zeros(2, dtype=torch.int64, device=device)
        self._c = TTFreq(capacity, self.table.data_ptr(), self.stats.data_ptr())

    def ref(self):
        return C.byref(self._c)


def tt_freq_reset(freq: Freq) -> None:
    _check(lib().tt_freq_reset(freq.ref(), _stream()))


def tt_freq_update(freq: Freq, indices: torch.Tensor) -> None:
    _dev(indices, torch.int64)
    _check(lib().tt_freq_update(freq.ref(), _ptr(indices), indices.numel(), _stream()))


def tt_freq_export(freq: Freq, rows: torch.Tensor, counts: torch.Tensor, n_out: torch.Tensor) -> None:
    _dev(rows, torch.int64)
    _dev(counts, torch.int64)
    _dev(n_out, torch.int64)
    assert rows.numel() >= freq.capacity and counts.numel() >= freq.capacity
    _check(lib().tt_freq_export(freq.ref(), _ptr(rows), _ptr(counts), _ptr(n_out), _stream()))


def tt_cache_lookup(cache: Cache, indices: torch.Tensor, slot: torch.Tensor) -> torch.Tensor:
    _dev(indices, torch.int64)
    _dev(slot, torch.int32)
    assert slot.numel() == indices.numel()
    _check(lib().tt_cache_lookup(cache.ref(), _ptr(indices), indices.numel(), _ptr(slot), _stream()))
    return slot


def tt_emb_debug_decode(shape: TTShape, indices: torch.Tensor) -> List[torch.Tensor]:
    _dev(indices, torch.int64)
    out = [torch.empty(indices.numel(), dtype=torch.int32, device=indices.device) for _ in range(3)]
    _check(lib().tt_emb_debug_decode(C.byref(shape), _ptr(indices), indices.numel(), _ptr(out[0]), _ptr(out[1]),
                                     _ptr(out[2]), _stream()))
    return out


def tt_emb_debug_decode_as(shape: TTShape, indices: torch.Tensor, mode: int) -> List[torch.Tensor]:
    _dev(indices, torch.int64)
    out = [torch.empty(indices.numel(), dtype=torch.int32, device=indices.device) for _ in range(3)]
    _check(lib().tt_emb_debug_decode_as(C.byref(shape), _ptr(indices), indices.numel(), int(mode), _ptr(out[0]),
                                        _ptr(out[1]), _ptr(out[2]), _stream()))
    return out


def tt_emb_debug_dedup(shape: TTShape, indices: torch.Tensor, which: int, slot: Optional[torch.Tensor] = None):
    """Returns (uniq, count, perm) trimmed to their valid lengths (this trims on the host)."""
    _dev(indices, torch.int64)
    L = indices.numel()
    dev = indices.device
    uniq = torch.empty(max(L, 1), dtype=torch.int64, device=dev)
    count = torch.empty(max(L, 1), dtype=torch.int32, device=dev)
    perm = torch.empty(max(L, 1), dtype=torch.int32, device=dev)
    n_out = torch.zeros(2, dtype=torch.int64, device=dev)
    ws = _ws(lib().tt_emb_dedup_workspace_bytes(L), dev)
    _check(lib().tt_emb_debug_dedup(C.byref(shape), _ptr(indices), L, _ptr(slot), int(which), _ptr(uniq), _ptr(count),
                                    _ptr(perm), _ptr(n_out), _ptr(ws), ws.numel(), _stream()))
    nu, kept = (int(x) for x in n_out.cpu())
    return uniq[:nu], count[:nu], perm[:kept]


def set_fast_path(mode: int) -> int:
    """0: generic kernels, 1: specialised (default), 2: specialised + grouping pre-pass always + list owners always,
    3: as 2 but the grouped backward with a kept T0 on tiles of positions, also with a cache.  Per thread; returns the old value."""
    return int(lib().tt_emb_debug_set_fast_path(int(mode)))


def tt_dense_bag_fwd(table: torch.Tensor, indices: torch.Tensor, offsets: Optional[torch.Tensor], n_bags: int,
                     output: torch.Tensor, alpha: Optional[torch.Tensor] = None) -> torch.Tensor:
    _dev(table, torch.float32)
    _dev(indices, torch.int64)
    _dev(output, torch.float32)
    _check(lib().tt_dense_bag_fwd(_ptr(table), table.shape[0], table.shape[1], _ptr(indices), indices.numel(),
                                  _ptr(offsets), n_bags, _ptr(alpha), _ptr(output), _stream()))
    return output


def tt_dense_bag_bwd_sgd(table: torch.Tensor, indices: torch.Tensor, offsets: Optional[torch.Tensor], n_bags: int,
                         grad_output: torch.Tensor, lr: float, alpha: Optional[torch.Tensor] = None) -> None:
    _dev(table, torch.float32)
    _dev(indices, torch.int64)
    _dev(grad_output, torch.float32)
    _check(lib().tt_dense_bag_bwd_sgd(_ptr(table), table.shape[0], table.shape[1], _ptr(indices), indices.numel(),
                                      _ptr(offsets), n_bags, _ptr(alpha), _ptr(grad_output), C.c_float(lr), _stream()))


def dense_bwd_workspace_bytes(L: int, N: int) -> int:
    return int(lib().tt_dense_bag_bwd_workspace_bytes(int(L), int(N)))


def tt_dense_bag_bwd_sgd_merged(table: torch.Tensor, indices: torch.Tensor, offsets: Optional[torch.Tensor], n_bags: int,
                                grad_output: torch.Tensor, lr: float, alpha: Optional[torch.Tensor] = None,
                                workspace: Optional[torch.Tensor] = None) -> None:
    _dev(table, torch.float32)
    _dev(indices, torch.int64)
    _dev(grad_output, torch.float32)
    if workspace is None:
        workspace = torch.empty(max(dense_bwd_workspace_bytes(indices.numel(), table.shape[1]), 256), dtype=torch.uint8,
                                device=table.device)
    _check(lib().tt_dense_bag_bwd_sgd_merged(_ptr(table), table.shape[0], table.shape[1], _ptr(indices), indices.numel(),
                                             _ptr(offsets), n_bags, _ptr(alpha), _ptr(grad_output), C.c_float(lr),
                                             _ptr(workspace), workspace.numel(), _stream()))


def tt_emb_mean_weights(offsets: torch.Tensor, n_bags: int, L: int, weights: torch.Tensor,
                        alpha: Optional[torch.Tensor] = None) -> torch.Tensor:
    _dev(offsets, torch.int64)
    _dev(weights, torch.float32)
    assert offsets.numel() == n_bags + 1 and weights.numel() >= L
    if alpha is not None:
        _dev(alpha, torch.float32)
    _check(lib().tt_emb_mean_weights(_ptr(offsets), n_bags, L, _ptr(alpha), _ptr(weights), _stream()))
    return weights


def tt_init_sampled_gaussian(shape: TTShape, cores: Sequence[torch.Tensor], seed: int) -> None:
    _check(lib().tt_init_sampled_gaussian(C.byref(shape), _ptr_array(cores), C.c_uint64(seed), _stream()))


class TTShapeD(C.Structure):
    _fields_ = [("d", C.c_int32), ("num_rows", C.c_int64), ("m", C.c_int32 * 4), ("n", C.c_int32 * 4), ("r", C.c_int32 * 5)]


def make_shape_d(num_rows: int, m: Sequence[int], n: Sequence[int], r: Sequence[int]) -> TTShapeD:
    d = len(m)
    assert len(n) == d and len(r) == d + 1
    s = TTShapeD()
    s.d, s.num_rows = d, num_rows
    for k in range(d):
        s.m[k], s.n[k] = m[k], n[k]
    for k in range(d + 1):
        s.r[k] = r[k]
    return s


def _ptr_array_d(ts: Sequence[torch.Tensor]):
    arr = (C.c_void_p * 4)()
    for k, t in enumerate(ts):
        arr[k] = _dev(t, torch.float32).data_ptr()
    return arr


def tt_embd_fwd(shape: TTShapeD, cores: Sequence[torch.Tensor], indices: torch.Tensor, offsets: Optional[torch.Tensor],
                n_bags: int, output: torch.Tensor, alpha: Optional[torch.Tensor] = None) -> torch.Tensor:
    _dev(indices, torch.int64)
    _dev(output, torch.float32)
    _check(lib().tt_embd_fwd(C.byref(shape), _ptr_array_d(cores), _ptr(indices), indices.numel(), _ptr(offsets), n_bags,
                             _ptr(alpha), _ptr(output), _stream()))
    return output


def tt_embd_bwd(shape: TTShapeD, cores: Sequence[torch.Tensor], indices: torch.Tensor, offsets: Optional[torch.Tensor],
                n_bags: int, grad_output: torch.Tensor, grad_cores: Sequence[torch.Tensor],
                alpha: Optional[torch.Tensor] = None) -> None:
    _dev(indices, torch.int64)
    _dev(grad_output, torch.float32)
    _check(lib().tt_embd_bwd(C.byref(shape), _ptr_array_d(cores), _ptr(indices), indices.numel(), _ptr(offsets), n_bags,
                             _ptr(alpha), _ptr(grad_output), _ptr_array_d(grad_cores), _stream()))


def tt_embd_sgd_update(shape: TTShapeD, cores: Sequence[torch.Tensor], grad_cores: Sequence[torch.Tensor], lr: float,
                       zero_grad: bool = False) -> None:
    _check(lib().tt_embd_sgd_update(C.byref(shape), _ptr_array_d(cores), _ptr_array_d(grad_cores), C.c_float(lr),
                                    int(zero_grad), _stream()))
