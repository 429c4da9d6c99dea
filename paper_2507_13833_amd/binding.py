"""ctypes binding of the C-ABI in include/dc.h -- argument marshalling only.

Every function has the name and argument order of its C counterpart.  Device
buffers are torch tensors (or raw integer device addresses); the stream defaults
to torch's current HIP stream.  No step of the path is computed here, and there is
no CPU fallback: if ``libdc.so`` has not been built, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdc.so")

DC_MAX_SEQ = 16384
DC_MAX_SEQ_LARGE = 1 << 20
DC_MAX_SHARDS = 1024
DC_MAX_FIELDS = 8
DC_MAX_SRC_SHARDS = 16
DC_REPACK_NOALLOC_WS_BYTES = 8 << 20

DC_OK = 0
DC_ERR_INVALID_ARG = 1
DC_ERR_NOT_DIVISIBLE = 2
DC_ERR_UNSUPPORTED_SIZE = 3
DC_ERR_WORKSPACE = 4
DC_ERR_HIP = 5
DC_ERR_SEQ_EXCEEDS_BUDGET = 6
DC_ERR_ZERO_LENGTH_SEQ = 7
DC_ERR_OVERFLOW = 8
DC_ERR_BAD_LAYOUT = 9

EXPORTS = ("dc_workspace_bytes", "dc_balance", "dc_group_advantage", "dc_plan", "dc_gather",
           "dc_repack", "dc_scatter_workspace_bytes", "dc_scatter", "dc_gae", "dc_balance_group_advantage",
           "dc_gather_advantage", "dc_balance_workspace_bytes", "dc_balance_ws", "dc_repack_noalloc", "dc_balance_plan_group_advantage", "dc_gather_timed", "dc_strerror")


class dc_params(C.Structure):
    _fields_ = [("n_seq", C.c_int32), ("n_shards", C.c_int32), ("cap", C.c_int32),
                ("align_tokens", C.c_int32), ("token_budget", C.c_int64), ("eps", C.c_double),
                ("ddof", C.c_int32), ("reserved", C.c_int32)]


class dc_source(C.Structure):
    _fields_ = [("n_src_shards", C.c_int32), ("reserved", C.c_int32),
                ("shard_seq_off", C.POINTER(C.c_int32)), ("shard_tokens", C.POINTER(C.c_int64)),
                ("d_src_tok_off", C.c_void_p)]


class dc_field(C.Structure):
    _fields_ = [("src_base", C.POINTER(C.c_void_p)), ("d_dst", C.c_void_p),
                ("elem_bytes", C.c_int32), ("reserved", C.c_int32)]


class DcError(RuntimeError):
    def __init__(self, code: int, where: str):
        super().__init__(f"{where}: {strerror(code)} (dc_status {code})")
        self.code = code


_lib = None


def load() -> C.CDLL:
    """Load libdc.so.  Raises if the HIP library has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with "
                               "`python -m paper_2507_13833_amd.build` (hipcc, gfx950); there is no fallback")
        lib = C.CDLL(LIB_PATH)
        lib.dc_workspace_bytes.restype = C.c_size_t
        lib.dc_workspace_bytes.argtypes = [C.POINTER(dc_params), C.c_int64]
        lib.dc_strerror.restype = C.c_char_p
        lib.dc_strerror.argtypes = [C.c_int]
        vp = C.c_void_p
        lib.dc_balance.restype = C.c_int
        lib.dc_balance.argtypes = [C.POINTER(dc_params), vp, vp, vp, vp, vp, vp, vp]
        lib.dc_balance_workspace_bytes.restype = C.c_size_t
        lib.dc_balance_workspace_bytes.argtypes = [C.POINTER(dc_params)]
        lib.dc_balance_ws.restype = C.c_int
        lib.dc_balance_ws.argtypes = [C.POINTER(dc_params), vp, vp, vp, vp, vp, vp, C.c_size_t, vp, vp]
        lib.dc_group_advantage.restype = C.c_int
        lib.dc_group_advantage.argtypes = [C.POINTER(dc_params), C.POINTER(dc_source), vp, vp, vp, C.c_int32,
                                           C.POINTER(vp), vp, C.POINTER(vp), vp, vp]
        lib.dc_plan.restype = C.c_int
        lib.dc_plan.argtypes = [C.POINTER(dc_params), C.POINTER(dc_source), vp, vp, vp, C.c_int64,
                                vp, vp, vp, vp, vp, vp, vp, C.c_size_t, vp, vp]
        lib.dc_gather.restype = C.c_int
        lib.dc_gather.argtypes = [C.POINTER(dc_params), C.POINTER(dc_source), C.POINTER(dc_field), C.c_int32,
                                  C.c_int64, vp, vp, C.c_size_t, vp, vp]
        lib.dc_gather_timed.restype = C.c_int
        lib.dc_gather_timed.argtypes = [C.POINTER(dc_params), C.POINTER(dc_source), C.POINTER(dc_field), C.c_int32,
                                        C.c_int64, vp, vp, C.c_size_t, vp, vp, vp, vp]
        lib.dc_gather_advantage.restype = C.c_int
        lib.dc_gather_advantage.argtypes = [C.POINTER(dc_params), C.POINTER(dc_source), C.POINTER(dc_field), C.c_int32,
                                            C.c_int32, vp, vp, vp, C.c_int64, vp, vp, C.c_size_t, vp, vp]
        lib.dc_repack.restype = C.c_int
        lib.dc_repack.argtypes = [C.POINTER(dc_params), C.POINTER(dc_source), vp, vp, vp,
                                  C.POINTER(dc_field), C.c_int32, C.c_int64,
                                  vp, vp, vp, vp, vp, vp, vp, C.c_size_t, vp, vp]
        lib.dc_repack_noalloc.restype = C.c_int
        lib.dc_repack_noalloc.argtypes = [C.POINTER(dc_params), C.POINTER(dc_source), vp, vp, vp,
                                          C.POINTER(dc_field), C.c_int32, C.c_int64,
                                          vp, vp, vp, vp, vp, vp, vp, vp]
        lib.dc_scatter_workspace_bytes.restype = C.c_size_t
        lib.dc_scatter_workspace_bytes.argtypes = [C.POINTER(dc_params), C.POINTER(dc_source)]
        lib.dc_scatter.restype = C.c_int
        lib.dc_scatter.argtypes = [C.POINTER(dc_params), C.POINTER(dc_source), vp, vp, C.POINTER(dc_field), C.c_int32,
                                   C.c_int64, vp, vp, C.c_size_t, vp, vp]
        lib.dc_gae.restype = C.c_int
        lib.dc_gae.argtypes = [C.POINTER(dc_params), C.POINTER(dc_source), vp, vp, C.POINTER(vp), C.POINTER(vp),
                               C.POINTER(vp), C.POINTER(vp), C.c_double, C.c_double, C.c_double,
                               C.POINTER(vp), C.POINTER(vp), vp, vp]
        lib.dc_balance_group_advantage.restype = C.c_int
        lib.dc_balance_group_advantage.argtypes = [C.POINTER(dc_params), C.POINTER(dc_source), vp, vp, vp, vp, vp, vp, vp,
                                                   C.c_int32, C.POINTER(vp), vp, C.POINTER(vp), vp, vp]
        lib.dc_balance_plan_group_advantage.restype = C.c_int
        lib.dc_balance_plan_group_advantage.argtypes = [C.POINTER(dc_params), C.POINTER(dc_source), vp, vp, vp, vp, vp, vp, vp,
                                                        C.c_int32, C.POINTER(vp), vp, C.POINTER(vp), C.c_int64,
                                                        vp, vp, vp, vp, vp, vp, vp, C.c_size_t, vp, vp]
        _lib = lib
    return _lib


def strerror(code: int) -> str:
    return load().dc_strerror(int(code)).decode()


def _ptr(x) -> Optional[int]:
    """Device address of a torch tensor (or pass an int / None through)."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if not x.is_cuda:
        raise TypeError("expected a device tensor")
    if not x.is_contiguous():
        raise TypeError("expected a contiguous tensor")
    return x.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def make_params(n_seq: int, n_shards: int, token_budget: int, eps: float = 1e-6, ddof: int = 1,
                cap: int = 0, align_tokens: int = 1) -> dc_params:
    return dc_params(n_seq, n_shards, cap, align_tokens, token_budget, eps, ddof, 0)


class Source:
    """Keeps the host arrays of a dc_source alive next to the struct."""

    def __init__(self, shard_seq_off: Sequence[int], shard_tokens: Sequence[int], d_src_tok_off):
        n = len(shard_tokens)
        self._seq_off = (C.c_int32 * (n + 1))(*[int(v) for v in shard_seq_off])
        self._tokens = (C.c_int64 * n)(*[int(v) for v in shard_tokens])
        self._keep = d_src_tok_off
        self.struct = dc_source(n, 0, C.cast(self._seq_off, C.POINTER(C.c_int32)),
                                C.cast(self._tokens, C.POINTER(C.c_int64)), _ptr(d_src_tok_off))
        self.n_src_shards = n


def _ptr_array(items: Sequence) -> C.Array:
    return (C.c_void_p * len(items))(*[_ptr(t) for t in items])


class Fields:
    """Host array of dc_field built from (src tensors per rollout shard, dst tensor, elem_bytes)."""

    def __init__(self, specs: Sequence[tuple]):
        self._src_arrays = []
        self._keep = specs
        self.array = (dc_field * max(1, len(specs)))()
        for i, (srcs, dst, elem_bytes) in enumerate(specs):
            arr = _ptr_array(srcs)
            self._src_arrays.append(arr)
            self.array[i] = dc_field(C.cast(arr, C.POINTER(C.c_void_p)), _ptr(dst), int(elem_bytes), 0)
        self.n = len(specs)


def _check(rc: int, where: str) -> None:
    if rc != DC_OK:
        raise DcError(rc, where)


def dc_workspace_bytes(prm: dc_params, dst_capacity_tokens: int) -> int:
    return int(load().dc_workspace_bytes(C.byref(prm), int(dst_capacity_tokens)))


def dc_balance(prm: dc_params, d_seq_len, d_perm, d_shard_seq_off, d_shard_of_seq, d_shard_load,
               d_status, stream=None) -> None:
    _check(load().dc_balance(C.byref(prm), _ptr(d_seq_len), _ptr(d_perm), _ptr(d_shard_seq_off),
                             _ptr(d_shard_of_seq), _ptr(d_shard_load), _ptr(d_status), _stream(stream)),
           "dc_balance")


def dc_balance_workspace_bytes(prm: dc_params) -> int:
    return int(load().dc_balance_workspace_bytes(C.byref(prm)))


def dc_balance_ws(prm: dc_params, d_seq_len, d_perm, d_shard_seq_off, d_shard_of_seq, d_shard_load,
                  d_ws, ws_bytes: int, d_status, stream=None) -> None:
    _check(load().dc_balance_ws(C.byref(prm), _ptr(d_seq_len), _ptr(d_perm), _ptr(d_shard_seq_off),
                                _ptr(d_shard_of_seq), _ptr(d_shard_load), _ptr(d_ws), int(ws_bytes), _ptr(d_status),
                                _stream(stream)),
           "dc_balance_ws")


def dc_group_advantage(prm: dc_params, src: Source, d_seq_len, d_reward, d_group_off, n_groups: int,
                       mask_src: Optional[Sequence], d_adv_seq, adv_tok_src: Optional[Sequence],
                       d_status, stream=None) -> None:
    m = _ptr_array(mask_src) if mask_src is not None else None
    a = _ptr_array(adv_tok_src) if adv_tok_src is not None else None
    _check(load().dc_group_advantage(C.byref(prm), C.byref(src.struct), _ptr(d_seq_len), _ptr(d_reward),
                                     _ptr(d_group_off), int(n_groups),
                                     C.cast(m, C.POINTER(C.c_void_p)) if m is not None else None,
                                     _ptr(d_adv_seq),
                                     C.cast(a, C.POINTER(C.c_void_p)) if a is not None else None,
                                     _ptr(d_status), _stream(stream)),
           "dc_group_advantage")


def dc_plan(prm: dc_params, src: Source, d_seq_len, d_perm, d_shard_seq_off, dst_capacity_tokens: int,
            d_dst_tok_off, d_shard_tok_off, d_shard_mb_off, d_mb_seq_off, d_cu_seqlens, d_n_mb,
            d_ws, ws_bytes: int, d_status, stream=None) -> None:
    _check(load().dc_plan(C.byref(prm), C.byref(src.struct), _ptr(d_seq_len), _ptr(d_perm), _ptr(d_shard_seq_off),
                          int(dst_capacity_tokens), _ptr(d_dst_tok_off), _ptr(d_shard_tok_off),
                          _ptr(d_shard_mb_off), _ptr(d_mb_seq_off), _ptr(d_cu_seqlens), _ptr(d_n_mb),
                          _ptr(d_ws), int(ws_bytes), _ptr(d_status), _stream(stream)),
           "dc_plan")


def dc_gather(prm: dc_params, src: Source, fields: Fields, dst_capacity_tokens: int, d_dst_tok_off,
              d_ws, ws_bytes: int, d_status, stream=None) -> None:
    _check(load().dc_gather(C.byref(prm), C.byref(src.struct), fields.array, fields.n, int(dst_capacity_tokens),
                            _ptr(d_dst_tok_off), _ptr(d_ws), int(ws_bytes), _ptr(d_status), _stream(stream)),
           "dc_gather")


def _event(ev) -> Optional[int]:
    """Raw hipEvent_t of a torch.cuda.Event that has been recorded at least once (torch creates the HIP event at
    its first record), or of an integer handle; None stays None."""
    if ev is None:
        return None
    if isinstance(ev, int):
        return ev or None
    h = ev.cuda_event
    h = getattr(h, "value", h)
    if not h:
        raise ValueError("the event has no HIP handle yet: record it once before passing it")
    return int(h)


def dc_gather_timed(prm: dc_params, src: Source, fields: Fields, dst_capacity_tokens: int, d_dst_tok_off,
                    d_ws, ws_bytes: int, d_status, event_begins, event_ends, stream=None) -> None:
    _check(load().dc_gather_timed(C.byref(prm), C.byref(src.struct), fields.array, fields.n, int(dst_capacity_tokens),
                                  _ptr(d_dst_tok_off), _ptr(d_ws), int(ws_bytes), _ptr(d_status), _stream(stream),
                                  _event(event_begins), _event(event_ends)),
           "dc_gather_timed")


def dc_gather_advantage(prm: dc_params, src: Source, fields: Fields, mask_field: int, d_perm, d_adv_seq,
                        d_adv_tok_dst, dst_capacity_tokens: int, d_dst_tok_off, d_ws, ws_bytes: int, d_status,
                        stream=None) -> None:
    _check(load().dc_gather_advantage(C.byref(prm), C.byref(src.struct), fields.array, fields.n, int(mask_field),
                                      _ptr(d_perm), _ptr(d_adv_seq), _ptr(d_adv_tok_dst), int(dst_capacity_tokens),
                                      _ptr(d_dst_tok_off), _ptr(d_ws), int(ws_bytes), _ptr(d_status),
                                      _stream(stream)),
           "dc_gather_advantage")


def dc_repack(prm: dc_params, src: Source, d_seq_len, d_perm, d_shard_seq_off, fields: Fields,
              dst_capacity_tokens: int, d_dst_tok_off, d_shard_tok_off, d_shard_mb_off, d_mb_seq_off,
              d_cu_seqlens, d_n_mb, d_ws, ws_bytes: int, d_status, stream=None) -> None:
    _check(load().dc_repack(C.byref(prm), C.byref(src.struct), _ptr(d_seq_len), _ptr(d_perm), _ptr(d_shard_seq_off),
                            fields.array, fields.n, int(dst_capacity_tokens), _ptr(d_dst_tok_off),
                            _ptr(d_shard_tok_off), _ptr(d_shard_mb_off), _ptr(d_mb_seq_off), _ptr(d_cu_seqlens),
                            _ptr(d_n_mb), _ptr(d_ws), int(ws_bytes), _ptr(d_status), _stream(stream)),
           "dc_repack")


def dc_repack_noalloc(prm: dc_params, src: Source, d_seq_len, d_perm, d_shard_seq_off, fields: Fields,
                      dst_capacity_tokens: int, d_dst_tok_off, d_shard_tok_off, d_shard_mb_off, d_mb_seq_off,
                      d_cu_seqlens, d_n_mb, d_status, stream=None) -> None:
    _check(load().dc_repack_noalloc(C.byref(prm), C.byref(src.struct), _ptr(d_seq_len), _ptr(d_perm),
                                    _ptr(d_shard_seq_off), fields.array, fields.n, int(dst_capacity_tokens),
                                    _ptr(d_dst_tok_off), _ptr(d_shard_tok_off), _ptr(d_shard_mb_off),
                                    _ptr(d_mb_seq_off), _ptr(d_cu_seqlens), _ptr(d_n_mb), _ptr(d_status),
                                    _stream(stream)),
           "dc_repack_noalloc")


def dc_scatter_workspace_bytes(prm: dc_params, src: Source) -> int:
    return int(load().dc_scatter_workspace_bytes(C.byref(prm), C.byref(src.struct)))


def dc_scatter(prm: dc_params, src: Source, d_seq_len, d_perm, fields: Fields, dst_capacity_tokens: int,
               d_dst_tok_off, d_ws, ws_bytes: int, d_status, stream=None) -> None:
    """fields: as for dc_gather, with the roles swapped (dst = training arena read, srcs = rollout buffers written)."""
    _check(load().dc_scatter(C.byref(prm), C.byref(src.struct), _ptr(d_seq_len), _ptr(d_perm), fields.array, fields.n,
                             int(dst_capacity_tokens), _ptr(d_dst_tok_off), _ptr(d_ws), int(ws_bytes),
                             _ptr(d_status), _stream(stream)),
           "dc_scatter")


def dc_gae(prm: dc_params, src: Source, d_seq_len, d_reward, value_src: Sequence, mask_src: Sequence,
           logp_src: Optional[Sequence], ref_src: Optional[Sequence], gamma: float, lam: float, kl_coef: float,
           adv_tok_src: Sequence, ret_tok_src: Sequence, d_status, stream=None) -> None:
    def arr(x):
        return C.cast(_ptr_array(x), C.POINTER(C.c_void_p)) if x is not None else None
    keep = [arr(value_src), arr(mask_src), arr(logp_src), arr(ref_src), arr(adv_tok_src), arr(ret_tok_src)]
    _check(load().dc_gae(C.byref(prm), C.byref(src.struct), _ptr(d_seq_len), _ptr(d_reward), keep[0], keep[1],
                         keep[2], keep[3], float(gamma), float(lam), float(kl_coef), keep[4], keep[5],
                         _ptr(d_status), _stream(stream)),
           "dc_gae")


def dc_balance_group_advantage(prm: dc_params, src: Source, d_seq_len, d_perm, d_shard_seq_off, d_shard_of_seq,
                               d_shard_load, d_reward, d_group_off, n_groups: int, mask_src: Optional[Sequence],
                               d_adv_seq, adv_tok_src: Optional[Sequence], d_status, stream=None) -> None:
    m = _ptr_array(mask_src) if mask_src is not None else None
    a = _ptr_array(adv_tok_src) if adv_tok_src is not None else None
    _check(load().dc_balance_group_advantage(
        C.byref(prm), C.byref(src.struct), _ptr(d_seq_len), _ptr(d_perm), _ptr(d_shard_seq_off), _ptr(d_shard_of_seq),
        _ptr(d_shard_load), _ptr(d_reward), _ptr(d_group_off), int(n_groups),
        C.cast(m, C.POINTER(C.c_void_p)) if m is not None else None, _ptr(d_adv_seq),
        C.cast(a, C.POINTER(C.c_void_p)) if a is not None else None, _ptr(d_status), _stream(stream)),
        "dc_balance_group_advantage")


def dc_balance_plan_group_advantage(prm: dc_params, src: Source, d_seq_len, d_perm, d_shard_seq_off, d_shard_of_seq,
                                    d_shard_load, d_reward, d_group_off, n_groups: int, mask_src: Optional[Sequence],
                                    d_adv_seq, adv_tok_src: Optional[Sequence], dst_capacity_tokens: int, d_dst_tok_off,
                                    d_shard_tok_off, d_shard_mb_off, d_mb_seq_off, d_cu_seqlens, d_n_mb, d_ws,
                                    ws_bytes: int, d_status, stream=None) -> None:
    m = _ptr_array(mask_src) if mask_src is not None else None
    a = _ptr_array(adv_tok_src) if adv_tok_src is not None else None
    _check(load().dc_balance_plan_group_advantage(
        C.byref(prm), C.byref(src.struct), _ptr(d_seq_len), _ptr(d_perm), _ptr(d_shard_seq_off), _ptr(d_shard_of_seq),
        _ptr(d_shard_load), _ptr(d_reward), _ptr(d_group_off), int(n_groups),
        C.cast(m, C.POINTER(C.c_void_p)) if m is not None else None, _ptr(d_adv_seq),
        C.cast(a, C.POINTER(C.c_void_p)) if a is not None else None, int(dst_capacity_tokens), _ptr(d_dst_tok_off),
        _ptr(d_shard_tok_off), _ptr(d_shard_mb_off), _ptr(d_mb_seq_off), _ptr(d_cu_seqlens), _ptr(d_n_mb),
        _ptr(d_ws), int(ws_bytes), _ptr(d_status), _stream(stream)),
        "dc_balance_plan_group_advantage")
