"""CPU oracle for the Data Coordinator reshard path -- TEST INFRASTRUCTURE ONLY.

Thin ctypes/NumPy marshalling over ``dc_oracle.c`` (plain C, float64 statistics,
Algorithm 1 as a scan over the workers per sequence, per-sequence copy loops).  Only tests, the smoke
check and the benchmark's CPU-baseline leg may import this package; the HIP
product path never does, and this package never imports the product.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import Optional, List, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dc_oracle.c")
_LIB = os.path.join(_HERE, "libdc_oracle.so")

_ERR = {1: "bad argument", 2: "N mod K != 0 (Algorithm 1 assertion)", 3: "sequence exceeds token budget",
        4: "zero or negative sequence length", 5: "out of memory"}


class OracleError(RuntimeError):
    def __init__(self, code: int):
        super().__init__(f"oracle error {code}: {_ERR.get(code, '?')}")
        self.code = code


def build(force: bool = False) -> str:
    """Compile dc_oracle.c with gcc into libdc_oracle.so next to it."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-shared", "-fPIC",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        for name in ("dco_balance", "dco_group_advantage", "dco_adv_broadcast", "dco_plan", "dco_gather",
                     "dco_scatter", "dco_gae"):
            getattr(_lib, name).restype = C.c_int
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def _chk(rc: int):
    if rc != 0:
        raise OracleError(rc)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


@dataclass
class Balance:
    perm: np.ndarray           # int32 [N]
    shard_seq_off: np.ndarray  # int32 [K+1]
    shard_of_seq: np.ndarray   # int32 [N]
    shard_load: np.ndarray     # int64 [K]


def balance(seq_len, K: int, cap: int = 0) -> Balance:
    """Algorithm 1 (Constrained LPT).  cap=0 -> C = N/K as in the paper."""
    S = _i32(seq_len)
    N = len(S)
    perm = np.empty(N, np.int32)
    off = np.empty(K + 1, np.int32)
    sos = np.empty(N, np.int32)
    load = np.empty(K, np.int64)
    _chk(_load().dco_balance(_p(S), C.c_int32(N), C.c_int32(K), C.c_int32(cap),
                             _p(perm), _p(off), _p(sos), _p(load)))
    return Balance(perm, off, sos, load)


def group_advantage(reward, group_off, eps: float, ddof: int = 1) -> np.ndarray:
    r = np.ascontiguousarray(reward, dtype=np.float32)
    go = _i32(group_off)
    out = np.zeros(len(r), np.float32)
    _chk(_load().dco_group_advantage(_p(r), _p(go), C.c_int32(len(go) - 1), C.c_double(eps),
                                     C.c_int32(ddof), _p(out)))
    return out


def adv_broadcast(adv_seq, seq_len, src_tok_off, src_shard_seq_off, src_shard_tokens,
                  mask_shards: Sequence[np.ndarray]) -> List[np.ndarray]:
    """Per-token advantages in the rollout layout, one array per rollout shard."""
    a = np.ascontiguousarray(adv_seq, dtype=np.float32)
    S = _i32(seq_len)
    sto = np.ascontiguousarray(src_tok_off, dtype=np.int64)
    outs = []
    for s, m in enumerate(mask_shards):
        m = np.ascontiguousarray(m, dtype=np.uint8)
        out = np.zeros(int(src_shard_tokens[s]), np.float32)
        _chk(_load().dco_adv_broadcast(_p(a), _p(S), _p(sto), C.c_int32(int(src_shard_seq_off[s])),
                                       C.c_int32(int(src_shard_seq_off[s + 1])), _p(m), _p(out)))
        outs.append(out)
    return outs


def gae(reward, seq_len, src_tok_off, src_shard_seq_off, src_shard_tokens, value_shards: Sequence[np.ndarray],
        mask_shards: Sequence[np.ndarray], gamma: float, lam: float, kl_coef: float = 0.0,
        logp_shards: Optional[Sequence[np.ndarray]] = None, ref_shards: Optional[Sequence[np.ndarray]] = None):
    """Generalized advantage estimation over the loss-bearing tokens of every sequence, rollout
    layout.  Returns (adv_tok shards, return shards), float32."""
    r = np.ascontiguousarray(reward, dtype=np.float32)
    S = _i32(seq_len)
    sto = np.ascontiguousarray(src_tok_off, dtype=np.int64)
    advs, rets = [], []
    for s, (v, m) in enumerate(zip(value_shards, mask_shards)):
        v = np.ascontiguousarray(v, dtype=np.float32)
        m = np.ascontiguousarray(m, dtype=np.uint8)
        lp = np.ascontiguousarray(logp_shards[s], dtype=np.float32) if logp_shards is not None else None
        rf = np.ascontiguousarray(ref_shards[s], dtype=np.float32) if ref_shards is not None else None
        n = int(src_shard_tokens[s])
        adv, ret = np.zeros(n, np.float32), np.zeros(n, np.float32)
        _chk(_load().dco_gae(_p(r), _p(S), _p(sto), C.c_int32(int(src_shard_seq_off[s])),
                             C.c_int32(int(src_shard_seq_off[s + 1])), _p(v), _p(m),
                             _p(lp) if lp is not None else None, _p(rf) if rf is not None else None,
                             C.c_double(gamma), C.c_double(lam), C.c_double(kl_coef), _p(adv), _p(ret)))
        advs.append(adv)
        rets.append(ret)
    return advs, rets


@dataclass
class Plan:
    dst_tok_off: np.ndarray    # int64 [N+1]
    shard_tok_off: np.ndarray  # int64 [K+1]
    shard_mb_off: np.ndarray   # int32 [K+1]
    mb_seq_off: np.ndarray     # int32 [M+1]
    cu_seqlens: np.ndarray     # int32 [N+M]
    n_mb: int


def plan(seq_len, perm, shard_seq_off, budget: int, align: int = 1) -> Plan:
    S = _i32(seq_len)
    N = len(S)
    pm = _i32(perm)
    off = _i32(shard_seq_off)
    K = len(off) - 1
    dst = np.zeros(N + 1, np.int64)
    sto = np.zeros(K + 1, np.int64)
    smo = np.zeros(K + 1, np.int32)
    mso = np.zeros(N + 1, np.int32)
    cu = np.zeros(2 * N + 1, np.int32)
    n_mb = C.c_int32(0)
    _chk(_load().dco_plan(_p(S), C.c_int32(N), _p(pm), _p(off), C.c_int32(K), C.c_int64(budget),
                          C.c_int32(align), _p(dst), _p(sto), _p(smo), _p(mso), _p(cu), C.byref(n_mb)))
    M = n_mb.value
    return Plan(dst, sto, smo, mso[:M + 1].copy(), cu[:N + M].copy(), M)


def gather(seq_len, perm, src_tok_off, src_shard_seq_off, src_shards: Sequence[np.ndarray],
           dst_tok_off, dst_tokens: int, fill=None) -> np.ndarray:
    """Repack one field; returns the destination arena (dst_tokens elements)."""
    S = _i32(seq_len)
    N = len(S)
    pm = _i32(perm)
    sto = np.ascontiguousarray(src_tok_off, dtype=np.int64)
    sso = _i32(src_shard_seq_off)
    dto = np.ascontiguousarray(dst_tok_off, dtype=np.int64)
    srcs = [np.ascontiguousarray(x) for x in src_shards]
    dt = srcs[0].dtype
    dst = np.zeros(dst_tokens, dt) if fill is None else np.full(dst_tokens, fill, dt)
    ptrs = (C.c_void_p * len(srcs))(*[x.ctypes.data for x in srcs])
    _chk(_load().dco_gather(_p(S), C.c_int32(N), _p(pm), _p(sto), _p(sso), C.c_int32(len(srcs)), ptrs,
                            _p(dst), C.c_int32(dt.itemsize), _p(dto)))
    return dst


def gather_slots(seq_len, perm, src_tok_off, src_shard_seq_off, src_shards: Sequence[np.ndarray],
                 dst_tok_off, dst: np.ndarray, j0: int, j1: int) -> None:
    """The same copy for the output slots [j0, j1) only, into a destination arena the caller made:
    dco_gather called on that part of perm / dst_tok_off.  Calls on disjoint slot ranges write
    disjoint elements, so they may run in threads of their own (ctypes releases the interpreter lock)."""
    S = _i32(seq_len)
    pm = _i32(perm)
    sto = np.ascontiguousarray(src_tok_off, dtype=np.int64)
    sso = _i32(src_shard_seq_off)
    dto = np.ascontiguousarray(dst_tok_off, dtype=np.int64)
    srcs = [np.ascontiguousarray(x) for x in src_shards]
    assert dst.flags.c_contiguous and dst.dtype == srcs[0].dtype and 0 <= j0 <= j1 <= len(pm)
    ptrs = (C.c_void_p * len(srcs))(*[x.ctypes.data for x in srcs])
    _chk(_load().dco_gather(_p(S), C.c_int32(j1 - j0), C.c_void_p(pm.ctypes.data + 4 * j0), _p(sto), _p(sso),
                            C.c_int32(len(srcs)), ptrs, _p(dst), C.c_int32(dst.dtype.itemsize),
                            C.c_void_p(dto.ctypes.data + 8 * j0)))


def scatter(seq_len, perm, src_tok_off, src_shard_seq_off, arena: np.ndarray, dst_tok_off,
            rollout_shards: Sequence[np.ndarray]) -> List[np.ndarray]:
    """Reverse of gather for one field: training arena -> copies of the given rollout buffers
    (one per rollout shard; elements outside every sequence keep the given values)."""
    S = _i32(seq_len)
    N = len(S)
    pm = _i32(perm)
    sto = np.ascontiguousarray(src_tok_off, dtype=np.int64)
    sso = _i32(src_shard_seq_off)
    dto = np.ascontiguousarray(dst_tok_off, dtype=np.int64)
    ar = np.ascontiguousarray(arena)
    outs = [np.array(x, dtype=ar.dtype, copy=True, order="C") for x in rollout_shards]
    ptrs = (C.c_void_p * len(outs))(*[x.ctypes.data for x in outs])
    _chk(_load().dco_scatter(_p(S), C.c_int32(N), _p(pm), _p(sto), _p(sso), C.c_int32(len(outs)), ptrs,
                             _p(ar), C.c_int32(ar.dtype.itemsize), _p(dto)))
    return outs
