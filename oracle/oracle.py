"""ctypes front end of the CPU oracle (ukv_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the
benchmark's cpu_baseline leg; never by the product package.  It marshals numpy
arrays into the C routines and does no arithmetic of its own.  Batches are
duck-typed (any object with the fields of a synthetic batch) so that this
module imports neither the input generators nor the HIP binding.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ukv_oracle.c")
_LIB = os.path.join(_HERE, "libukv_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP over requests)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.check_call(cmd)
    return _LIB


def bind(cdll):
    """Declare the return types of the oracle's entry points on a loaded library."""
    for name in ("ukv_oracle_gather", "ukv_oracle_scatter", "ukv_oracle_append", "ukv_oracle_attention",
                 "ukv_oracle_attention_range", "ukv_oracle_merge", "ukv_oracle_prefill", "ukv_oracle_threads"):
        getattr(cdll, name).restype = C.c_int
    return cdll


def _load():
    global _lib
    if _lib is None:
        _lib = bind(C.CDLL(build()))
    return _lib


def _p(a: np.ndarray, ty):
    return a.ctypes.data_as(C.POINTER(ty))


def _arr(a, dtype) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=dtype)


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise RuntimeError(f"{what} failed with oracle error {rc}")


def threads() -> int:
    return int(_load().ukv_oracle_threads())


def gather(pool_u16: np.ndarray, page_bytes: int, table: np.ndarray, n_kv_heads: int, head_dim: int,
           n_tokens: int):
    """Contiguous bf16 bit patterns K[n,H,d], V[n,H,d] of one request."""
    lib = _load()
    pool = pool_u16.view(np.uint8)
    table = _arr(table, np.int32)
    k = np.empty((n_tokens, n_kv_heads, head_dim), np.uint16)
    v = np.empty_like(k)
    rc = lib.ukv_oracle_gather(_p(pool, C.c_uint8), C.c_uint64(pool.size), C.c_uint32(page_bytes),
                               _p(table, C.c_int32), C.c_uint64(table.size), C.c_uint32(n_kv_heads),
                               C.c_uint32(head_dim), C.c_uint64(n_tokens), _p(k, C.c_uint16), _p(v, C.c_uint16))
    _check(rc, "gather")
    return k, v


def scatter(pool_u16: np.ndarray, page_bytes: int, table: np.ndarray, k: np.ndarray, v: np.ndarray,
            first_token: int = 0) -> None:
    """Write contiguous bf16 bit patterns K[n,H,d], V[n,H,d] as tokens [first_token, first_token + n) of one
    request, in place (first_token > 0: the bulk append of a chunk behind the tokens already stored)."""
    lib = _load()
    pool = pool_u16.view(np.uint8)
    assert pool.flags.writeable and pool.flags.c_contiguous
    table = _arr(table, np.int32)
    k, v = _arr(k, np.uint16), _arr(v, np.uint16)
    n, H, d = k.shape
    rc = lib.ukv_oracle_scatter(_p(pool, C.c_uint8), C.c_uint64(pool.size), C.c_uint32(page_bytes),
                                _p(table, C.c_int32), C.c_uint64(table.size), C.c_uint32(H), C.c_uint32(d),
                                C.c_uint64(first_token), C.c_uint64(n), _p(k, C.c_uint16), _p(v, C.c_uint16))
    _check(rc, "scatter")


def _per_request_shapes(batch):
    sid = np.asarray(batch.service_id, dtype=np.int64)
    Q = _arr([batch.services[s].n_q_heads for s in sid], np.uint32)
    H = _arr([batch.services[s].n_kv_heads for s in sid], np.uint32)
    d = _arr([batch.services[s].head_dim for s in sid], np.uint32)
    sc = _arr([batch.services[s].softmax_scale for s in sid], np.float64)
    return Q, H, d, sc


def append(batch, pool_u16: np.ndarray, new_k: np.ndarray, new_v: np.ndarray) -> None:
    """Write each request's new token (index ctx_len-1) into the host pool image, in place."""
    lib = _load()
    _, H, d, _ = _per_request_shapes(batch)
    pool = pool_u16.view(np.uint8)
    assert pool.flags.writeable and pool.flags.c_contiguous
    ctx = _arr(batch.ctx_len, np.uint32)
    toff = _arr(batch.table_off, np.uint64)
    tlen = _arr(batch.table_cap, np.uint64)
    pt = _arr(batch.page_table, np.int32)
    nk, nv = _arr(new_k, np.uint16), _arr(new_v, np.uint16)
    noff = _arr(batch.new_off, np.uint64)
    rc = lib.ukv_oracle_append(_p(pool, C.c_uint8), C.c_uint64(pool.size), C.c_uint32(batch.page_bytes),
                               C.c_uint32(ctx.size), _p(H, C.c_uint32), _p(d, C.c_uint32), _p(ctx, C.c_uint32),
                               _p(toff, C.c_uint64), _p(tlen, C.c_uint64), _p(pt, C.c_int32),
                               _p(nk, C.c_uint16), _p(nv, C.c_uint16), _p(noff, C.c_uint64))
    _check(rc, "append")


def attention(batch, pool_u16: np.ndarray, q: Optional[np.ndarray] = None, n_threads: int = 0,
              requests: Optional[Sequence[int]] = None) -> np.ndarray:
    """fp64 decode attention of the batch; returns the flat output (layout of batch.out_off).

    requests: optional subset of request indices; the other outputs are left at NaN.
    """
    lib = _load()
    Q, H, d, sc = _per_request_shapes(batch)
    pool = pool_u16.view(np.uint8)
    ctx = _arr(batch.ctx_len, np.uint32)
    toff = _arr(batch.table_off, np.uint64)
    tlen = _arr(batch.table_cap, np.uint64)
    pt = _arr(batch.page_table, np.int32)
    qq = _arr(batch.q if q is None else q, np.uint16)
    qoff = _arr(batch.q_off, np.uint64)
    ooff = _arr(batch.out_off, np.uint64)
    out = np.full(batch.out_elems, np.nan, np.float64)
    if requests is not None:
        idx = np.asarray(list(requests), dtype=np.int64)
        Q, H, d, sc, ctx, toff, tlen, qoff, ooff = (np.ascontiguousarray(a[idx]) for a in
                                                     (Q, H, d, sc, ctx, toff, tlen, qoff, ooff))
    rc = lib.ukv_oracle_attention(_p(pool, C.c_uint8), C.c_uint64(pool.size), C.c_uint32(batch.page_bytes),
                                  C.c_uint32(ctx.size), _p(Q, C.c_uint32), _p(H, C.c_uint32), _p(d, C.c_uint32),
                                  _p(sc, C.c_double), _p(ctx, C.c_uint32), _p(toff, C.c_uint64),
                                  _p(tlen, C.c_uint64), _p(pt, C.c_int32), _p(qq, C.c_uint16),
                                  _p(qoff, C.c_uint64), _p(out, C.c_double), _p(ooff, C.c_uint64),
                                  C.c_int(n_threads))
    _check(rc, "attention")
    return out


def attention_range(pool_u16: np.ndarray, page_bytes: int, table: np.ndarray, n_q_heads: int, n_kv_heads: int,
                    head_dim: int, scale: float, t0: int, t1: int, q_bits: np.ndarray):
    """(m[Q], l[Q], acc[Q,d]) of one request over tokens [t0, t1), fp64."""
    lib = _load()
    pool = pool_u16.view(np.uint8)
    table = _arr(table, np.int32)
    qq = _arr(q_bits, np.uint16)
    m = np.empty(n_q_heads, np.float64)
    l = np.empty(n_q_heads, np.float64)
    acc = np.empty((n_q_heads, head_dim), np.float64)
    rc = lib.ukv_oracle_attention_range(_p(pool, C.c_uint8), C.c_uint64(pool.size), C.c_uint32(page_bytes),
                                        _p(table, C.c_int32), C.c_uint64(table.size), C.c_uint32(n_q_heads),
                                        C.c_uint32(n_kv_heads), C.c_uint32(head_dim), C.c_double(scale),
                                        C.c_uint64(t0), C.c_uint64(t1), _p(qq, C.c_uint16), _p(m, C.c_double),
                                        _p(l, C.c_double), _p(acc, C.c_double))
    _check(rc, "attention_range")
    return m, l, acc


def prefill(pool_u16: np.ndarray, page_bytes: int, table: np.ndarray, n_q_heads: int, n_kv_heads: int,
            head_dim: int, scale: float, ctx_len: int, positions, q_rows: np.ndarray, n_threads: int = 0):
    """Causal prefill attention of one request at the listed positions: q_rows[k] ([Q, d] bf16 bits) is the
    query of position positions[k] and attends to tokens 0..positions[k].  Returns fp64 [n_pos, Q, d]."""
    lib = _load()
    pool = pool_u16.view(np.uint8)
    table = _arr(table, np.int32)
    pos = _arr(positions, np.uint32)
    qq = _arr(q_rows, np.uint16).reshape(pos.size, n_q_heads, head_dim)
    out = np.empty((pos.size, n_q_heads, head_dim), np.float64)
    rc = lib.ukv_oracle_prefill(_p(pool, C.c_uint8), C.c_uint64(pool.size), C.c_uint32(page_bytes),
                                _p(table, C.c_int32), C.c_uint64(table.size), C.c_uint32(n_q_heads),
                                C.c_uint32(n_kv_heads), C.c_uint32(head_dim), C.c_double(scale),
                                C.c_uint32(ctx_len), C.c_uint32(pos.size), _p(pos, C.c_uint32), _p(qq, C.c_uint16),
                                _p(out, C.c_double), C.c_int(n_threads))
    _check(rc, "prefill")
    return out


def merge(m: np.ndarray, l: np.ndarray, acc: np.ndarray) -> np.ndarray:
    """Combine range statistics of ONE query head: m[c], l[c], acc[c,d] -> out[d]."""
    lib = _load()
    m, l, acc = _arr(m, np.float64), _arr(l, np.float64), _arr(acc, np.float64)
    out = np.empty(acc.shape[1], np.float64)
    rc = lib.ukv_oracle_merge(C.c_uint32(m.size), C.c_uint32(acc.shape[1]), _p(m, C.c_double), _p(l, C.c_double),
                              _p(acc, C.c_double), _p(out, C.c_double))
    _check(rc, "merge")
    return out
