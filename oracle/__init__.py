"""ctypes front end of the fp64 CPU oracle (``oracle_attn.c``).

TEST INFRASTRUCTURE ONLY.  The oracle is the plain definition of the chunked
block-diffusion attention step (Optimus Sec. 4 and Sec. 6) in fp64; the tests,
the smoke check and the benchmark's cpu_baseline leg are its only callers.  It
imports nothing from the HIP package and the HIP package imports nothing from
here.

All array arguments are numpy arrays: bf16 data as ``uint16`` bit patterns,
descriptors as ``int32``.  Outputs are ``float64``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle_attn.c")
_SRCS = [_SRC, os.path.join(_HERE, "oracle_commit.c")]
_LIB = os.path.join(_HERE, "liboracle_attn.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile ``oracle_attn.c`` with gcc into ``liboracle_attn.so`` (in place)."""
    if force or not os.path.exists(_LIB) or \
            os.path.getmtime(_LIB) < max(os.path.getmtime(f) for f in _SRCS):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               *_SRCS, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class Params(ctypes.Structure):
    _fields_ = [
        ("num_q_heads", ctypes.c_int32),
        ("num_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32),
        ("page_size", ctypes.c_int32),
        ("block_size", ctypes.c_int32),
        ("mask_mode", ctypes.c_int32),
        ("kv_layout", ctypes.c_int32),
        ("max_pages_per_req", ctypes.c_int32),
        ("k_stride_page", ctypes.c_int64),
        ("k_stride_head", ctypes.c_int64),
        ("v_stride_page", ctypes.c_int64),
        ("v_stride_head", ctypes.c_int64),
        ("scale", ctypes.c_double),
    ]


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_num_threads.restype = ctypes.c_int
        for name in ("oracle_kv_append", "oracle_chunked_attention", "oracle_chunked_attention_pos",
                     "oracle_attention_probs",
                     "oracle_partial_row"):
            getattr(_lib, name).restype = ctypes.c_int
        _lib.oracle_merge_partials.restype = None
        _lib.oracle_commit.restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def make_params(*, num_q_heads, num_kv_heads, head_dim, page_size, block_size,
                max_pages_per_req, mask_mode=0, kv_layout=1, scale=0.0,
                k_stride_page=None, k_stride_head=None, v_stride_page=None,
                v_stride_head=None) -> Params:
    """Strides default to a dense pool ``[num_pages, Hkv, P*D]``."""
    tile = page_size * head_dim
    p = Params()
    p.num_q_heads, p.num_kv_heads, p.head_dim = num_q_heads, num_kv_heads, head_dim
    p.page_size, p.block_size, p.mask_mode, p.kv_layout = page_size, block_size, mask_mode, kv_layout
    p.max_pages_per_req = max_pages_per_req
    p.k_stride_head = tile if k_stride_head is None else k_stride_head
    p.v_stride_head = tile if v_stride_head is None else v_stride_head
    p.k_stride_page = num_kv_heads * tile if k_stride_page is None else k_stride_page
    p.v_stride_page = num_kv_heads * tile if v_stride_page is None else v_stride_page
    p.scale = float(scale)
    return p


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _u16(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, a.dtype
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16))


def _f64(a):
    assert a.dtype == np.float64 and a.flags.c_contiguous
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def kv_append(p: Params, cu_q, prefix_len, block_table, k_new, v_new, k_pool, v_pool) -> None:
    """In place: scatter chunk K/V rows to logical slots L_i..L_i+c_i-1 of the pools."""
    lib = _load()
    cu, cu_p = _i32(cu_q)
    pl, pl_p = _i32(prefix_len)
    bt, bt_p = _i32(block_table)
    kn, kn_p = _u16(k_new)
    vn, vn_p = _u16(v_new)
    assert k_pool.dtype == np.uint16 and k_pool.flags.c_contiguous
    assert v_pool.dtype == np.uint16 and v_pool.flags.c_contiguous
    rc = lib.oracle_kv_append(ctypes.byref(p), ctypes.c_int32(len(pl)), cu_p, pl_p, bt_p, kn_p, vn_p,
                              k_pool.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16)),
                              v_pool.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16)))
    if rc != 0:
        raise ValueError("oracle_kv_append: bad descriptor")


def chunked_attention(p: Params, cu_q, prefix_len, block_start, block_table, q, k_new, v_new,
                      k_pool, v_pool, q_pos=None) -> np.ndarray:
    """fp64 ``[T, Hq, D]`` attention output of the whole ragged batch.  ``q_pos``: optional
    int32 ``[T]`` sequence positions of the chunk tokens (mask mode 1 only)."""
    lib = _load()
    cu, cu_p = _i32(cu_q)
    pl, pl_p = _i32(prefix_len)
    bs, bs_p = _i32(block_start)
    bt, bt_p = _i32(block_table)
    qq, q_p = _u16(q)
    kn, kn_p = _u16(k_new)
    vn, vn_p = _u16(v_new)
    kp, kp_p = _u16(k_pool)
    vp, vp_p = _u16(v_pool)
    T = int(cu[-1])
    out = np.zeros((T, p.num_q_heads, p.head_dim), dtype=np.float64)
    if q_pos is None:
        pos_p = ctypes.POINTER(ctypes.c_int32)()
    else:
        pos, pos_p = _i32(q_pos)
        assert len(pos) == T
    rc = lib.oracle_chunked_attention_pos(ctypes.byref(p), ctypes.c_int32(len(pl)), cu_p, pl_p, bs_p,
                                          bt_p, q_p, kn_p, vn_p, kp_p, vp_p, pos_p, _f64(out))
    if rc != 0:
        raise ValueError("oracle_chunked_attention: bad descriptor")
    return out


def attention_probs(p: Params, cu_q, prefix_len, block_start, block_table, q, k_new, v_new,
                    k_pool, v_pool, i: int, j: int, h: int) -> np.ndarray:
    """Normalised softmax row of chunk token j of request i, query head h."""
    lib = _load()
    cu, cu_p = _i32(cu_q)
    pl, pl_p = _i32(prefix_len)
    bs, bs_p = _i32(block_start)
    bt, bt_p = _i32(block_table)
    qq, q_p = _u16(q)
    kn, kn_p = _u16(k_new)
    vn, vn_p = _u16(v_new)
    kp, kp_p = _u16(k_pool)
    vp, vp_p = _u16(v_pool)
    n = int(pl[i] + cu[i + 1] - cu[i])
    probs = np.zeros(n, dtype=np.float64)
    rc = lib.oracle_attention_probs(ctypes.byref(p), ctypes.c_int32(len(pl)), cu_p, pl_p, bs_p,
                                    bt_p, q_p, kn_p, vn_p, kp_p, vp_p, ctypes.c_int32(i),
                                    ctypes.c_int32(j), ctypes.c_int32(h), _f64(probs))
    if rc != 0:
        raise ValueError("oracle_attention_probs: bad argument")
    return probs


def partial_row(p: Params, cu_q, prefix_len, block_start, block_table, q, k_new, v_new, k_pool,
                v_pool, i: int, j: int, h: int, lo: int, hi: int):
    """Un-normalised partial ``(o_part[D], m, l)`` of one row over keys [lo, hi)."""
    lib = _load()
    cu, cu_p = _i32(cu_q)
    pl, pl_p = _i32(prefix_len)
    bs, bs_p = _i32(block_start)
    bt, bt_p = _i32(block_table)
    qq, q_p = _u16(q)
    kn, kn_p = _u16(k_new)
    vn, vn_p = _u16(v_new)
    kp, kp_p = _u16(k_pool)
    vp, vp_p = _u16(v_pool)
    o = np.zeros(p.head_dim, dtype=np.float64)
    m = ctypes.c_double()
    l = ctypes.c_double()
    rc = lib.oracle_partial_row(ctypes.byref(p), ctypes.c_int32(len(pl)), cu_p, pl_p, bs_p, bt_p,
                                q_p, kn_p, vn_p, kp_p, vp_p, ctypes.c_int32(i), ctypes.c_int32(j),
                                ctypes.c_int32(h), ctypes.c_int32(lo), ctypes.c_int32(hi), _f64(o),
                                ctypes.byref(m), ctypes.byref(l))
    if rc != 0:
        raise ValueError("oracle_partial_row: bad argument")
    return o, m.value, l.value


def merge_partials(o_part: np.ndarray, m: np.ndarray, l: np.ndarray) -> np.ndarray:
    """Merge S partials of one row: ``o_part [S, D]``, ``m [S]``, ``l [S]`` -> ``o [D]``."""
    lib = _load()
    o_part = np.ascontiguousarray(o_part, dtype=np.float64)
    m = np.ascontiguousarray(m, dtype=np.float64)
    l = np.ascontiguousarray(l, dtype=np.float64)
    S, D = o_part.shape
    o = np.zeros(D, dtype=np.float64)
    lib.oracle_merge_partials(ctypes.c_int32(S), ctypes.c_int32(D), _f64(o_part), _f64(m), _f64(l),
                              _f64(o))
    return o


def commit(logits_bits: np.ndarray, vocab: int, threshold: float, cu_q=None, min_commit: int = 0):
    """Commit step on bf16 logits ``[T, row_stride]`` (uint16 bit patterns).

    Returns ``(token int32 [T], confidence float64 [T], commit int32 [T])``.
    """
    lib = _load()
    logits_bits = np.ascontiguousarray(logits_bits)
    assert logits_bits.dtype == np.uint16 and logits_bits.ndim == 2
    T, stride = logits_bits.shape
    token = np.zeros(T, dtype=np.int32)
    conf = np.zeros(T, dtype=np.float64)
    com = np.zeros(T, dtype=np.int32)
    if cu_q is None:
        cu_p, batch = ctypes.POINTER(ctypes.c_int32)(), 0
    else:
        cu, cu_p = _i32(cu_q)
        batch = len(cu) - 1
    rc = lib.oracle_commit(ctypes.c_int32(T), ctypes.c_int32(vocab), ctypes.c_int64(stride),
                           logits_bits.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16)),
                           ctypes.c_double(threshold), ctypes.c_int32(batch), cu_p,
                           ctypes.c_int32(min_commit),
                           token.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), _f64(conf),
                           com.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)))
    if rc != 0:
        raise ValueError("oracle_commit: bad argument")
    return token, conf, com


from .oracle_reorg import reorganise  # noqa: E402,F401  (step-wise reorganisation, Sec. 4.4)
from . import oracle_selector as selector  # noqa: E402,F401  (chunk-size selection, Sec. 5)
