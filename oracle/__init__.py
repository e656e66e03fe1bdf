"""fp64 CPU oracle of the SeerAttention-R decode hot path (test infrastructure).

Only tests/, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may
import this package.  It wraps ``seer_oracle.c`` (plain C, fp64, built with gcc) through
ctypes and shares nothing with the HIP library.  See the header of ``seer_oracle.c`` for
the definitions it writes out and the passages of the paper they follow.

Inputs are CPU tensors/arrays: bf16 data as ``torch.bfloat16`` tensors (or uint16 arrays of
the raw bits), int32 lengths and indices.  Outputs are numpy arrays (fp64 / int32).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "seer_oracle.c")
_SO = os.path.join(_HERE, "libseer_oracle.so")
_lib = None

SELECT_TOPK = 0
SELECT_THRESHOLD = 1
SELECT_TOPP = 2


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP, -O2, no fast-math)."""
    stale = (not os.path.exists(_SO)) or os.path.getmtime(_SO) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _SO + f".tmp{os.getpid()}"
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-ffp-contract=off",
               "-o", tmp, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _SO)
    return _SO


class _KV(ctypes.Structure):
    _fields_ = [
        ("k", ctypes.c_void_p),
        ("v", ctypes.c_void_p),
        ("stride_seq", ctypes.c_int64),
        ("stride_head", ctypes.c_int64),
        ("stride_token", ctypes.c_int64),
        ("page_table", ctypes.c_void_p),
        ("max_pages", ctypes.c_int32),
        ("page_size", ctypes.c_int32),
    ]


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_SO)
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_gate_select.restype = ctypes.c_int
        lib.oracle_gate_select.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
            ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_int, ctypes.c_int32, ctypes.c_void_p, ctypes.c_double, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p]
        lib.oracle_sparse_decode.restype = ctypes.c_int
        lib.oracle_sparse_decode.argtypes = [
            ctypes.c_void_p, ctypes.POINTER(_KV), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_float, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        lib.oracle_sparse_decode_multi.restype = ctypes.c_int
        lib.oracle_sparse_decode_multi.argtypes = [
            ctypes.c_void_p, ctypes.POINTER(_KV), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_float, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        lib.oracle_gate_q.restype = ctypes.c_int
        lib.oracle_gate_q.argtypes = [ctypes.c_void_p] * 4 + [ctypes.c_int, ctypes.c_void_p] + [ctypes.c_int] * 5 + \
            [ctypes.c_void_p, ctypes.c_void_p]
        lib.oracle_kc_update.restype = ctypes.c_int
        lib.oracle_kc_update.argtypes = [ctypes.POINTER(_KV), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                         ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p] + \
            [ctypes.c_int] * 6 + [ctypes.c_void_p, ctypes.c_void_p]
        lib.oracle_attn_ground_truth.restype = ctypes.c_int
        lib.oracle_attn_ground_truth.argtypes = [ctypes.c_void_p, ctypes.POINTER(_KV), ctypes.c_void_p] + \
            [ctypes.c_int] * 6 + [ctypes.c_float, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _bits(x) -> np.ndarray:
    """bf16 tensor (or uint16 array) -> uint16 numpy array of the raw bits (no copy if possible)."""
    if isinstance(x, np.ndarray):
        assert x.dtype == np.uint16
        return x
    import torch
    assert x.dtype == torch.bfloat16 and x.device.type == "cpu"
    return x.view(torch.int16).numpy().view(np.uint16)


def _i32(x) -> Optional[np.ndarray]:
    if x is None:
        return None
    if not isinstance(x, np.ndarray):
        x = x.cpu().numpy()
    return np.ascontiguousarray(x, dtype=np.int32)


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def gate_select(q_gate, kc_cache, seqlens, block_size: int, *, mode: int = SELECT_TOPK,
                budget_tokens: int = 0, budget_blocks=None, threshold: float = 0.0,
                max_sel: int, return_scores: bool = False):
    """Block selection of the AttnGate (Eq. 1c, Sec. 3.1, Sec. 3.2).

    q_gate [B,Hkv,Dg] bf16, kc_cache [B,Hkv,nb_max,Dg] bf16 (last dim contiguous, other dims
    may be strided), seqlens [B] int32.  Returns (block_idx [B,Hkv,max_sel] int32 ascending,
    -1 padded; nblk [B,Hkv] int32[, scores [B,Hkv,nb_max] fp64]).
    """
    lib = _load()
    qg = _bits(q_gate)
    kc = _bits(kc_cache)
    B, Hkv, Dg = qg.shape
    assert kc.shape[0] == B and kc.shape[1] == Hkv and kc.shape[3] == Dg
    nb_max = kc.shape[2]
    qg = np.ascontiguousarray(qg)
    es = kc.itemsize
    assert kc.strides[3] == es
    sb, sh, sj = (kc.strides[0] // es, kc.strides[1] // es, kc.strides[2] // es)
    sl = _i32(seqlens)
    bb = _i32(budget_blocks)
    idx = np.empty((B, Hkv, max_sel), dtype=np.int32)
    cnt = np.empty((B, Hkv), dtype=np.int32)
    scores = np.empty((B, Hkv, nb_max), dtype=np.float64) if return_scores else None
    rc = lib.oracle_gate_select(_ptr(qg), _ptr(kc), sb, sh, sj, _ptr(sl), B, Hkv, Dg, nb_max,
                                block_size, mode, int(budget_tokens), _ptr(bb), float(threshold),
                                _ptr(idx), _ptr(cnt), max_sel, _ptr(scores))
    if rc != 0:
        raise ValueError("oracle_gate_select: a selection does not fit max_sel")
    return (idx, cnt, scores) if return_scores else (idx, cnt)


@dataclass
class KVLayout:
    """Addressing of a bf16 KV cache held in CPU tensors (elements, last dim contiguous).

    contiguous: k/v are [B,Hkv,S_max,d]-shaped views (any strides on the first three dims);
    paged: k/v are pools [n_pages,Hkv,page_size,d] plus page_table [B,max_pages] int32.
    """
    k: object
    v: object
    page_table: object = None
    page_size: int = 0


def sparse_decode(q, kv: KVLayout, seqlens, block_idx, nblk, block_size: int, scale: float,
                  group_filter=None):
    """Attention of the new token over the selected blocks only (Sec. 3.3).

    q [B,Hq,d] bf16.  block_idx None means dense (all blocks).  Returns (out [B,Hq,d] fp64,
    lse [B,Hq] fp64).  Groups with group_filter == 0 are left as NaN.
    """
    lib = _load()
    qb = np.ascontiguousarray(_bits(q))
    B, Hq, d = qb.shape
    kb, vb = _bits(kv.k), _bits(kv.v)
    assert kb.shape == vb.shape and kb.strides == vb.strides and kb.shape[3] == d
    Hkv = kb.shape[1]
    es = kb.itemsize
    assert kb.strides[3] == es
    st = _KV()
    st.k = kb.ctypes.data
    st.v = vb.ctypes.data
    st.stride_seq, st.stride_head, st.stride_token = (kb.strides[0] // es, kb.strides[1] // es,
                                                      kb.strides[2] // es)
    pt = _i32(kv.page_table)
    if pt is not None:
        assert pt.shape[0] == B and kv.page_size > 0
        st.page_table = pt.ctypes.data
        st.max_pages = pt.shape[1]
        st.page_size = kv.page_size
    else:
        assert kb.shape[0] == B
        st.page_table = None
        st.max_pages = 0
        st.page_size = 0
    sl = _i32(seqlens)
    bi = _i32(block_idx)
    nk = _i32(nblk)
    max_sel = 0
    if bi is not None:
        assert bi.shape[:2] == (B, Hkv) and nk.shape == (B, Hkv)
        max_sel = bi.shape[2]
    gf = None
    if group_filter is not None:
        gf = np.ascontiguousarray(np.asarray(group_filter).reshape(B * Hkv), dtype=np.uint8)
    out = np.full((B, Hq, d), np.nan, dtype=np.float64)
    lse = np.full((B, Hq), np.nan, dtype=np.float64)
    rc = lib.oracle_sparse_decode(_ptr(qb), ctypes.byref(st), _ptr(sl), _ptr(bi), _ptr(nk), max_sel,
                                  B, Hq, Hkv, d, block_size, ctypes.c_float(scale), _ptr(out),
                                  _ptr(lse), _ptr(gf))
    if rc != 0:
        raise ValueError("oracle_sparse_decode: bad head counts")
    return out, lse


def _f32(x) -> np.ndarray:
    if not isinstance(x, np.ndarray):
        x = x.cpu().numpy()
    return np.ascontiguousarray(x, dtype=np.float32)


def _kv_struct(k, page_table, page_size, B):
    kb = _bits(k)
    es = kb.itemsize
    assert kb.strides[3] == es
    st = _KV()
    st.k = kb.ctypes.data
    st.v = kb.ctypes.data
    st.stride_seq, st.stride_head, st.stride_token = (kb.strides[0] // es, kb.strides[1] // es, kb.strides[2] // es)
    pt = _i32(page_table)
    if pt is not None:
        st.page_table, st.max_pages, st.page_size = pt.ctypes.data, pt.shape[1], page_size
    else:
        assert kb.shape[0] == B
        st.page_table, st.max_pages, st.page_size = None, 0, 0
    return st, kb, pt


def gate_q(q_nope, wq, rope_cos, rope_sin, seqlens):
    """Q branch of the AttnGate (Eq. 1a).  q_nope [B,Hq,d] bf16 (pre-RoPE queries of the current
    token), wq [Hkv,Dg,g*d] bf16, rope tables [n_pos,Dg/2] fp32, seqlens [B].
    Returns (q_gate fp64 [B,Hkv,Dg] unrounded, q_gate bf16 bits uint16 [B,Hkv,Dg])."""
    lib = _load()
    qb = np.ascontiguousarray(_bits(q_nope))
    wb = np.ascontiguousarray(_bits(wq))
    B, Hq, d = qb.shape
    Hkv, Dg, gd = wb.shape
    assert Hq % Hkv == 0 and gd == (Hq // Hkv) * d
    co, si = _f32(rope_cos), _f32(rope_sin)
    assert co.shape == si.shape and co.shape[1] == Dg // 2
    sl = _i32(seqlens)
    out = np.empty((B, Hkv, Dg), dtype=np.float64)
    bits = np.empty((B, Hkv, Dg), dtype=np.uint16)
    rc = lib.oracle_gate_q(_ptr(qb), _ptr(wb), _ptr(co), _ptr(si), co.shape[0], _ptr(sl), B, Hq, Hkv, d, Dg,
                           _ptr(out), _ptr(bits))
    if rc != 0:
        raise ValueError(f"oracle_gate_q failed ({rc}): bad head counts or a position beyond the rope table")
    return out, bits


def kc_update(k_nope, wk, rope_cos, rope_sin, seqlens, block_size: int, nb_max: int, *, block_begin=None,
              block_end=None, page_table=None, page_size: int = 0, out=None, out_bits=None):
    """K branch of the AttnGate (Eq. 1b): entries [block_begin, block_end) of the K Compression
    Cache of every sequence (default: all full blocks).  k_nope: pre-RoPE keys in KV-cache layout
    (contiguous [B,Hkv,S,d] or paged pool), wk [Hkv,Dg,3d] bf16.
    Returns (kc fp64 [B,Hkv,nb_max,Dg] (NaN where not computed), kc bf16 bits uint16 (0 there))."""
    lib = _load()
    wb = np.ascontiguousarray(_bits(wk))
    Hkv, Dg, d3 = wb.shape
    d = d3 // 3
    sl = _i32(seqlens)
    B = sl.shape[0]
    st, kb, pt = _kv_struct(k_nope, page_table, page_size, B)
    assert kb.shape[1] == Hkv and kb.shape[3] == d
    co, si = _f32(rope_cos), _f32(rope_sin)
    bb, be = _i32(block_begin), _i32(block_end)
    if out is None:
        out = np.full((B, Hkv, nb_max, Dg), np.nan, dtype=np.float64)
    if out_bits is None:
        out_bits = np.zeros((B, Hkv, nb_max, Dg), dtype=np.uint16)
    rc = lib.oracle_kc_update(ctypes.byref(st), _ptr(wb), _ptr(co), _ptr(si), co.shape[0], _ptr(sl), _ptr(bb),
                              _ptr(be), B, Hkv, d, Dg, nb_max, block_size, _ptr(out), _ptr(out_bits))
    if rc != 0:
        raise ValueError(f"oracle_kc_update failed ({rc})")
    return out, out_bits


def sparse_decode_multi(q, kv: KVLayout, seqlens, block_idx, nblk, block_size: int, scale: float):
    """T new tokens per sequence in one step (Sec. 6.3 direction): q [B,T,Hq,d] bf16, the queries are
    the last T tokens of each sequence, causal among themselves, one block list per (sequence, kv
    head).  Returns (out [B,T,Hq,d] fp64, lse [B,T,Hq] fp64)."""
    lib = _load()
    qb = np.ascontiguousarray(_bits(q))
    B, T, Hq, d = qb.shape
    kb, vb = _bits(kv.k), _bits(kv.v)
    assert kb.shape == vb.shape and kb.strides == vb.strides and kb.shape[3] == d
    Hkv = kb.shape[1]
    st, _, pt = _kv_struct(kv.k, kv.page_table, kv.page_size, B)
    st.v = vb.ctypes.data
    sl, bi, nk = _i32(seqlens), _i32(block_idx), _i32(nblk)
    max_sel = bi.shape[2] if bi is not None else 0
    out = np.full((B, T, Hq, d), np.nan, dtype=np.float64)
    lse = np.full((B, T, Hq), np.nan, dtype=np.float64)
    rc = lib.oracle_sparse_decode_multi(_ptr(qb), ctypes.byref(st), _ptr(sl), _ptr(bi), _ptr(nk), max_sel, B, T,
                                        Hq, Hkv, d, block_size, ctypes.c_float(scale), _ptr(out), _ptr(lse), None)
    if rc != 0:
        raise ValueError("oracle_sparse_decode_multi: bad sizes")
    return out, lse


def attn_ground_truth(q, k, v, block_size: int, scale: float, seqlens=None):
    """Training-side ground truth of the AttnGate (Sec. 2.3) together with the dense causal
    attention it is pooled from.  q [B,T,Hq,d] bf16; k, v [B,Hkv,T,d] bf16 views (any strides on the
    first three dims); seqlens [B] or None.  Returns (out [B,T,Hq,d], lse [B,T,Hq],
    gt [B,Hkv,T,ceil(T/block_size)]) as fp64 arrays; every gt row of a real query sums to 1."""
    lib = _load()
    qb = np.ascontiguousarray(_bits(q))
    B, T, Hq, d = qb.shape
    kb, vb = _bits(k), _bits(v)
    assert kb.shape == vb.shape and kb.strides == vb.strides and kb.shape[0] == B and kb.shape[3] == d
    assert kb.shape[2] >= T
    Hkv = kb.shape[1]
    st, _, _ = _kv_struct(k, None, 0, B)
    st.v = vb.ctypes.data
    sl = _i32(seqlens)
    nb = (T + block_size - 1) // block_size
    out = np.full((B, T, Hq, d), np.nan, dtype=np.float64)
    lse = np.full((B, T, Hq), np.nan, dtype=np.float64)
    gt = np.full((B, Hkv, T, nb), np.nan, dtype=np.float64)
    rc = lib.oracle_attn_ground_truth(_ptr(qb), ctypes.byref(st), _ptr(sl), B, T, Hq, Hkv, d, block_size,
                                      ctypes.c_float(scale), _ptr(out), _ptr(lse), _ptr(gt))
    if rc != 0:
        raise ValueError("oracle_attn_ground_truth: bad sizes")
    return out, lse, gt
