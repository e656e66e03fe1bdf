"""ctypes binding of libseer.so.  Same names as the C entry points (minus the ``seer_``
prefix); every function only checks dtypes/devices, extracts pointers, strides and the
current HIP stream, and forwards.  There is no CPU fallback: if the library cannot be loaded
the import of a function's first use raises."""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libseer.so")
_lib = None

SELECT_TOPK = 0
SELECT_THRESHOLD = 1
SELECT_TOPP = 2
HINT_RAGGED_LISTS = 1
NOALLOC_SCRATCH_BYTES = 32 << 20
KNOB_DECODE_IMPL = 0
KNOB_DECODE_SPLITS = 1
KNOB_GATE_IMPL = 3
KERNEL_CLASSES = ("gate_score", "gate_select", "decode_split", "decode_merge", "stream_read", "gate_q", "kc_update",
                  "attn_fwd", "gt_finalize")


class SeerError(RuntimeError):
    def __init__(self, fn: str, status: int, text: str):
        super().__init__(f"{fn} failed: {text} (status {status})")
        self.status = status


class _KVLayout(ctypes.Structure):
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


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libseer.so (building it first only if it is not there)."""
    global _lib
    if _lib is not None:
        return _lib
    path = os.environ.get("SEER_LIB", _LIB_PATH)     # SEER_LIB: an alternative build of the same library
    if path == _LIB_PATH and not os.path.exists(_LIB_PATH):
        from . import build as _build
        _build.build()
    lib = ctypes.CDLL(path)
    c_int, c_i64, c_vp, c_sz, c_u32 = ctypes.c_int, ctypes.c_int64, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_uint32
    lib.seer_version.restype = c_int
    lib.seer_status_string.restype = ctypes.c_char_p
    lib.seer_status_string.argtypes = [c_int]
    lib.seer_gate_workspace_bytes.restype = c_int
    lib.seer_gate_workspace_bytes.argtypes = [c_int, c_int, c_int, ctypes.POINTER(c_sz)]
    lib.seer_decode_workspace_bytes.restype = c_int
    lib.seer_decode_workspace_bytes.argtypes = [c_int, c_int, c_int, c_int, c_int, ctypes.POINTER(c_sz)]
    lib.seer_decode_plan.restype = c_int
    lib.seer_decode_plan.argtypes = [c_int, c_int, c_int, c_int, c_u32, ctypes.POINTER(c_int), ctypes.POINTER(c_int)]
    lib.seer_gate_select.restype = c_int
    lib.seer_gate_select.argtypes = [c_vp, c_vp, c_i64, c_i64, c_i64, c_vp, c_int, c_int, c_int, c_int,
                                     c_int, c_int, ctypes.c_int32, c_vp, ctypes.c_double, c_vp, c_vp,
                                     c_int, c_vp, c_sz, c_u32, c_vp]
    lib.seer_sparse_decode.restype = c_int
    lib.seer_sparse_decode.argtypes = [c_vp, ctypes.POINTER(_KVLayout), c_vp, c_vp, c_vp, c_int, c_int,
                                       c_int, c_int, c_int, c_int, ctypes.c_float, c_vp, c_int, c_vp,
                                       c_vp, c_sz, c_u32, c_vp]
    lib.seer_sparse_decode_noalloc.restype = c_int
    lib.seer_sparse_decode_noalloc.argtypes = [c_vp, ctypes.POINTER(_KVLayout), c_vp, c_vp, c_vp, c_int, c_int,
                                               c_int, c_int, c_int, c_int, ctypes.c_float, c_vp, c_int, c_vp,
                                               c_u32, c_vp]
    lib.seer_sparse_decode_multi.restype = c_int
    lib.seer_sparse_decode_multi.argtypes = [c_vp, ctypes.POINTER(_KVLayout), c_vp, c_vp, c_vp, c_int, c_int, c_int,
                                             c_int, c_int, c_int, c_int, ctypes.c_float, c_vp, c_int, c_vp,
                                             c_vp, c_sz, c_u32, c_vp]
    lib.seer_dense_decode.restype = c_int
    lib.seer_dense_decode.argtypes = [c_vp, ctypes.POINTER(_KVLayout), c_vp, c_int, c_int, c_int, c_int,
                                      c_int, c_int, ctypes.c_float, c_vp, c_int, c_vp, c_vp, c_sz, c_u32, c_vp]
    lib.seer_gate_q.restype = c_int
    lib.seer_gate_q.argtypes = [c_vp, c_vp, c_vp, c_vp, c_int, c_vp, c_int, c_int, c_int, c_int, c_int, c_vp, c_vp]
    lib.seer_gate_select_q.restype = c_int
    lib.seer_gate_select_q.argtypes = [c_vp, c_vp, c_vp, c_vp, c_int, c_vp, c_i64, c_i64, c_i64, c_vp, c_int, c_int, c_int,
                                       c_int, c_int, c_int, c_int, c_int, ctypes.c_int32, c_vp, ctypes.c_double, c_vp,
                                       c_vp, c_int, c_vp, c_vp, c_sz, c_u32, c_vp]
    lib.seer_kc_update.restype = c_int
    lib.seer_kc_update.argtypes = [ctypes.POINTER(_KVLayout), c_vp, c_vp, c_vp, c_int, c_vp, c_vp, c_vp, c_int, c_int,
                                   c_int, c_int, c_int, c_int, c_int, c_vp, c_i64, c_i64, c_i64, c_vp]
    lib.seer_attn_ground_truth_workspace_bytes.restype = c_int
    lib.seer_attn_ground_truth_workspace_bytes.argtypes = [c_int] * 6 + [ctypes.POINTER(c_sz)]
    lib.seer_attn_ground_truth.restype = c_int
    lib.seer_attn_ground_truth.argtypes = [c_vp, ctypes.POINTER(_KVLayout), c_vp, c_int, c_int, c_int, c_int, c_int,
                                           c_int, ctypes.c_float, c_vp, c_int, c_vp, c_vp, c_vp, c_sz, c_vp]
    lib.seer_hbm_read_probe.restype = c_int
    lib.seer_hbm_read_probe.argtypes = [c_vp, c_sz, c_vp, c_vp]
    lib.seer_set_knob.restype = c_int
    lib.seer_set_knob.argtypes = [c_int, c_int]
    lib.seer_get_knob.restype = c_int
    lib.seer_get_knob.argtypes = [c_int, ctypes.POINTER(c_int)]
    lib.seer_profile_enable.restype = c_int
    lib.seer_profile_enable.argtypes = [c_int]
    lib.seer_profile_reset.restype = c_int
    lib.seer_profile_durations.restype = c_int
    lib.seer_profile_durations.argtypes = [c_int, ctypes.POINTER(ctypes.c_double), c_int, ctypes.POINTER(c_int)]
    _lib = lib
    return lib


def _check(fn: str, status: int):
    if status != 0:
        raise SeerError(fn, status, load_library().seer_status_string(status).decode())


def version() -> int:
    return int(load_library().seer_version())


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream() -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _want(t: torch.Tensor, dtype, name: str):
    if t.dtype != dtype:
        raise TypeError(f"{name}: expected {dtype}, got {t.dtype}")
    if not t.is_cuda:
        raise ValueError(f"{name}: expected a device tensor")


def gate_workspace_bytes(B: int, Hkv: int, nb_max: int) -> int:
    n = ctypes.c_size_t(0)
    _check("seer_gate_workspace_bytes", load_library().seer_gate_workspace_bytes(B, Hkv, nb_max, ctypes.byref(n)))
    return int(n.value)


def decode_workspace_bytes(B: int, Hq: int, Hkv: int, d: int, max_blocks: int) -> int:
    n = ctypes.c_size_t(0)
    _check("seer_decode_workspace_bytes",
           load_library().seer_decode_workspace_bytes(B, Hq, Hkv, d, max_blocks, ctypes.byref(n)))
    return int(n.value)


def _hints(ragged: bool) -> int:
    return HINT_RAGGED_LISTS if ragged else 0


def decode_plan(B: int, Hkv: int, max_blocks: int, block_size: int, ragged: bool = False):
    """seer_decode_plan: (num_splits, blocks_per_split) the decode calls will use for these sizes."""
    ns, per = ctypes.c_int(0), ctypes.c_int(0)
    _check("seer_decode_plan",
           load_library().seer_decode_plan(B, Hkv, max_blocks, block_size, _hints(ragged), ctypes.byref(ns),
                                           ctypes.byref(per)))
    return int(ns.value), int(per.value)


def _workspace(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)


def gate_select(q_gate: torch.Tensor, kc_cache: torch.Tensor, seqlens: torch.Tensor, block_size: int, *,
                mode: int = SELECT_TOPK, budget_tokens: int = 0, budget_blocks: Optional[torch.Tensor] = None,
                threshold: float = 0.0, max_sel: int, block_idx: Optional[torch.Tensor] = None,
                nblk: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                ragged: bool = False):
    """seer_gate_select.  q_gate [B,Hkv,Dg] bf16, kc_cache [B,Hkv,nb_max,Dg] bf16 (last dim
    contiguous), seqlens [B] int32.  Returns (block_idx [B,Hkv,max_sel] int32, nblk [B,Hkv] int32)."""
    lib = load_library()
    _want(q_gate, torch.bfloat16, "q_gate"); _want(kc_cache, torch.bfloat16, "kc_cache")
    _want(seqlens, torch.int32, "seqlens")
    B, Hkv, Dg = q_gate.shape
    if kc_cache.dim() != 4 or kc_cache.shape[0] != B or kc_cache.shape[1] != Hkv or kc_cache.shape[3] != Dg:
        raise ValueError("kc_cache must be [B,Hkv,nb_max,Dg]")
    if kc_cache.stride(3) != 1 or not q_gate.is_contiguous() or not seqlens.is_contiguous():
        raise ValueError("q_gate/seqlens must be contiguous and kc_cache contiguous in its last dim")
    nb_max = kc_cache.shape[2]
    dev = q_gate.device
    if block_idx is None:
        block_idx = torch.empty(B, Hkv, max_sel, dtype=torch.int32, device=dev)
    if nblk is None:
        nblk = torch.empty(B, Hkv, dtype=torch.int32, device=dev)
    _want(block_idx, torch.int32, "block_idx"); _want(nblk, torch.int32, "nblk")
    if budget_blocks is not None:
        _want(budget_blocks, torch.int32, "budget_blocks")
    if workspace is None:
        workspace = _workspace(gate_workspace_bytes(B, Hkv, nb_max), dev)
    st = lib.seer_gate_select(_ptr(q_gate), _ptr(kc_cache), kc_cache.stride(0), kc_cache.stride(1),
                              kc_cache.stride(2), _ptr(seqlens), B, Hkv, Dg, nb_max, block_size, mode,
                              int(budget_tokens), _ptr(budget_blocks), float(threshold), _ptr(block_idx),
                              _ptr(nblk), max_sel, _ptr(workspace), workspace.numel(), _hints(ragged), _stream())
    _check("seer_gate_select", st)
    return block_idx, nblk


def _layout(k: torch.Tensor, v: torch.Tensor, page_table: Optional[torch.Tensor], page_size: int) -> _KVLayout:
    _want(k, torch.bfloat16, "k"); _want(v, torch.bfloat16, "v")
    if k.dim() != 4 or k.shape != v.shape or k.stride() != v.stride() or k.stride(3) != 1:
        raise ValueError("k and v must be 4-D, same shape and strides, contiguous in the last dim")
    lay = _KVLayout()
    lay.k = k.data_ptr()
    lay.v = v.data_ptr()
    lay.stride_seq, lay.stride_head, lay.stride_token = k.stride(0), k.stride(1), k.stride(2)
    if page_table is not None:
        _want(page_table, torch.int32, "page_table")
        if not page_table.is_contiguous():
            raise ValueError("page_table must be contiguous")
        lay.page_table = page_table.data_ptr()
        lay.max_pages = page_table.shape[1]
        lay.page_size = page_size
    else:
        lay.page_table = None
        lay.max_pages = 0
        lay.page_size = 0
    return lay


def _decode_out(q, out, lse, out_dtype):
    B, Hq, d = q.shape
    if out is None:
        out = torch.empty(B, Hq, d, dtype=out_dtype, device=q.device)
    if out.dtype not in (torch.bfloat16, torch.float32) or not out.is_contiguous():
        raise TypeError("out must be contiguous bf16 or fp32")
    if lse is None:
        lse = torch.empty(B, Hq, dtype=torch.float32, device=q.device)
    _want(lse, torch.float32, "lse")
    return out, lse


def sparse_decode(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, seqlens: torch.Tensor,
                  block_idx: torch.Tensor, nblk: torch.Tensor, block_size: int, scale: float, *,
                  page_table: Optional[torch.Tensor] = None, page_size: int = 0,
                  out: Optional[torch.Tensor] = None, lse: Optional[torch.Tensor] = None,
                  out_dtype=torch.bfloat16, workspace: Optional[torch.Tensor] = None, ragged: bool = False):
    """seer_sparse_decode.  q [B,Hq,d] bf16; k/v contiguous [B,Hkv,S,d] views or paged pools
    [n_pages,Hkv,page,d] with page_table [B,max_pages]; block_idx [B,Hkv,max_sel], nblk [B,Hkv]
    int32.  Returns (out [B,Hq,d], lse [B,Hq] fp32)."""
    lib = load_library()
    _want(q, torch.bfloat16, "q"); _want(seqlens, torch.int32, "seqlens")
    _want(block_idx, torch.int32, "block_idx"); _want(nblk, torch.int32, "nblk")
    if not (q.is_contiguous() and block_idx.is_contiguous() and nblk.is_contiguous()):
        raise ValueError("q, block_idx and nblk must be contiguous")
    B, Hq, d = q.shape
    Hkv = k.shape[1]
    max_sel = block_idx.shape[2]
    lay = _layout(k, v, page_table, page_size)
    out, lse = _decode_out(q, out, lse, out_dtype)
    if workspace is None:
        workspace = _workspace(decode_workspace_bytes(B, Hq, Hkv, d, max_sel), q.device)
    st = lib.seer_sparse_decode(_ptr(q), ctypes.byref(lay), _ptr(seqlens), _ptr(block_idx), _ptr(nblk),
                                max_sel, B, Hq, Hkv, d, block_size, ctypes.c_float(scale), _ptr(out),
                                0 if out.dtype == torch.bfloat16 else 1, _ptr(lse), _ptr(workspace),
                                workspace.numel(), _hints(ragged), _stream())
    _check("seer_sparse_decode", st)
    return out, lse


def sparse_decode_noalloc(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, seqlens: torch.Tensor,
                          block_idx: torch.Tensor, nblk: torch.Tensor, block_size: int, scale: float, *,
                          out: torch.Tensor, lse: torch.Tensor, page_table: Optional[torch.Tensor] = None,
                          page_size: int = 0, ragged: bool = False):
    """seer_sparse_decode_noalloc: seer_sparse_decode on the library's built-in scratch array.  Neither
    the library nor this wrapper allocates: out [B,Hq,d] (bf16 or fp32) and lse [B,Hq] fp32 are the
    caller's.  Returns (out, lse)."""
    lib = load_library()
    _want(q, torch.bfloat16, "q"); _want(seqlens, torch.int32, "seqlens")
    _want(block_idx, torch.int32, "block_idx"); _want(nblk, torch.int32, "nblk"); _want(lse, torch.float32, "lse")
    if not (q.is_contiguous() and block_idx.is_contiguous() and nblk.is_contiguous() and out.is_contiguous()
            and lse.is_contiguous()):
        raise ValueError("q, block_idx, nblk, out and lse must be contiguous")
    if out.dtype not in (torch.bfloat16, torch.float32) or not out.is_cuda:
        raise TypeError("out must be a bf16 or fp32 device tensor")
    B, Hq, d = q.shape
    if tuple(out.shape) != (B, Hq, d) or tuple(lse.shape) != (B, Hq):
        raise ValueError("out must be [B,Hq,d] and lse [B,Hq]")
    Hkv = k.shape[1]
    max_sel = block_idx.shape[2]
    lay = _layout(k, v, page_table, page_size)
    st = lib.seer_sparse_decode_noalloc(_ptr(q), ctypes.byref(lay), _ptr(seqlens), _ptr(block_idx), _ptr(nblk),
                                        max_sel, B, Hq, Hkv, d, block_size, ctypes.c_float(scale), _ptr(out),
                                        0 if out.dtype == torch.bfloat16 else 1, _ptr(lse), _hints(ragged),
                                        _stream())
    _check("seer_sparse_decode_noalloc", st)
    return out, lse


def sparse_decode_multi(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, seqlens: torch.Tensor,
                        block_idx: torch.Tensor, nblk: torch.Tensor, block_size: int, scale: float, *,
                        page_table: Optional[torch.Tensor] = None, page_size: int = 0,
                        out: Optional[torch.Tensor] = None, lse: Optional[torch.Tensor] = None,
                        out_dtype=torch.bfloat16, workspace: Optional[torch.Tensor] = None, ragged: bool = False):
    """seer_sparse_decode_multi.  q [B,q_len,Hq,d] bf16 (the last q_len tokens of each sequence).
    Returns (out [B,q_len,Hq,d], lse [B,q_len,Hq] fp32)."""
    lib = load_library()
    _want(q, torch.bfloat16, "q"); _want(seqlens, torch.int32, "seqlens")
    _want(block_idx, torch.int32, "block_idx"); _want(nblk, torch.int32, "nblk")
    if q.dim() != 4 or not (q.is_contiguous() and block_idx.is_contiguous() and nblk.is_contiguous()):
        raise ValueError("q must be contiguous [B,q_len,Hq,d]; block_idx and nblk contiguous")
    B, T, Hq, d = q.shape
    Hkv = k.shape[1]
    max_sel = block_idx.shape[2]
    lay = _layout(k, v, page_table, page_size)
    if out is None:
        out = torch.empty(B, T, Hq, d, dtype=out_dtype, device=q.device)
    if lse is None:
        lse = torch.empty(B, T, Hq, dtype=torch.float32, device=q.device)
    if workspace is None:
        workspace = _workspace(decode_workspace_bytes(B, Hq * T, Hkv, d, max_sel), q.device)
    st = lib.seer_sparse_decode_multi(_ptr(q), ctypes.byref(lay), _ptr(seqlens), _ptr(block_idx), _ptr(nblk),
                                      max_sel, B, T, Hq, Hkv, d, block_size, ctypes.c_float(scale), _ptr(out),
                                      0 if out.dtype == torch.bfloat16 else 1, _ptr(lse), _ptr(workspace),
                                      workspace.numel(), _hints(ragged), _stream())
    _check("seer_sparse_decode_multi", st)
    return out, lse


def attn_ground_truth_workspace_bytes(B: int, T: int, Hq: int, Hkv: int, d: int, block_size: int) -> int:
    n = ctypes.c_size_t(0)
    _check("seer_attn_ground_truth_workspace_bytes",
           load_library().seer_attn_ground_truth_workspace_bytes(B, T, Hq, Hkv, d, block_size, ctypes.byref(n)))
    return int(n.value)


def attn_ground_truth(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, block_size: int, scale: float, *,
                      seqlens: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None,
                      lse: Optional[torch.Tensor] = None, gt: Optional[torch.Tensor] = None,
                      out_dtype=torch.bfloat16, workspace: Optional[torch.Tensor] = None):
    """seer_attn_ground_truth.  q [B,T,Hq,d] bf16 contiguous; k/v [B,Hkv,>=T,d] bf16 views; seqlens [B]
    int32 or None.  Returns (out [B,T,Hq,d], lse [B,T,Hq] fp32, gt [B,Hkv,T,ceil(T/block_size)] fp32)."""
    lib = load_library()
    _want(q, torch.bfloat16, "q")
    if q.dim() != 4 or not q.is_contiguous():
        raise ValueError("q must be contiguous [B,T,Hq,d]")
    B, T, Hq, d = q.shape
    Hkv = k.shape[1]
    if k.shape[0] != B or k.shape[2] < T:
        raise ValueError("k/v must hold at least T tokens for each of the B sequences")
    lay = _layout(k, v, None, 0)
    if seqlens is not None:
        _want(seqlens, torch.int32, "seqlens")
        if not seqlens.is_contiguous() or seqlens.numel() != B:
            raise ValueError("seqlens must be contiguous [B]")
    nb = (T + block_size - 1) // block_size
    if out is None:
        out = torch.empty(B, T, Hq, d, dtype=out_dtype, device=q.device)
    if out.dtype not in (torch.bfloat16, torch.float32) or not out.is_contiguous():
        raise TypeError("out must be contiguous bf16 or fp32")
    if lse is None:
        lse = torch.empty(B, T, Hq, dtype=torch.float32, device=q.device)
    if gt is None:
        gt = torch.empty(B, Hkv, T, nb, dtype=torch.float32, device=q.device)
    _want(lse, torch.float32, "lse"); _want(gt, torch.float32, "gt")
    if not (lse.is_contiguous() and gt.is_contiguous()) or gt.shape != (B, Hkv, T, nb):
        raise ValueError("lse and gt must be contiguous; gt [B,Hkv,T,nb]")
    if workspace is None:
        workspace = _workspace(attn_ground_truth_workspace_bytes(B, T, Hq, Hkv, d, block_size), q.device)
    st = lib.seer_attn_ground_truth(_ptr(q), ctypes.byref(lay), _ptr(seqlens), B, T, Hq, Hkv, d, block_size,
                                    ctypes.c_float(scale), _ptr(out), 0 if out.dtype == torch.bfloat16 else 1,
                                    _ptr(lse), _ptr(gt), _ptr(workspace), workspace.numel(), _stream())
    _check("seer_attn_ground_truth", st)
    return out, lse, gt


def dense_decode(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, seqlens: torch.Tensor, max_blocks: int,
                 block_size: int, scale: float, *, page_table: Optional[torch.Tensor] = None,
                 page_size: int = 0, out: Optional[torch.Tensor] = None, lse: Optional[torch.Tensor] = None,
                 out_dtype=torch.bfloat16, workspace: Optional[torch.Tensor] = None, ragged: bool = False):
    """seer_dense_decode: the same kernels over every block of every sequence."""
    lib = load_library()
    _want(q, torch.bfloat16, "q"); _want(seqlens, torch.int32, "seqlens")
    if not q.is_contiguous():
        raise ValueError("q must be contiguous")
    B, Hq, d = q.shape
    Hkv = k.shape[1]
    lay = _layout(k, v, page_table, page_size)
    out, lse = _decode_out(q, out, lse, out_dtype)
    if workspace is None:
        workspace = _workspace(decode_workspace_bytes(B, Hq, Hkv, d, max_blocks), q.device)
    st = lib.seer_dense_decode(_ptr(q), ctypes.byref(lay), _ptr(seqlens), max_blocks, B, Hq, Hkv, d,
                               block_size, ctypes.c_float(scale), _ptr(out),
                               0 if out.dtype == torch.bfloat16 else 1, _ptr(lse), _ptr(workspace),
                               workspace.numel(), _hints(ragged), _stream())
    _check("seer_dense_decode", st)
    return out, lse


def _rope(rope_cos, rope_sin, Dg):
    _want(rope_cos, torch.float32, "rope_cos"); _want(rope_sin, torch.float32, "rope_sin")
    if rope_cos.shape != rope_sin.shape or rope_cos.dim() != 2 or rope_cos.shape[1] != Dg // 2 or \
            not (rope_cos.is_contiguous() and rope_sin.is_contiguous()):
        raise ValueError("rope tables must be contiguous [n_pos, Dg/2] fp32")
    return rope_cos.shape[0]


def gate_q(q_nope: torch.Tensor, wq: torch.Tensor, rope_cos: torch.Tensor, rope_sin: torch.Tensor,
           seqlens: torch.Tensor, *, q_gate: Optional[torch.Tensor] = None):
    """seer_gate_q.  q_nope [B,Hq,d] bf16, wq [Hkv,Dg,g*d] bf16, rope tables [n_pos,Dg/2] fp32.
    Returns q_gate [B,Hkv,Dg] bf16."""
    lib = load_library()
    _want(q_nope, torch.bfloat16, "q_nope"); _want(wq, torch.bfloat16, "wq"); _want(seqlens, torch.int32, "seqlens")
    if not (q_nope.is_contiguous() and wq.is_contiguous()):
        raise ValueError("q_nope and wq must be contiguous")
    B, Hq, d = q_nope.shape
    Hkv, Dg, gd = wq.shape
    if Hq % Hkv or gd != (Hq // Hkv) * d:
        raise ValueError("wq must be [Hkv, Dg, (Hq/Hkv)*d]")
    n_pos = _rope(rope_cos, rope_sin, Dg)
    if q_gate is None:
        q_gate = torch.empty(B, Hkv, Dg, dtype=torch.bfloat16, device=q_nope.device)
    _want(q_gate, torch.bfloat16, "q_gate")
    st = lib.seer_gate_q(_ptr(q_nope), _ptr(wq), _ptr(rope_cos), _ptr(rope_sin), n_pos, _ptr(seqlens), B, Hq, Hkv,
                         d, Dg, _ptr(q_gate), _stream())
    _check("seer_gate_q", st)
    return q_gate


def gate_select_q(q_nope: torch.Tensor, wq: torch.Tensor, rope_cos: torch.Tensor, rope_sin: torch.Tensor,
                  kc_cache: torch.Tensor, seqlens: torch.Tensor, block_size: int, *, mode: int = SELECT_TOPK,
                  budget_tokens: int = 0, budget_blocks: Optional[torch.Tensor] = None, threshold: float = 0.0,
                  max_sel: int, block_idx: Optional[torch.Tensor] = None, nblk: Optional[torch.Tensor] = None,
                  q_gate: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None, ragged: bool = False):
    """seer_gate_select_q: gate query from the pre-RoPE queries (q_nope [B,Hq,d], wq [Hkv,Dg,g*d], rope
    tables) and block selection against kc_cache in one call.  q_gate (bf16 [B,Hkv,Dg]) receives the gate
    query when given.  Returns (block_idx, nblk)."""
    lib = load_library()
    _want(q_nope, torch.bfloat16, "q_nope"); _want(wq, torch.bfloat16, "wq"); _want(kc_cache, torch.bfloat16, "kc_cache")
    _want(seqlens, torch.int32, "seqlens")
    if not (q_nope.is_contiguous() and wq.is_contiguous() and seqlens.is_contiguous()):
        raise ValueError("q_nope, wq and seqlens must be contiguous")
    B, Hq, d = q_nope.shape
    Hkv, Dg, gd = wq.shape
    if Hq % Hkv or gd != (Hq // Hkv) * d:
        raise ValueError("wq must be [Hkv, Dg, (Hq/Hkv)*d]")
    if kc_cache.dim() != 4 or kc_cache.shape[0] != B or kc_cache.shape[1] != Hkv or kc_cache.shape[3] != Dg or \
            kc_cache.stride(3) != 1:
        raise ValueError("kc_cache must be [B,Hkv,nb_max,Dg], contiguous in its last dim")
    n_pos = _rope(rope_cos, rope_sin, Dg)
    nb_max = kc_cache.shape[2]
    dev = q_nope.device
    if block_idx is None:
        block_idx = torch.empty(B, Hkv, max_sel, dtype=torch.int32, device=dev)
    if nblk is None:
        nblk = torch.empty(B, Hkv, dtype=torch.int32, device=dev)
    _want(block_idx, torch.int32, "block_idx"); _want(nblk, torch.int32, "nblk")
    if budget_blocks is not None:
        _want(budget_blocks, torch.int32, "budget_blocks")
    if q_gate is not None:
        _want(q_gate, torch.bfloat16, "q_gate")
        if tuple(q_gate.shape) != (B, Hkv, Dg) or not q_gate.is_contiguous():
            raise ValueError("q_gate must be contiguous [B,Hkv,Dg]")
    if workspace is None:
        workspace = _workspace(gate_workspace_bytes(B, Hkv, nb_max), dev)
    st = lib.seer_gate_select_q(_ptr(q_nope), _ptr(wq), _ptr(rope_cos), _ptr(rope_sin), n_pos, _ptr(kc_cache),
                                kc_cache.stride(0), kc_cache.stride(1), kc_cache.stride(2), _ptr(seqlens), B, Hq, Hkv, d,
                                Dg, nb_max, block_size, mode, int(budget_tokens), _ptr(budget_blocks), float(threshold),
                                _ptr(block_idx), _ptr(nblk), max_sel, _ptr(q_gate), _ptr(workspace), workspace.numel(),
                                _hints(ragged), _stream())
    _check("seer_gate_select_q", st)
    return block_idx, nblk


def kc_update(k_nope: torch.Tensor, wk: torch.Tensor, rope_cos: torch.Tensor, rope_sin: torch.Tensor,
              seqlens: torch.Tensor, block_size: int, kc_cache: torch.Tensor, *, max_blocks: Optional[int] = None,
              block_begin: Optional[torch.Tensor] = None, block_end: Optional[torch.Tensor] = None,
              page_table: Optional[torch.Tensor] = None, page_size: int = 0):
    """seer_kc_update.  k_nope: pre-RoPE keys in KV-cache layout; wk [Hkv,Dg,3d] bf16;
    kc_cache [B,Hkv,nb_max,Dg] bf16 (updated in place, last dim contiguous)."""
    lib = load_library()
    _want(wk, torch.bfloat16, "wk"); _want(seqlens, torch.int32, "seqlens"); _want(kc_cache, torch.bfloat16, "kc_cache")
    if not wk.is_contiguous() or kc_cache.dim() != 4 or kc_cache.stride(3) != 1:
        raise ValueError("wk must be contiguous and kc_cache [B,Hkv,nb_max,Dg] contiguous in its last dim")
    lay = _layout(k_nope, k_nope, page_table, page_size)
    B, Hkv, nb_max, Dg = kc_cache.shape
    d = k_nope.shape[3]
    if wk.shape != (Hkv, Dg, 3 * d):
        raise ValueError("wk must be [Hkv, Dg, 3*d]")
    n_pos = _rope(rope_cos, rope_sin, Dg)
    for name, t in (("block_begin", block_begin), ("block_end", block_end)):
        if t is not None:
            _want(t, torch.int32, name)
    st = lib.seer_kc_update(ctypes.byref(lay), _ptr(wk), _ptr(rope_cos), _ptr(rope_sin), n_pos, _ptr(seqlens),
                            _ptr(block_begin), _ptr(block_end), max_blocks or nb_max, B, Hkv, d, Dg, nb_max,
                            block_size, _ptr(kc_cache), kc_cache.stride(0), kc_cache.stride(1), kc_cache.stride(2),
                            _stream())
    _check("seer_kc_update", st)
    return kc_cache


def hbm_read_probe(src: torch.Tensor, sink: torch.Tensor):
    """seer_hbm_read_probe: stream-read all bytes of `src` (contiguous device tensor)."""
    if not (src.is_cuda and src.is_contiguous() and sink.is_cuda and sink.numel() * sink.element_size() >= 16):
        raise ValueError("src must be a contiguous device tensor and sink hold 16 bytes")
    nbytes = src.numel() * src.element_size() // 16 * 16
    _check("seer_hbm_read_probe", load_library().seer_hbm_read_probe(_ptr(src), nbytes, _ptr(sink), _stream()))
    return nbytes


def set_knob(knob: int, value: int):
    _check("seer_set_knob", load_library().seer_set_knob(knob, value))


def get_knob(knob: int) -> int:
    v = ctypes.c_int(0)
    _check("seer_get_knob", load_library().seer_get_knob(knob, ctypes.byref(v)))
    return int(v.value)


def profile_enable(on: bool):
    _check("seer_profile_enable", load_library().seer_profile_enable(1 if on else 0))


def profile_reset():
    _check("seer_profile_reset", load_library().seer_profile_reset())


def profile_durations(which: int):
    """seer_profile_durations: the duration in ms of every launch of one kernel class since the last reset."""
    lib = load_library()
    n = ctypes.c_int(0)
    _check("seer_profile_durations", lib.seer_profile_durations(which, None, 0, ctypes.byref(n)))
    buf = (ctypes.c_double * max(n.value, 1))()
    _check("seer_profile_durations", lib.seer_profile_durations(which, buf, n.value, ctypes.byref(n)))
    return [float(buf[i]) for i in range(n.value)]


def profile_read(which: int):
    """(launches, total_ms) of one kernel class since the last reset."""
    d = profile_durations(which)
    return len(d), float(sum(d))
