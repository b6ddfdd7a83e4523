"""ctypes binding of libinstattn.so: argument marshalling only.

Same entry points as include/instattn.h, taking torch tensors (device memory and
streams come from PyTorch; every step of the path runs in the library's HIP
kernels).  There is no fallback: if the library has not been built, loading
raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libinstattn.so")

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_RUNTIME = range(5)
KV_CONTIGUOUS, KV_PAGED = 0, 1
F16, F32 = 0, 1


class KvDesc(ctypes.Structure):
    """Mirror of instattn_kv_desc."""
    _fields_ = [
        ("k", ctypes.c_void_p), ("v", ctypes.c_void_p),
        ("layout", ctypes.c_int32), ("page_size", ctypes.c_int32),
        ("stride_b", ctypes.c_int64), ("stride_h", ctypes.c_int64), ("stride_t", ctypes.c_int64),
        ("capacity", ctypes.c_int32), ("max_pages_per_seq", ctypes.c_int32),
        ("num_pages", ctypes.c_int32), ("reserved", ctypes.c_int32),
        ("page_table", ctypes.c_void_p),
    ]


class SparfAux(ctypes.Structure):
    """Mirror of instattn_sparf_aux."""
    _fields_ = [
        ("kt", ctypes.c_void_p),
        ("stride_b", ctypes.c_int64), ("stride_h", ctypes.c_int64), ("stride_d", ctypes.c_int64),
        ("vsum", ctypes.c_void_p),
        ("capacity", ctypes.c_int32), ("page_size", ctypes.c_int32),
        ("page_table", ctypes.c_void_p),
        ("max_pages_per_seq", ctypes.c_int32), ("num_pages", ctypes.c_int32),
    ]


class InstattnError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: %s (status %d)" % (where, status_string(status), status))


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded library.  Raises if it has not been built (no fallback path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                "libinstattn.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
        L = ctypes.CDLL(LIB_PATH)
        vp, i, sz, f = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t, ctypes.c_float
        L.instattn_version.restype = i
        L.instattn_version.argtypes = []
        L.instattn_status_string.restype = ctypes.c_char_p
        L.instattn_status_string.argtypes = [i]
        L.instattn_set_option.restype = i
        L.instattn_set_option.argtypes = [ctypes.c_char_p, i]
        L.instattn_get_option.restype = i
        L.instattn_get_option.argtypes = [ctypes.c_char_p, ctypes.POINTER(i)]
        L.instattn_decode_launches.restype = i
        L.instattn_decode_launches.argtypes = [i, i, i, i, i, i, i, ctypes.POINTER(ctypes.c_int32)]
        L.instattn_kv_append.restype = i
        L.instattn_kv_append.argtypes = [ctypes.POINTER(KvDesc), vp, vp, vp, i, i, i, vp]
        L.instattn_kv_write.restype = i
        L.instattn_kv_write.argtypes = [ctypes.POINTER(KvDesc), vp, vp, vp, vp, i, i, i, i, vp]
        L.instattn_decode_plan.restype = i
        L.instattn_decode_plan.argtypes = [i, i, i, i, i, ctypes.POINTER(i), ctypes.POINTER(i)]
        L.instattn_decode_workspace_size.restype = sz
        L.instattn_decode_workspace_size.argtypes = [i, i, i, i, i]
        decode_args = [vp, ctypes.POINTER(KvDesc), vp, i, i, i, i, f, vp, i, vp, vp, sz, i, vp]
        L.instattn_decode.restype = i
        L.instattn_decode.argtypes = decode_args
        L.instattn_decode_partial.restype = i
        L.instattn_decode_partial.argtypes = decode_args
        L.instattn_append_decode.restype = i
        L.instattn_append_decode.argtypes = [vp, vp, vp] + decode_args[1:]
        L.instattn_append_decode_partial.restype = i
        L.instattn_append_decode_partial.argtypes = [vp, vp, vp] + decode_args[1:]
        L.instattn_decode_static.restype = i
        L.instattn_decode_static.argtypes = [vp, ctypes.POINTER(KvDesc), vp, i, i, i, i, f, vp, i, vp, i, vp]
        L.instattn_decode_merge.restype = i
        L.instattn_decode_merge.argtypes = [vp, i, i, i, i, i, vp, i, vp, vp, sz, i, vp]
        pk, pa = ctypes.POINTER(KvDesc), ctypes.POINTER(SparfAux)
        L.instattn_sparf_build.restype = i
        L.instattn_sparf_build.argtypes = [pk, pa, vp, i, i, i, vp, sz, vp]
        L.instattn_sparf_build_workspace_size.restype = sz
        L.instattn_sparf_build_workspace_size.argtypes = [i, i, i]
        L.instattn_sparf_append.restype = i
        L.instattn_sparf_append.argtypes = [pk, pa, vp, vp, vp, i, i, i, vp]
        L.instattn_sparf_plan.restype = i
        L.instattn_sparf_plan.argtypes = [i, i, i, i, i, i, i, ctypes.POINTER(ctypes.c_int32)]
        L.instattn_sparf_workspace_size.restype = sz
        L.instattn_sparf_workspace_size.argtypes = [i, i, i, i, i]
        L.instattn_sparf_append_decode.restype = i
        L.instattn_sparf_append_decode.argtypes = [vp, vp, vp, pk, pa, vp, i, i, i, i, f, i, i, i, vp, i, vp, vp,
                                                   vp, sz, i, vp]
        L.instattn_sparf_decode.restype = i
        L.instattn_sparf_decode.argtypes = [vp, pk, pa, vp, i, i, i, i, f, i, i, i, vp, i, vp, vp,
                                            vp, sz, i, vp]
        L.instattn_probe_read.restype = i
        L.instattn_probe_read.argtypes = [vp, sz, vp, vp]
        L.instattn_probe_copy.restype = i
        L.instattn_probe_copy.argtypes = [vp, vp, sz, vp]
        L.instattn_probe_read_columns.restype = i
        L.instattn_probe_read_columns.argtypes = [vp, sz, sz, i, i, i, i, vp, vp]
        _lib = L
    return _lib


def version() -> int:
    return lib().instattn_version()


def status_string(status: int) -> str:
    return lib().instattn_status_string(int(status)).decode()


OPTIONS = ("INSTATTN_CHUNK", "INSTATTN_ROTATE", "INSTATTN_COMPACT", "INSTATTN_MHA_RING", "INSTATTN_SPARF_DISTRIBUTED",
           "INSTATTN_SPARF_THREE_LAUNCHES", "INSTATTN_SPARF_WIDE", "INSTATTN_SPARF_SPLIT_TAIL")


def set_option(name: str, value: Optional[int]) -> None:
    """Force one of the host's choices (None or a negative value: hand it back)."""
    _check(lib().instattn_set_option(name.encode(), -1 if value is None else int(value)),
           "instattn_set_option")


def get_option(name: str) -> int:
    v = ctypes.c_int(0)
    _check(lib().instattn_get_option(name.encode(), ctypes.byref(v)), "instattn_get_option")
    return v.value


def _check(status: int, where: str) -> None:
    if status != OK:
        raise InstattnError(status, where)


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _p(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def kv_desc(k_cache: torch.Tensor, v_cache: torch.Tensor,
            page_table: Optional[torch.Tensor] = None) -> KvDesc:
    """Descriptor for [B, Hkv, capacity, D] caches or [num_pages, Hkv, page_size, D] pools."""
    assert k_cache.dtype == torch.float16 and v_cache.dtype == torch.float16
    assert k_cache.shape == v_cache.shape and k_cache.stride() == v_cache.stride()
    assert k_cache.stride(3) == 1
    d = KvDesc()
    d.k, d.v = k_cache.data_ptr(), v_cache.data_ptr()
    d.stride_b, d.stride_h, d.stride_t = k_cache.stride(0), k_cache.stride(1), k_cache.stride(2)
    d.reserved = 0
    if page_table is None:
        d.layout = KV_CONTIGUOUS
        d.capacity = k_cache.shape[2]
        d.page_table = None
    else:
        assert page_table.dtype == torch.int32 and page_table.is_contiguous()
        d.layout = KV_PAGED
        d.page_size = k_cache.shape[2]
        d.max_pages_per_seq = page_table.shape[1]
        d.num_pages = k_cache.shape[0]
        d.capacity = d.page_size * d.max_pages_per_seq
        d.page_table = page_table.data_ptr()
    d.tensors = (k_cache, v_cache, page_table)   # the struct holds bare addresses: keep their owners alive with it
    return d


def kv_append(desc: KvDesc, k_new: torch.Tensor, v_new: torch.Tensor, seq_lens: torch.Tensor,
              stream=None) -> None:
    B, Hkv, D = k_new.shape
    assert k_new.is_contiguous() and v_new.is_contiguous() and seq_lens.dtype == torch.int32
    _check(lib().instattn_kv_append(ctypes.byref(desc), _p(k_new), _p(v_new), _p(seq_lens),
                                    B, Hkv, D, _stream(stream)), "instattn_kv_append")


def kv_write(desc: KvDesc, k_src: torch.Tensor, v_src: torch.Tensor, start: torch.Tensor,
             count: torch.Tensor, stream=None) -> None:
    B, Hkv, N, D = k_src.shape
    assert k_src.is_contiguous() and v_src.is_contiguous() and k_src.dtype == torch.float16
    assert start.dtype == torch.int32 and count.dtype == torch.int32
    _check(lib().instattn_kv_write(ctypes.byref(desc), _p(k_src), _p(v_src), _p(start), _p(count),
                                   B, Hkv, D, N, _stream(stream)), "instattn_kv_write")


def decode_plan(batch: int, num_q_heads: int, num_kv_heads: int, head_dim: int,
                max_seq_len: int) -> Tuple[int, int]:
    chunk, splits = ctypes.c_int(0), ctypes.c_int(0)
    _check(lib().instattn_decode_plan(batch, num_q_heads, num_kv_heads, head_dim, max_seq_len,
                                      ctypes.byref(chunk), ctypes.byref(splits)),
           "instattn_decode_plan")
    return chunk.value, splits.value


def decode_launches(batch: int, num_q_heads: int, num_kv_heads: int, head_dim: int, max_seq_len: int,
                    with_append: bool = False, paged: bool = False) -> dict:
    """Which kernels a dense decode of these sizes launches (host arithmetic only)."""
    out = (ctypes.c_int32 * 4)()
    _check(lib().instattn_decode_launches(batch, num_q_heads, num_kv_heads, head_dim, max_seq_len,
                                          KV_PAGED if paged else KV_CONTIGUOUS, int(with_append), out),
           "instattn_decode_launches")
    return {"append": bool(out[0]), "unit_list": bool(out[1]), "split_pass": bool(out[2]), "merge": bool(out[3])}


def decode_workspace_size(batch: int, num_q_heads: int, num_kv_heads: int, head_dim: int,
                          max_seq_len: int) -> int:
    return lib().instattn_decode_workspace_size(batch, num_q_heads, num_kv_heads, head_dim,
                                                max_seq_len)


def _decode_args(q, desc, seq_lens, num_kv_heads, scale, out, lse, workspace, max_seq_len, stream):
    B, Hq, D = q.shape
    assert q.dtype == torch.float16 and q.is_contiguous() and out.is_contiguous()
    assert seq_lens.dtype == torch.int32 and out.shape == q.shape
    assert out.dtype in (torch.float16, torch.float32)
    assert lse is None or (lse.dtype == torch.float32 and lse.is_contiguous())
    return (_p(q), ctypes.byref(desc), _p(seq_lens), B, Hq, num_kv_heads, D, float(scale),
            _p(out), F16 if out.dtype == torch.float16 else F32, _p(lse), _p(workspace),
            workspace.numel() * workspace.element_size(), int(max_seq_len), _stream(stream))


def decode(q, desc: KvDesc, seq_lens, num_kv_heads: int, scale: float, out, workspace,
           max_seq_len: int, lse=None, stream=None) -> None:
    _check(lib().instattn_decode(*_decode_args(q, desc, seq_lens, num_kv_heads, scale, out, lse,
                                               workspace, max_seq_len, stream)), "instattn_decode")


STATIC_SCRATCH_BYTES = 32 << 20


def decode_static(q, desc: KvDesc, seq_lens, num_kv_heads: int, scale: float, out, max_seq_len: int,
                  lse=None, stream=None) -> None:
    """instattn_decode on the library's own scratch: no workspace argument, nothing allocated."""
    a = _decode_args(q, desc, seq_lens, num_kv_heads, scale, out, lse, out, max_seq_len, stream)
    _check(lib().instattn_decode_static(*a[:11], a[13], a[14]), "instattn_decode_static")


def append_decode(q, k_new, v_new, desc: KvDesc, seq_lens, num_kv_heads: int, scale: float, out,
                  workspace, max_seq_len: int, lse=None, stream=None) -> None:
    assert k_new.is_contiguous() and v_new.is_contiguous() and k_new.dtype == torch.float16
    args = _decode_args(q, desc, seq_lens, num_kv_heads, scale, out, lse, workspace, max_seq_len,
                        stream)
    _check(lib().instattn_append_decode(args[0], _p(k_new), _p(v_new), *args[1:]),
           "instattn_append_decode")


def append_decode_partial(q, k_new, v_new, desc: KvDesc, seq_lens, num_kv_heads: int, scale: float, out,
                          workspace, max_seq_len: int, lse=None, stream=None) -> None:
    assert k_new.is_contiguous() and v_new.is_contiguous() and k_new.dtype == torch.float16
    args = _decode_args(q, desc, seq_lens, num_kv_heads, scale, out, lse, workspace, max_seq_len,
                        stream)
    _check(lib().instattn_append_decode_partial(args[0], _p(k_new), _p(v_new), *args[1:]),
           "instattn_append_decode_partial")


def decode_partial(q, desc: KvDesc, seq_lens, num_kv_heads: int, scale: float, out, workspace,
                   max_seq_len: int, lse=None, stream=None) -> None:
    _check(lib().instattn_decode_partial(*_decode_args(q, desc, seq_lens, num_kv_heads, scale, out,
                                                       lse, workspace, max_seq_len, stream)),
           "instattn_decode_partial")


def decode_merge(seq_lens, num_q_heads: int, num_kv_heads: int, capacity: int, out, workspace,
                 max_seq_len: int, lse=None, stream=None) -> None:
    B, Hq, D = out.shape
    _check(lib().instattn_decode_merge(
        _p(seq_lens), B, num_q_heads, num_kv_heads, D, int(capacity), _p(out),
        F16 if out.dtype == torch.float16 else F32, _p(lse), _p(workspace),
        workspace.numel() * workspace.element_size(), int(max_seq_len), _stream(stream)),
        "instattn_decode_merge")


def alloc_workspace(batch: int, num_q_heads: int, num_kv_heads: int, head_dim: int,
                    max_seq_len: int, device) -> torch.Tensor:
    n = decode_workspace_size(batch, num_q_heads, num_kv_heads, head_dim, max_seq_len)
    if n == 0:
        raise InstattnError(ERR_INVALID_ARG, "instattn_decode_workspace_size")
    return torch.empty(n, dtype=torch.uint8, device=device)


def probe_read(src: torch.Tensor, sink: torch.Tensor, stream=None) -> None:
    _check(lib().instattn_probe_read(_p(src), src.numel() * src.element_size(), _p(sink),
                                     _stream(stream)), "instattn_probe_read")


def probe_read_columns(kt: torch.Tensor, r: int, positions: int, sink: torch.Tensor, stream=None) -> None:
    """kt: contiguous component-major copy [B, Hkv, D, capacity] fp16."""
    Bn, Hkv, D, cap = kt.shape
    assert kt.dtype == torch.float16 and kt.is_contiguous()
    _check(lib().instattn_probe_read_columns(_p(kt), D * cap * 2, cap * 2, Bn * Hkv, D, int(r), int(positions),
                                             _p(sink), _stream(stream)), "instattn_probe_read_columns")


def probe_copy(src: torch.Tensor, dst: torch.Tensor, stream=None) -> None:
    _check(lib().instattn_probe_copy(_p(src), _p(dst), src.numel() * src.element_size(),
                                     _stream(stream)), "instattn_probe_copy")


# ---------------------------------------------------------------------- SparF
def sparf_aux(kt: torch.Tensor, vsum: torch.Tensor, page_table: Optional[torch.Tensor] = None) -> SparfAux:
    """Descriptor for vsum [B, Hkv, D] fp32 and kt fp16: [B, Hkv, D, capacity], or, with
    a page table [B, max_pages] int32, a pool [num_pages, Hkv, D, page_size]."""
    assert kt.dtype == torch.float16 and kt.stride(3) == 1
    assert vsum.dtype == torch.float32 and vsum.is_contiguous()
    a = SparfAux()
    a.kt, a.vsum = kt.data_ptr(), vsum.data_ptr()
    a.stride_b, a.stride_h, a.stride_d = kt.stride(0), kt.stride(1), kt.stride(2)
    if page_table is None:
        a.capacity, a.page_size, a.page_table = kt.shape[3], 0, None
        a.max_pages_per_seq = a.num_pages = 0
    else:
        assert page_table.dtype == torch.int32 and page_table.is_contiguous()
        a.page_size, a.num_pages = kt.shape[3], kt.shape[0]
        a.max_pages_per_seq = page_table.shape[1]
        a.capacity = a.page_size * a.max_pages_per_seq
        a.page_table = page_table.data_ptr()
    a.tensors = (kt, vsum, page_table)           # keeps the owners of the addresses alive with the struct
    return a


def sparf_build_workspace_size(batch: int, num_kv_heads: int, head_dim: int) -> int:
    return lib().instattn_sparf_build_workspace_size(batch, num_kv_heads, head_dim)


def sparf_build(desc: KvDesc, aux: SparfAux, seq_lens, num_kv_heads: int, head_dim: int,
                stream=None, workspace="auto") -> None:
    """workspace: a uint8 device tensor, None (one block sums the V rows of a pair), or
    "auto": a scratch tensor of the size the library asks for, allocated here."""
    if isinstance(workspace, str):
        n = sparf_build_workspace_size(seq_lens.numel(), num_kv_heads, head_dim)
        workspace = torch.empty(n, dtype=torch.uint8, device=seq_lens.device) if n else None
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().instattn_sparf_build(ctypes.byref(desc), ctypes.byref(aux), _p(seq_lens),
                                      seq_lens.numel(), num_kv_heads, head_dim, _p(workspace), nbytes,
                                      _stream(stream)),
           "instattn_sparf_build")


def sparf_append(desc: KvDesc, aux: SparfAux, k_new, v_new, seq_lens, stream=None) -> None:
    B, Hkv, D = k_new.shape
    assert k_new.is_contiguous() and v_new.is_contiguous()
    _check(lib().instattn_sparf_append(ctypes.byref(desc), ctypes.byref(aux), _p(k_new), _p(v_new),
                                       _p(seq_lens), B, Hkv, D, _stream(stream)),
           "instattn_sparf_append")


def sparf_plan(batch: int, num_q_heads: int, num_kv_heads: int, head_dim: int, max_seq_len: int,
               k: int, with_append: bool = False) -> dict:
    """What a SparF decode of these sizes launches (host arithmetic only)."""
    out = (ctypes.c_int32 * 6)()
    _check(lib().instattn_sparf_plan(batch, num_q_heads, num_kv_heads, head_dim, max_seq_len, k,
                                     int(with_append), out), "instattn_sparf_plan")
    return {"launches": out[0], "one_launch_threads": out[1], "append_fused": bool(out[2]),
            "selection": out[3], "select_and_gather": bool(out[4]), "slices": out[5]}


def sparf_workspace_size(batch: int, num_q_heads: int, head_dim: int, max_seq_len: int,
                         k: int) -> int:
    return lib().instattn_sparf_workspace_size(batch, num_q_heads, head_dim, max_seq_len, k)


def sparf_decode(q, desc: KvDesc, aux: SparfAux, seq_lens, num_kv_heads: int, scale: float,
                 r: int, k: int, l: int, out, workspace, max_seq_len: int, sel_rows=None,
                 alpha=None, stream=None) -> None:
    B, Hq, D = q.shape
    assert q.dtype == torch.float16 and q.is_contiguous() and out.is_contiguous()
    assert sel_rows is None or (sel_rows.dtype == torch.int32 and sel_rows.shape == (B, Hq, k))
    assert alpha is None or (alpha.dtype == torch.float32 and alpha.shape == (B, Hq))
    _check(lib().instattn_sparf_decode(
        _p(q), ctypes.byref(desc), ctypes.byref(aux), _p(seq_lens), B, Hq, num_kv_heads, D,
        float(scale), int(r), int(k), int(l), _p(out),
        F16 if out.dtype == torch.float16 else F32, _p(sel_rows), _p(alpha), _p(workspace),
        workspace.numel() * workspace.element_size(), int(max_seq_len), _stream(stream)),
        "instattn_sparf_decode")


def sparf_append_decode(q, k_new, v_new, desc: KvDesc, aux: SparfAux, seq_lens, num_kv_heads: int,
                        scale: float, r: int, k: int, l: int, out, workspace, max_seq_len: int,
                        sel_rows=None, alpha=None, stream=None) -> None:
    B, Hq, D = q.shape
    assert q.dtype == torch.float16 and q.is_contiguous() and out.is_contiguous()
    assert k_new.dtype == torch.float16 and k_new.is_contiguous() and k_new.shape == (B, num_kv_heads, D)
    assert v_new.dtype == torch.float16 and v_new.is_contiguous() and v_new.shape == (B, num_kv_heads, D)
    assert sel_rows is None or (sel_rows.dtype == torch.int32 and sel_rows.shape == (B, Hq, k))
    assert alpha is None or (alpha.dtype == torch.float32 and alpha.shape == (B, Hq))
    _check(lib().instattn_sparf_append_decode(
        _p(q), _p(k_new), _p(v_new), ctypes.byref(desc), ctypes.byref(aux), _p(seq_lens), B, Hq,
        num_kv_heads, D, float(scale), int(r), int(k), int(l), _p(out),
        F16 if out.dtype == torch.float16 else F32, _p(sel_rows), _p(alpha), _p(workspace),
        workspace.numel() * workspace.element_size(), int(max_seq_len), _stream(stream)),
        "instattn_sparf_append_decode")
