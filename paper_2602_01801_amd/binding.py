"""ctypes front end of libfastar.so: argument marshalling only.

Every step of the path runs in the library's HIP kernels; PyTorch supplies device memory and the
stream.  Function names and argument meaning follow ``include/fastar.h``.  There is no fallback:
if the library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfastar.so")

F32, BF16 = 0, 1
OP_COMPRESS, OP_SELECT_SELF, OP_SELECT_CROSS, OP_SELECT_LSH, OP_SELECT_BUCKETS, OP_ATTN = 1, 2, 3, 4, 5, 6
REP_LAST, REP_MEAN, REP_MEDOID = 0, 1, 2

_lib = None


class FastarError(RuntimeError):
    pass


class _CacheStruct(ctypes.Structure):
    _fields_ = [("K", ctypes.c_void_p), ("V", ctypes.c_void_p), ("code", ctypes.c_void_p), ("cnt", ctypes.c_void_p),
                ("stamp", ctypes.c_void_p), ("len", ctypes.c_void_p), ("H", ctypes.c_int32), ("C", ctypes.c_int32),
                ("d", ctypes.c_int32), ("r", ctypes.c_int32), ("dtype", ctypes.c_int32)]


class _CodecStruct(ctypes.Structure):
    _fields_ = [("R", ctypes.c_void_p), ("qscale", ctypes.c_float), ("shift", ctypes.c_int32)]


def lib() -> ctypes.CDLL:
    """Load libfastar.so (built in-tree by ``paper_2602_01801_amd.build``).  Fails loudly when absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FastarError(f"{LIB_PATH} is missing: run `python -m paper_2602_01801_amd.build` "
                              "(or __graft_entry__.build()) first; there is no fallback path")
        L = ctypes.CDLL(LIB_PATH)
        L.fastar_init.restype = ctypes.c_int
        L.fastar_init.argtypes = []
        L.fastar_version.restype = ctypes.c_char_p
        L.fastar_strerror.restype = ctypes.c_char_p
        L.fastar_strerror.argtypes = [ctypes.c_int]
        L.fastar_workspace_bytes.restype = ctypes.c_size_t
        L.fastar_workspace_bytes.argtypes = [ctypes.c_int] * 8
        L.fastar_encode.restype = ctypes.c_int
        L.fastar_encode.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_int,
                                    ctypes.POINTER(_CodecStruct), ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
        L.tempcache_compress.restype = ctypes.c_int
        L.tempcache_compress.argtypes = [ctypes.POINTER(_CacheStruct), ctypes.POINTER(_CodecStruct), ctypes.c_void_p,
                                         ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_int,
                                         ctypes.c_int, ctypes.c_int32, ctypes.c_int32, ctypes.c_int, ctypes.c_void_p,
                                         ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t,
                                         ctypes.c_int, ctypes.c_void_p]
        L.ann_cross_attn_fwd.restype = ctypes.c_int
        L.ann_cross_attn_fwd.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p,
                                         ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                         ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_float, ctypes.c_void_p,
                                         ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        L.ann_select_self.restype = ctypes.c_int
        L.ann_select_self.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int,
                                      ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                      ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                      ctypes.c_size_t, ctypes.c_void_p]
        L.ann_select_self_forced.restype = ctypes.c_int
        L.ann_select_self_forced.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p] + \
            [ctypes.c_int] * 9 + [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        L.ann_prompt_buckets.restype = ctypes.c_int
        L.ann_prompt_buckets.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p] + \
            [ctypes.c_int] * 4 + [ctypes.c_void_p, ctypes.c_void_p]
        L.ann_select_buckets.restype = ctypes.c_int
        L.ann_select_buckets.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p] + \
            [ctypes.c_int] * 9 + [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        L.fastar_encode_packed.restype = ctypes.c_int
        L.fastar_encode_packed.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_int,
                                           ctypes.POINTER(_CodecStruct), ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
        L.ann_select_self_packed.restype = ctypes.c_int
        L.ann_select_self_packed.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p] + \
            [ctypes.c_int] * 10 + [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        L.ann_select_lsh_buckets.restype = ctypes.c_int
        L.ann_select_lsh_buckets.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p] + \
            [ctypes.c_int] * 11 + [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        L.ann_select_self_static.restype = ctypes.c_int
        L.ann_select_self_static.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int,
                                             ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                             ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        L.ann_select_cross.restype = ctypes.c_int
        L.ann_select_cross.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_int, ctypes.c_int,
                                       ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p,
                                       ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        L.sparse_attn_fwd.restype = ctypes.c_int
        L.sparse_attn_fwd.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                      ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                      ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                      ctypes.c_float, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        L.sparse_attn_fwd_ws.restype = ctypes.c_int
        L.sparse_attn_fwd_ws.argtypes = L.sparse_attn_fwd.argtypes[:-1] + [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        L.fastar_kv_to_fp8.restype = ctypes.c_int
        L.fastar_kv_to_fp8.argtypes = [ctypes.POINTER(_CacheStruct), ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p,
                                       ctypes.c_void_p]
        L.sparse_attn_fwd_fp8.restype = ctypes.c_int
        L.sparse_attn_fwd_fp8.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                          ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p,
                                          ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_float,
                                          ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        L.sparse_attn_fwd_fp8_ws.restype = ctypes.c_int
        L.sparse_attn_fwd_fp8_ws.argtypes = L.sparse_attn_fwd_fp8.argtypes[:-1] + [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        L.fastar_encode_sign.restype = ctypes.c_int
        L.fastar_encode_sign.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_int, ctypes.c_void_p,
                                         ctypes.c_float, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
        L.ann_select_lsh.restype = ctypes.c_int
        L.ann_select_lsh.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p] + \
            [ctypes.c_int] * 7 + [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        L.fastar_probe_mfma_bf16.restype = ctypes.c_int
        L.fastar_probe_mfma_bf16.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.POINTER(ctypes.c_double), ctypes.c_void_p]
        L.fastar_probe_copy.restype = ctypes.c_int
        L.fastar_probe_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        L.fastar_debug_plan_wait.restype = ctypes.c_int
        L.fastar_debug_plan_wait.argtypes = [ctypes.c_int, ctypes.c_int]
        _lib = L
    return _lib


EXPORTS = ("fastar_init", "fastar_version", "fastar_strerror", "fastar_workspace_bytes", "fastar_encode", "tempcache_compress",
           "ann_cross_attn_fwd",
           "ann_select_self", "ann_select_self_forced", "ann_select_self_static", "ann_prompt_buckets", "ann_select_buckets", "fastar_encode_packed", "ann_select_self_packed", "ann_select_cross", "sparse_attn_fwd", "sparse_attn_fwd_ws", "fastar_kv_to_fp8",
           "sparse_attn_fwd_fp8", "sparse_attn_fwd_fp8_ws", "fastar_encode_sign", "ann_select_lsh", "ann_select_lsh_buckets",
           "fastar_probe_mfma_bf16", "fastar_probe_copy", "fastar_debug_plan_wait")


def init() -> None:
    """fastar_init: one-time kernel set-up for the current device (optional; needed before graph capture)."""
    _check(lib().fastar_init(), "fastar_init")


def _check(rc: int, what: str):
    if rc != 0:
        raise FastarError(f"{what}: {lib().fastar_strerror(rc).decode()} ({rc})")


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t):
    return None if t is None else t.data_ptr()


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"dtype must be float32 or bfloat16, got {t.dtype}")


def _dev(t: torch.Tensor, dtype=None):
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("tensors must be contiguous device tensors")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"expected {dtype}, got {t.dtype}")
    return t


def workspace_bytes(op: int, H: int, n_q: int, n_k: int, r: int = 32, BQ: int = 128, BK: int = 64,
                    n_rep: int = 4) -> int:
    return int(lib().fastar_workspace_bytes(op, H, n_q, n_k, r, BQ, BK, n_rep))


def _workspace(ws, nbytes: int, device):
    if ws is None:
        ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)
    if ws.numel() * ws.element_size() < nbytes:
        raise FastarError("workspace too small")
    return ws


@dataclass
class Codec:
    """Definition of the ANN code: +-1 projection R [d,r] (device int8), quantiser scale, requantise shift."""
    R: torch.Tensor
    qscale: float
    shift: int

    def struct(self) -> _CodecStruct:
        _dev(self.R, torch.int8)
        return _CodecStruct(self.R.data_ptr(), float(self.qscale), int(self.shift))


@dataclass
class Cache:
    """Device buffers of the bounded per-head KV cache with multiplicities (capacity C slots per head)."""
    K: torch.Tensor      # [H,C,d]
    V: torch.Tensor      # [H,C,d]
    code: torch.Tensor   # [H,C,r] int8
    cnt: torch.Tensor    # [H,C] int32
    stamp: torch.Tensor  # [H,C] int32
    len: torch.Tensor    # [H] int32

    @classmethod
    def empty(cls, H: int, C: int, d: int, r: int, dtype: torch.dtype, device="cuda") -> "Cache":
        z = lambda *s, dt: torch.zeros(*s, dtype=dt, device=device)
        return cls(z(H, C, d, dt=dtype), z(H, C, d, dt=dtype), z(H, C, r, dt=torch.int8), z(H, C, dt=torch.int32),
                   z(H, C, dt=torch.int32), z(H, dt=torch.int32))

    @property
    def shape(self):
        H, C, d = self.K.shape
        return H, C, d, self.code.shape[2]

    def struct(self) -> _CacheStruct:
        H, C, d, r = self.shape
        for t in (self.K, self.V, self.code, self.cnt, self.stamp, self.len):
            _dev(t)
        return _CacheStruct(self.K.data_ptr(), self.V.data_ptr(), self.code.data_ptr(), self.cnt.data_ptr(),
                            self.stamp.data_ptr(), self.len.data_ptr(), H, C, d, r, _dtype_code(self.K))

    def nbytes(self) -> int:
        return sum(t.numel() * t.element_size() for t in (self.K, self.V, self.code, self.cnt, self.stamp, self.len))


def encode(x: torch.Tensor, codec: Codec, out: torch.Tensor | None = None) -> torch.Tensor:
    """x [..., d] -> int8 codes [..., r]."""
    _dev(x)
    d, r = codec.R.shape
    n_vec = x.numel() // d
    if out is None:
        out = torch.empty(x.shape[:-1] + (r,), dtype=torch.int8, device=x.device)
    cs = codec.struct()
    _check(lib().fastar_encode(x.data_ptr(), _dtype_code(x), n_vec, d, ctypes.byref(cs), r, out.data_ptr(), _stream()),
           "fastar_encode")
    return out


def encode_packed(x: torch.Tensor, codec: Codec, bits: int, out: torch.Tensor | None = None) -> torch.Tensor:
    """x [..., d] -> codes of `bits` (2, 4 or 8) bits per entry, packed: uint8 [..., r*bits/8]."""
    _dev(x)
    d, r = codec.R.shape
    n_vec = x.numel() // d
    if out is None:
        out = torch.empty(x.shape[:-1] + (r * bits // 8,), dtype=torch.uint8, device=x.device)
    cs = codec.struct()
    _check(lib().fastar_encode_packed(x.data_ptr(), _dtype_code(x), n_vec, d, ctypes.byref(cs), r, bits, out.data_ptr(),
                                      _stream()), "fastar_encode_packed")
    return out


def ann_select_self_packed(qcode, kcode, length, bits: int, BQ: int, n_rep: int, BK: int, n_sel: int, n_sink: int = 0,
                           n_local: int = 0, ws=None, out=None):
    """AnnSA on packed codes (uint8 [H,n,r*bits/8]): the selection ann_select_self makes on the unpacked entries."""
    _dev(qcode, torch.uint8)
    _dev(kcode, torch.uint8)
    _dev(length, torch.int32)
    H, n_q, rb = qcode.shape
    r = rb * 8 // bits
    C = kcode.shape[1]
    n_qb = (n_q + BQ - 1) // BQ
    ws = _workspace(ws, workspace_bytes(OP_SELECT_SELF, H, n_q, C, r, BQ, BK, n_rep), qcode.device)
    if out is None:
        out = (torch.empty((H, n_qb, n_sel), dtype=torch.int32, device=qcode.device),
               torch.empty((H, n_qb), dtype=torch.int32, device=qcode.device))
    sel, nsel = out
    _check(lib().ann_select_self_packed(qcode.data_ptr(), n_q, kcode.data_ptr(), length.data_ptr(), H, C, r, bits, BQ,
                                        n_rep, BK, n_sel, n_sink, n_local, sel.data_ptr(), nsel.data_ptr(), ws.data_ptr(),
                                        ws.numel() * ws.element_size(), _stream()), "ann_select_self_packed")
    return sel, nsel


def tempcache_compress(cache: Cache, codec: Codec, K_new, V_new, P_new=None, cand=None, metric: int = 0,
                       tau2_q16: int = 53084, frame_id: int = 0, rep_mode: int = 0, ws=None, out=None,
                       ws_persistent: bool = False):
    """Merge one frame into ``cache`` in place.  Returns (merge_map [H,n] int32, merged [H,n] uint8, stats [H,8]).
    rep_mode: REP_LAST (0) keeps the last key of a merged group, REP_MEAN (1) its multiplicity-weighted mean.
    ws_persistent: ``ws`` was zero-filled once and has since been written only by calls on this cache (one launch less)."""
    if ws_persistent and ws is None:
        raise ValueError("ws_persistent needs the caller's own workspace")
    H, C, d, r = cache.shape
    _dev(K_new, cache.K.dtype)
    _dev(V_new, cache.K.dtype)
    n_new = K_new.shape[1]
    if P_new is not None:
        _dev(P_new, cache.K.dtype)
    n_cand = 0
    if cand is not None:
        _dev(cand, torch.int32)
        n_cand = cand.shape[1]
    ws = _workspace(ws, workspace_bytes(OP_COMPRESS, H, n_new, C, r), K_new.device)
    if out is None:
        out = (torch.empty((H, n_new), dtype=torch.int32, device=K_new.device),
               torch.empty((H, n_new), dtype=torch.uint8, device=K_new.device),
               torch.empty((H, 8), dtype=torch.int32, device=K_new.device))
    merge_map, merged, stats = out
    cs, ks = cache.struct(), codec.struct()
    _check(lib().tempcache_compress(ctypes.byref(cs), ctypes.byref(ks), K_new.data_ptr(), V_new.data_ptr(),
                                    _ptr(P_new), n_new, _ptr(cand), n_cand, metric, tau2_q16, frame_id,
                                    int(rep_mode), merge_map.data_ptr(), merged.data_ptr(), stats.data_ptr(), ws.data_ptr(),
                                    ws.numel() * ws.element_size(), 1 if ws_persistent else 0, _stream()),
           "tempcache_compress")
    return merge_map, merged, stats


def ann_select_self(qcode, kcode, length, BQ: int, n_rep: int, BK: int, n_sel: int, ws=None, out=None, n_sink: int = 0,
                    n_local: int = 0):
    """AnnSA: (sel [H,n_qb,n_sel] int32 ascending / -1 padded, nsel [H,n_qb] int32).  n_sink / n_local > 0 calls
    ann_select_self_forced (first / last live key blocks always selected)."""
    _dev(qcode, torch.int8)
    _dev(kcode, torch.int8)
    _dev(length, torch.int32)
    H, n_q, r = qcode.shape
    C = kcode.shape[1]
    n_qb = (n_q + BQ - 1) // BQ
    ws = _workspace(ws, workspace_bytes(OP_SELECT_SELF, H, n_q, C, r, BQ, BK, n_rep), qcode.device)
    if out is None:
        out = (torch.empty((H, n_qb, n_sel), dtype=torch.int32, device=qcode.device),
               torch.empty((H, n_qb), dtype=torch.int32, device=qcode.device))
    sel, nsel = out
    if n_sink or n_local:
        _check(lib().ann_select_self_forced(qcode.data_ptr(), n_q, kcode.data_ptr(), length.data_ptr(), H, C, r, BQ, n_rep,
                                            BK, n_sel, n_sink, n_local, sel.data_ptr(), nsel.data_ptr(), ws.data_ptr(),
                                            ws.numel() * ws.element_size(), _stream()), "ann_select_self_forced")
        return sel, nsel
    _check(lib().ann_select_self(qcode.data_ptr(), n_q, kcode.data_ptr(), length.data_ptr(), H, C, r, BQ, n_rep, BK,
                                 n_sel, sel.data_ptr(), nsel.data_ptr(), ws.data_ptr(),
                                 ws.numel() * ws.element_size(), _stream()), "ann_select_self")
    return sel, nsel


def ann_select_self_static(qcode, kcode, length, BQ: int, n_rep: int, BK: int, n_sel: int, out):
    """AnnSA on the library's static scratch: the call allocates nothing, so the outputs (sel, nsel) must be given."""
    _dev(qcode, torch.int8)
    _dev(kcode, torch.int8)
    _dev(length, torch.int32)
    H, n_q, r = qcode.shape
    C = kcode.shape[1]
    sel, nsel = out
    _dev(sel, torch.int32)
    _dev(nsel, torch.int32)
    n_qb = (n_q + BQ - 1) // BQ
    if tuple(sel.shape) != (H, n_qb, n_sel) or tuple(nsel.shape) != (H, n_qb):
        raise ValueError("out must be (sel [H,n_qb,n_sel], nsel [H,n_qb])")
    _check(lib().ann_select_self_static(qcode.data_ptr(), n_q, kcode.data_ptr(), length.data_ptr(), H, C, r, BQ, n_rep,
                                        BK, n_sel, sel.data_ptr(), nsel.data_ptr(), _stream()), "ann_select_self_static")
    return sel, nsel


def prompt_buckets(code, pcode, m: int = 1, idx=None, out=None):
    """The m nearest prompt tokens of every code row: bucket [H,C,m] int32.  idx [H,n] int32 names the rows to assign
    (the others keep what `out` holds); without it every row is assigned."""
    _dev(code, torch.int8)
    _dev(pcode, torch.int8)
    H, C, r = code.shape
    n_p = pcode.shape[1]
    if out is None:
        out = torch.full((H, C, m), -1, dtype=torch.int32, device=code.device)
    if idx is not None:
        _dev(idx, torch.int32)
    n = C if idx is None else idx.shape[1]
    _check(lib().ann_prompt_buckets(code.data_ptr(), C, idx.data_ptr() if idx is not None else None, n, pcode.data_ptr(),
                                    n_p, H, r, m, out.data_ptr(), _stream()), "ann_prompt_buckets")
    return out


def ann_select_buckets(qbucket, kbucket, length, n_p: int, BQ: int, BK: int, n_sel: int, n_sink: int = 0, n_local: int = 0,
                       ws=None, out=None):
    """AnnSA on prompt-induced buckets: (sel [H,n_qb,n_sel] int32 ascending / -1 padded, nsel [H,n_qb] int32)."""
    _dev(qbucket, torch.int32)
    _dev(kbucket, torch.int32)
    _dev(length, torch.int32)
    H, n_q, m = qbucket.shape
    C = kbucket.shape[1]
    n_qb = (n_q + BQ - 1) // BQ
    ws = _workspace(ws, workspace_bytes(OP_SELECT_BUCKETS, H, n_q, C, n_p, BQ, BK, 0), qbucket.device)
    if out is None:
        out = (torch.empty((H, n_qb, n_sel), dtype=torch.int32, device=qbucket.device),
               torch.empty((H, n_qb), dtype=torch.int32, device=qbucket.device))
    sel, nsel = out
    _check(lib().ann_select_buckets(qbucket.data_ptr(), n_q, kbucket.data_ptr(), length.data_ptr(), H, C, m, n_p, BQ, BK,
                                    n_sel, n_sink, n_local, sel.data_ptr(), nsel.data_ptr(), ws.data_ptr(),
                                    ws.numel() * ws.element_size(), _stream()), "ann_select_buckets")
    return sel, nsel


def ann_select_cross(qcode, pcode, BQ: int, n_sel: int, ws=None, out=None):
    """AnnCA: (sel [H,n_qb,n_sel] prompt-token ids ascending / -1 padded, nsel [H,n_qb])."""
    _dev(qcode, torch.int8)
    _dev(pcode, torch.int8)
    H, n_q, r = qcode.shape
    n_p = pcode.shape[1]
    n_qb = (n_q + BQ - 1) // BQ
    ws = _workspace(ws, workspace_bytes(OP_SELECT_CROSS, H, n_q, n_p, r, BQ), qcode.device)
    if out is None:
        out = (torch.empty((H, n_qb, n_sel), dtype=torch.int32, device=qcode.device),
               torch.empty((H, n_qb), dtype=torch.int32, device=qcode.device))
    sel, nsel = out
    _check(lib().ann_select_cross(qcode.data_ptr(), n_q, pcode.data_ptr(), n_p, H, r, BQ, n_sel, sel.data_ptr(),
                                  nsel.data_ptr(), ws.data_ptr(), ws.numel() * ws.element_size(), _stream()),
           "ann_select_cross")
    return sel, nsel


def encode_sign(x: torch.Tensor, R: torch.Tensor, qscale: float, out: torch.Tensor | None = None) -> torch.Tensor:
    """x [..., d], R [d, n_bits] int8 (+-1) -> sign codes [..., n_bits/32] as int32 words (bit patterns)."""
    _dev(x)
    _dev(R, torch.int8)
    d, n_bits = R.shape
    if x.shape[-1] != d or not x.is_contiguous() or not R.is_contiguous():
        raise ValueError("encode_sign: x must be contiguous [..., d] and R contiguous [d, n_bits]")
    n_vec = x.numel() // d
    if out is None:
        out = torch.empty(x.shape[:-1] + (n_bits // 32,), dtype=torch.int32, device=x.device)
    _check(lib().fastar_encode_sign(x.data_ptr(), _dtype_code(x), n_vec, d, R.data_ptr(), float(qscale), n_bits,
                                    out.data_ptr(), _stream()), "fastar_encode_sign")
    return out


def ann_select_lsh(qbits, kbits, length, BQ: int, n_rep: int, BK: int, n_sel: int, ws=None, out=None):
    """Selection on sign codes: (sel [H,n_qb,n_sel] int32 ascending / -1 padded, nsel [H,n_qb] int32)."""
    _dev(qbits, torch.int32)
    _dev(kbits, torch.int32)
    _dev(length, torch.int32)
    H, n_q, W = qbits.shape
    C = kbits.shape[1]
    n_qb = (n_q + BQ - 1) // BQ
    ws = _workspace(ws, workspace_bytes(OP_SELECT_LSH, H, n_q, C, 32 * W, BQ, BK, n_rep), qbits.device)
    if out is None:
        out = (torch.empty((H, n_qb, n_sel), dtype=torch.int32, device=qbits.device),
               torch.empty((H, n_qb), dtype=torch.int32, device=qbits.device))
    sel, nsel = out
    _check(lib().ann_select_lsh(qbits.data_ptr(), n_q, kbits.data_ptr(), length.data_ptr(), H, C, 32 * W, BQ, n_rep,
                                BK, n_sel, sel.data_ptr(), nsel.data_ptr(), ws.data_ptr(),
                                ws.numel() * ws.element_size(), _stream()), "ann_select_lsh")
    return sel, nsel


def ann_select_lsh_buckets(qbits, kbits, length, band_bits: int, radius: int, BQ: int, n_rep: int, BK: int, n_sel: int,
                           n_sink: int = 0, n_local: int = 0, ws=None, out=None):
    """Hash-table form of ann_select_lsh (bands = tables, buckets at most `radius` bits apart collide)."""
    _dev(qbits, torch.int32)
    _dev(kbits, torch.int32)
    _dev(length, torch.int32)
    H, n_q, W = qbits.shape
    C = kbits.shape[1]
    n_qb = (n_q + BQ - 1) // BQ
    ws = _workspace(ws, workspace_bytes(OP_SELECT_LSH, H, n_q, C, 32 * W, BQ, BK, n_rep), qbits.device)
    if out is None:
        out = (torch.empty((H, n_qb, n_sel), dtype=torch.int32, device=qbits.device),
               torch.empty((H, n_qb), dtype=torch.int32, device=qbits.device))
    sel, nsel = out
    _check(lib().ann_select_lsh_buckets(qbits.data_ptr(), n_q, kbits.data_ptr(), length.data_ptr(), H, C, 32 * W,
                                        band_bits, radius, BQ, n_rep, BK, n_sel, n_sink, n_local, sel.data_ptr(),
                                        nsel.data_ptr(), ws.data_ptr(), ws.numel() * ws.element_size(), _stream()),
           "ann_select_lsh_buckets")
    return sel, nsel


def ann_cross_attn_fwd(Q, qcode, Kp, Vp, pcode, BQ: int, n_sel: int, scale: float, out=None):
    """AnnCA selection and the attention over it in one launch.  Returns (sel [H,n_qb,n_sel], nsel [H,n_qb], O)."""
    _dev(Q)
    _dev(Kp, Q.dtype)
    _dev(Vp, Q.dtype)
    _dev(qcode, torch.int8)
    _dev(pcode, torch.int8)
    H, n_q, d = Q.shape
    n_p, r = pcode.shape[1], pcode.shape[2]
    n_qb = (n_q + BQ - 1) // BQ
    if out is None:
        out = (torch.empty((H, n_qb, n_sel), dtype=torch.int32, device=Q.device),
               torch.empty((H, n_qb), dtype=torch.int32, device=Q.device), torch.empty_like(Q))
    sel, nsel, O = out
    _check(lib().ann_cross_attn_fwd(Q.data_ptr(), qcode.data_ptr(), n_q, Kp.data_ptr(), Vp.data_ptr(), pcode.data_ptr(),
                                    n_p, H, d, _dtype_code(Q), r, BQ, n_sel, float(scale), sel.data_ptr(),
                                    nsel.data_ptr(), O.data_ptr(), _stream()), "ann_cross_attn_fwd")
    return sel, nsel, O


def sparse_attn_fwd(Q, K, V, cnt, length, sel, nsel, BQ: int, BK: int, scale: float, out=None, want_lse: bool = True,
                    ws=None):
    """Block-sparse attention.  Returns (O [H,n_q,d] in Q's dtype, lse [H,n_q] float32 or None).
    ws: uint8 device workspace of workspace_bytes(OP_ATTN, ...) -> sparse_attn_fwd_ws (persistent kernel where it pays)."""
    _dev(Q)
    _dev(K, Q.dtype)
    _dev(V, Q.dtype)
    _dev(length, torch.int32)
    _dev(sel, torch.int32)
    _dev(nsel, torch.int32)
    if cnt is not None:
        _dev(cnt, torch.int32)
    H, n_q, d = Q.shape
    C = K.shape[1]
    n_sel = sel.shape[2]
    if out is None:
        out = (torch.empty_like(Q), torch.empty((H, n_q), dtype=torch.float32, device=Q.device) if want_lse else None)
    O, lse = out
    if ws is not None:
        _dev(ws, torch.uint8)
        _check(lib().sparse_attn_fwd_ws(Q.data_ptr(), n_q, K.data_ptr(), V.data_ptr(), _ptr(cnt), length.data_ptr(), H, C,
                                        d, _dtype_code(Q), sel.data_ptr(), nsel.data_ptr(), BQ, BK, n_sel, float(scale),
                                        O.data_ptr(), _ptr(lse), ws.data_ptr(), ws.numel(), _stream()),
               "sparse_attn_fwd_ws")
        return O, lse
    _check(lib().sparse_attn_fwd(Q.data_ptr(), n_q, K.data_ptr(), V.data_ptr(), _ptr(cnt), length.data_ptr(), H, C, d,
                                 _dtype_code(Q), sel.data_ptr(), nsel.data_ptr(), BQ, BK, n_sel, float(scale),
                                 O.data_ptr(), _ptr(lse), _stream()), "sparse_attn_fwd")
    return O, lse


def kv8_empty(H: int, C: int, d: int = 128, device="cuda"):
    """Zero-filled 8-bit copy of a cache of capacity C: (K8 [H,Cp,d], V8T [H,Cp/64,d,64]) uint8, Cp = C rounded up to 64."""
    n_blk = (C + 63) // 64
    return (torch.zeros((H, n_blk * 64, d), dtype=torch.uint8, device=device),
            torch.zeros((H, n_blk, d, 64), dtype=torch.uint8, device=device))


def kv_to_fp8(cache: Cache, K8: torch.Tensor, V8T: torch.Tensor, stamp_lo: int = -2 ** 31) -> None:
    """fastar_kv_to_fp8: rewrite the blocks of the 8-bit copy that hold a live slot with stamp >= stamp_lo."""
    H, C, d, _ = cache.shape
    n_blk = (C + 63) // 64
    _dev(K8, torch.uint8)
    _dev(V8T, torch.uint8)
    if tuple(K8.shape) != (H, n_blk * 64, d) or tuple(V8T.shape) != (H, n_blk, d, 64):
        raise ValueError("K8 must be [H,Cp,d] and V8T [H,Cp/64,d,64] with Cp = C rounded up to a multiple of 64")
    cs = cache.struct()
    _check(lib().fastar_kv_to_fp8(ctypes.byref(cs), int(stamp_lo), K8.data_ptr(), V8T.data_ptr(), _stream()),
           "fastar_kv_to_fp8")


def sparse_attn_fwd_fp8(Q, K8, V8T, cnt, length, C: int, sel, nsel, BQ: int, BK: int, scale: float, out=None,
                        want_lse: bool = True, ws=None):
    """Block-sparse attention over the 8-bit cache copy.  Returns (O [H,n_q,d] bf16, lse [H,n_q] float32 or None).
    ws: workspace of workspace_bytes(OP_ATTN, ...) -> sparse_attn_fwd_fp8_ws."""
    _dev(Q, torch.bfloat16)
    _dev(K8, torch.uint8)
    _dev(V8T, torch.uint8)
    _dev(length, torch.int32)
    _dev(sel, torch.int32)
    _dev(nsel, torch.int32)
    if cnt is not None:
        _dev(cnt, torch.int32)
    H, n_q, d = Q.shape
    n_blk = (C + 63) // 64
    if tuple(K8.shape) != (H, n_blk * 64, d) or tuple(V8T.shape) != (H, n_blk, d, 64):
        raise ValueError("K8 must be [H,Cp,d] and V8T [H,Cp/64,d,64] with Cp = C rounded up to a multiple of 64")
    n_sel = sel.shape[2]
    if out is None:
        out = (torch.empty_like(Q), torch.empty((H, n_q), dtype=torch.float32, device=Q.device) if want_lse else None)
    O, lse = out
    if ws is not None:
        _dev(ws, torch.uint8)
        _check(lib().sparse_attn_fwd_fp8_ws(Q.data_ptr(), n_q, K8.data_ptr(), V8T.data_ptr(), _ptr(cnt), length.data_ptr(),
                                            H, C, d, sel.data_ptr(), nsel.data_ptr(), BQ, BK, n_sel, float(scale),
                                            O.data_ptr(), _ptr(lse), ws.data_ptr(), ws.numel(), _stream()),
               "sparse_attn_fwd_fp8_ws")
        return O, lse
    _check(lib().sparse_attn_fwd_fp8(Q.data_ptr(), n_q, K8.data_ptr(), V8T.data_ptr(), _ptr(cnt), length.data_ptr(), H, C,
                                     d, sel.data_ptr(), nsel.data_ptr(), BQ, BK, n_sel, float(scale), O.data_ptr(),
                                     _ptr(lse), _stream()), "sparse_attn_fwd_fp8")
    return O, lse


def probe_mfma_bf16(iters: int = 20000, random_operands: bool = False) -> float:
    """Measured register-resident bf16 matrix-core rate in TFLOP/s (times one probe launch with events); with
    random_operands the multipliers see data like real keys and queries and the chip holds a lower clock."""
    sink = torch.zeros(1, dtype=torch.float32, device="cuda")
    flops = ctypes.c_double(0.0)
    ro = 1 if random_operands else 0
    _check(lib().fastar_probe_mfma_bf16(200, ro, sink.data_ptr(), ctypes.byref(flops), _stream()), "fastar_probe_mfma_bf16")
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    _check(lib().fastar_probe_mfma_bf16(iters, ro, sink.data_ptr(), ctypes.byref(flops), _stream()), "fastar_probe_mfma_bf16")
    e1.record()
    torch.cuda.synchronize()
    return flops.value / (e0.elapsed_time(e1) * 1e-3) / 1e12


def debug_plan_wait(spin_limit: int = -1, extra_arrivals: int = 0) -> None:
    """Test hook (fastar_debug_plan_wait): bound the eviction plan's waits and add arrivals that never come."""
    _check(lib().fastar_debug_plan_wait(spin_limit, extra_arrivals), "fastar_debug_plan_wait")


def probe_copy(mib: int = 1024, reps: int = 5) -> float:
    """Measured streaming-copy rate in GB/s (read + write bytes over time)."""
    src = torch.ones(mib << 20, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    _check(lib().fastar_probe_copy(src.data_ptr(), dst.data_ptr(), src.numel(), _stream()), "fastar_probe_copy")
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        _check(lib().fastar_probe_copy(src.data_ptr(), dst.data_ptr(), src.numel(), _stream()), "fastar_probe_copy")
    e1.record()
    torch.cuda.synchronize()
    return 2.0 * src.numel() * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9
