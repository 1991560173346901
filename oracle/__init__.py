"""CPU oracle of the FAST-AR attention hot path.  TEST INFRASTRUCTURE ONLY.

Thin numpy/ctypes front end of ``fastar_oracle.c`` (plain C, fp64 accumulation, integer
decisions).  Only ``tests/``, ``__graft_entry__.smoke()`` and ``bench.py``'s cpu_baseline leg
may import this package; it imports nothing from the GPU package and shares no code with it.

Tensors travel in storage form: ``float32`` arrays (dtype code 0) or ``uint16`` arrays of
bfloat16 bit patterns (dtype code 1).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fastar_oracle.c")
_LIB = os.path.join(_HERE, "libfastar_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP over heads / query blocks; no fast-math, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math",
               "-Wall", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        for name in ("oracle_encode", "oracle_tempcache_compress", "oracle_ann_select_self",
                     "oracle_ann_select_cross", "oracle_sparse_attn_fwd", "oracle_recall_density",
                     "oracle_encode_sign", "oracle_ann_select_lsh", "oracle_fp8_encode", "oracle_fp8_decode",
                     "oracle_kv_to_fp8", "oracle_sparse_attn_fwd_fp8", "oracle_ann_select_self_forced",
                     "oracle_prompt_buckets", "oracle_ann_select_buckets", "oracle_encode_packed", "oracle_unpack_codes", "oracle_ann_select_lsh_buckets"):
            getattr(_lib, name).restype = ctypes.c_int
    return _lib


def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return 0
    if a.dtype == np.uint16:
        return 1
    raise TypeError(f"storage dtype must be float32 or uint16 (bf16 bits), got {a.dtype}")


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype=None):
    a = np.ascontiguousarray(a) if dtype is None else np.ascontiguousarray(a, dtype=dtype)
    return a


def _check(rc, what):
    if rc != 0:
        raise RuntimeError(f"{what} failed with code {rc}")


# ----------------------------------------------------------------------------------------------


def encode(x: np.ndarray, R: np.ndarray, qscale, shift: int) -> np.ndarray:
    """x [..., d] (storage form) -> int8 codes [..., r]."""
    x = _c(x)
    R = _c(R, np.int8)
    d, r = R.shape
    assert x.shape[-1] == d
    n_vec = x.size // d
    code = np.empty(x.shape[:-1] + (r,), dtype=np.int8)
    rc = _load().oracle_encode(_p(x), _dtype_code(x), ctypes.c_int64(n_vec), d, _p(R), r,
                               ctypes.c_float(float(np.float32(qscale))), int(shift), _p(code))
    _check(rc, "oracle_encode")
    return code


def encode_packed(x: np.ndarray, R: np.ndarray, qscale, shift: int, bits: int) -> np.ndarray:
    """x [..., d] (storage form) -> packed codes [..., r*bits/8] uint8, `bits` per entry (2, 4 or 8)."""
    x = _c(x)
    R = _c(R, np.int8)
    d, r = R.shape
    assert x.shape[-1] == d
    n_vec = x.size // d
    packed = np.empty(x.shape[:-1] + (r * bits // 8,), dtype=np.uint8)
    rc = _load().oracle_encode_packed(_p(x), _dtype_code(x), ctypes.c_int64(n_vec), d, _p(R), r,
                                      ctypes.c_float(float(np.float32(qscale))), int(shift), int(bits), _p(packed))
    _check(rc, "oracle_encode_packed")
    return packed


def unpack_codes(packed: np.ndarray, r: int, bits: int) -> np.ndarray:
    """packed [..., r*bits/8] uint8 -> int8 entries [..., r]."""
    packed = _c(packed, np.uint8)
    n_vec = packed.size // (r * bits // 8)
    code = np.empty(packed.shape[:-1] + (r,), dtype=np.int8)
    _check(_load().oracle_unpack_codes(_p(packed), ctypes.c_int64(n_vec), r, int(bits), _p(code)), "oracle_unpack_codes")
    return code


@dataclass
class Cache:
    """Per-head bounded KV cache with multiplicities (host arrays, capacity C slots per head)."""
    K: np.ndarray       # [H,C,d] storage form: representative (most recent) keys
    V: np.ndarray       # [H,C,d] storage form: mean values
    code: np.ndarray    # [H,C,r] int8
    cnt: np.ndarray     # [H,C] int32 multiplicity m
    stamp: np.ndarray   # [H,C] int32 frame id of last refresh
    len: np.ndarray     # [H] int32 live slots

    @classmethod
    def empty(cls, H: int, C: int, d: int, r: int, dtype: str) -> "Cache":
        st = np.float32 if dtype == "fp32" else np.uint16
        return cls(K=np.zeros((H, C, d), st), V=np.zeros((H, C, d), st), code=np.zeros((H, C, r), np.int8),
                   cnt=np.zeros((H, C), np.int32), stamp=np.zeros((H, C), np.int32), len=np.zeros(H, np.int32))

    def copy(self) -> "Cache":
        return Cache(self.K.copy(), self.V.copy(), self.code.copy(), self.cnt.copy(), self.stamp.copy(),
                     self.len.copy())


def tempcache_compress(cache: Cache, R, qscale, shift, K_new, V_new, P_new=None, cand=None, metric: int = 0,
                       tau2_q16: int = 53084, frame_id: int = 0, rep_mode: int = 0):
    """Merge one frame of tokens into ``cache`` in place.  Returns (merge_map, merged, stats).
    rep_mode: 0 keeps the last key of a merged group, 1 its multiplicity-weighted mean key."""
    H, C, d = cache.K.shape
    r = cache.code.shape[2]
    K_new = _c(K_new)
    V_new = _c(V_new)
    assert K_new.dtype == cache.K.dtype and V_new.dtype == cache.K.dtype
    assert K_new.shape[0] == H and K_new.shape[2] == d and V_new.shape == K_new.shape
    n_new = K_new.shape[1]
    if P_new is not None:
        P_new = _c(P_new)
        assert P_new.shape == K_new.shape and P_new.dtype == K_new.dtype
    n_cand = 0
    if cand is not None:
        cand = _c(cand, np.int32)
        assert cand.shape[0] == H
        n_cand = cand.shape[1]
    R = _c(R, np.int8)
    for a in (cache.K, cache.V, cache.code, cache.cnt, cache.stamp, cache.len):
        assert a.flags.c_contiguous
    merge_map = np.empty((H, n_new), np.int32)
    merged = np.empty((H, n_new), np.uint8)
    stats = np.zeros((H, 8), np.int32)
    rc = _load().oracle_tempcache_compress(
        _p(cache.K), _p(cache.V), _p(cache.code), _p(cache.cnt), _p(cache.stamp), _p(cache.len), H, C, d, r,
        _dtype_code(cache.K), _p(R), ctypes.c_float(float(np.float32(qscale))), int(shift),
        _p(K_new), _p(V_new), _p(P_new), n_new, _p(cand), n_cand, int(metric), ctypes.c_int32(int(tau2_q16)),
        ctypes.c_int32(int(frame_id)), int(rep_mode), _p(merge_map), _p(merged), _p(stats))
    _check(rc, "oracle_tempcache_compress")
    return merge_map, merged, stats


def ann_select_self(qcode, kcode, length, BQ: int, n_rep: int, BK: int, n_sel: int, n_sink: int = 0, n_local: int = 0):
    """qcode [H,n_q,r], kcode [H,C,r], length [H] -> (sel [H,n_qb,n_sel] ascending / -1 padded, nsel [H,n_qb]).
    n_sink / n_local: first / last live key blocks that are always selected (they count against n_sel)."""
    qcode = _c(qcode, np.int8)
    kcode = _c(kcode, np.int8)
    length = _c(length, np.int32)
    H, n_q, r = qcode.shape
    C = kcode.shape[1]
    n_qb = (n_q + BQ - 1) // BQ
    sel = np.empty((H, n_qb, n_sel), np.int32)
    nsel = np.empty((H, n_qb), np.int32)
    rc = _load().oracle_ann_select_self_forced(_p(qcode), n_q, _p(kcode), _p(length), H, C, r, BQ, n_rep, BK, n_sel,
                                               n_sink, n_local, _p(sel), _p(nsel))
    _check(rc, "oracle_ann_select_self_forced")
    return sel, nsel


def prompt_buckets(code, pcode, m: int = 1):
    """code [H,n,r], pcode [H,n_p,r] -> bucket [H,n,m]: the m nearest prompt tokens of every code (best first)."""
    code = _c(code, np.int8)
    pcode = _c(pcode, np.int8)
    H, n, r = code.shape
    n_p = pcode.shape[1]
    bucket = np.empty((H, n, m), np.int32)
    _check(_load().oracle_prompt_buckets(_p(code), n, _p(pcode), n_p, H, r, m, _p(bucket)), "oracle_prompt_buckets")
    return bucket


def ann_select_buckets(qbucket, kbucket, length, n_p: int, BQ: int, BK: int, n_sel: int, n_sink: int = 0,
                       n_local: int = 0):
    """qbucket [H,n_q,m], kbucket [H,C,m], length [H] -> (sel [H,n_qb,n_sel], nsel): key blocks that share a
    prompt-induced bucket with the query block, the n_sel with the most shared buckets."""
    qbucket = _c(qbucket, np.int32)
    kbucket = _c(kbucket, np.int32)
    length = _c(length, np.int32)
    H, n_q, m = qbucket.shape
    C = kbucket.shape[1]
    n_qb = (n_q + BQ - 1) // BQ
    sel = np.empty((H, n_qb, n_sel), np.int32)
    nsel = np.empty((H, n_qb), np.int32)
    _check(_load().oracle_ann_select_buckets(_p(qbucket), n_q, _p(kbucket), _p(length), H, C, m, n_p, BQ, BK, n_sel,
                                             n_sink, n_local, _p(sel), _p(nsel)), "oracle_ann_select_buckets")
    return sel, nsel


def ann_select_cross(qcode, pcode, BQ: int, n_sel: int):
    """qcode [H,n_q,r], pcode [H,n_p,r] -> (sel [H,n_qb,n_sel] prompt-token ids ascending, nsel)."""
    qcode = _c(qcode, np.int8)
    pcode = _c(pcode, np.int8)
    H, n_q, r = qcode.shape
    n_p = pcode.shape[1]
    n_qb = (n_q + BQ - 1) // BQ
    sel = np.empty((H, n_qb, n_sel), np.int32)
    nsel = np.empty((H, n_qb), np.int32)
    rc = _load().oracle_ann_select_cross(_p(qcode), n_q, _p(pcode), n_p, H, r, BQ, n_sel, _p(sel), _p(nsel))
    _check(rc, "oracle_ann_select_cross")
    return sel, nsel


def encode_sign(x, R, qscale: float):
    """x [..., d] storage form, R [d, n_bits] int8 (+-1) -> bits [..., n_bits/32] uint32 (Sec. 5.1, LSH paragraph)."""
    x = _c(x)
    R = _c(R, np.int8)
    d, n_bits = R.shape
    assert x.shape[-1] == d and n_bits % 32 == 0
    n_vec = int(np.prod(x.shape[:-1]))
    bits = np.empty(x.shape[:-1] + (n_bits // 32,), np.uint32)
    rc = _load().oracle_encode_sign(_p(x), _dtype_code(x), ctypes.c_int64(n_vec), d, _p(R), n_bits,
                                    ctypes.c_float(float(np.float32(qscale))), _p(bits))
    _check(rc, "oracle_encode_sign")
    return bits


def ann_select_lsh(qbits, kbits, length, BQ: int, n_rep: int, BK: int, n_sel: int):
    """qbits [H,n_q,W], kbits [H,C,W] uint32, length [H] -> (sel [H,n_qb,n_sel] ascending / -1 padded, nsel)."""
    qbits = _c(qbits, np.uint32)
    kbits = _c(kbits, np.uint32)
    length = _c(length, np.int32)
    H, n_q, W = qbits.shape
    C = kbits.shape[1]
    n_qb = (n_q + BQ - 1) // BQ
    sel = np.empty((H, n_qb, n_sel), np.int32)
    nsel = np.empty((H, n_qb), np.int32)
    rc = _load().oracle_ann_select_lsh(_p(qbits), n_q, _p(kbits), _p(length), H, C, 32 * W, BQ, n_rep, BK, n_sel,
                                       _p(sel), _p(nsel))
    _check(rc, "oracle_ann_select_lsh")
    return sel, nsel


def ann_select_lsh_buckets(qbits, kbits, length, band_bits: int, radius: int, BQ: int, n_rep: int, BK: int, n_sel: int,
                           n_sink: int = 0, n_local: int = 0):
    """Hash-table form of ann_select_lsh: bands of band_bits bits are the tables, a pair collides in a table when its
    buckets differ in at most `radius` bits; key blocks without a collision are no candidates."""
    qbits = _c(qbits, np.uint32)
    kbits = _c(kbits, np.uint32)
    length = _c(length, np.int32)
    H, n_q, W = qbits.shape
    C = kbits.shape[1]
    n_qb = (n_q + BQ - 1) // BQ
    sel = np.empty((H, n_qb, n_sel), np.int32)
    nsel = np.empty((H, n_qb), np.int32)
    rc = _load().oracle_ann_select_lsh_buckets(_p(qbits), n_q, _p(kbits), _p(length), H, C, 32 * W, band_bits, radius,
                                               BQ, n_rep, BK, n_sel, n_sink, n_local, _p(sel), _p(nsel))
    _check(rc, "oracle_ann_select_lsh_buckets")
    return sel, nsel


def sparse_attn_fwd(Q, K, V, cnt, length, sel, nsel, BQ: int, BK: int, scale: float):
    """Block-sparse attention in fp64.  Returns (O [H,n_q,d] float64, lse [H,n_q] float64)."""
    Q = _c(Q)
    K = _c(K)
    V = _c(V)
    assert Q.dtype == K.dtype == V.dtype
    H, n_q, d = Q.shape
    C = K.shape[1]
    length = _c(length, np.int32)
    sel = _c(sel, np.int32)
    nsel = _c(nsel, np.int32)
    n_sel = sel.shape[2]
    if cnt is not None:
        cnt = _c(cnt, np.int32)
    O = np.empty((H, n_q, d), np.float64)
    lse = np.empty((H, n_q), np.float64)
    rc = _load().oracle_sparse_attn_fwd(_p(Q), n_q, _p(K), _p(V), _p(cnt), _p(length), H, C, d, _dtype_code(Q),
                                        _p(sel), _p(nsel), BQ, BK, n_sel, ctypes.c_double(scale), _p(O), _p(lse))
    _check(rc, "oracle_sparse_attn_fwd")
    return O, lse


def recall_density(Q, K, cnt, length, sel, nsel, BQ: int, BK: int, scale: float, q_stride: int = 1):
    """Attention recall and density of a selection (on every q_stride-th query)."""
    Q = _c(Q)
    K = _c(K)
    H, n_q, d = Q.shape
    C = K.shape[1]
    length = _c(length, np.int32)
    sel = _c(sel, np.int32)
    nsel = _c(nsel, np.int32)
    if cnt is not None:
        cnt = _c(cnt, np.int32)
    out = np.zeros(2, np.float64)
    rc = _load().oracle_recall_density(_p(Q), n_q, _p(K), _p(cnt), _p(length), H, C, d, _dtype_code(Q), _p(sel),
                                       _p(nsel), BQ, BK, sel.shape[2], ctypes.c_double(scale), int(q_stride), _p(out))
    _check(rc, "oracle_recall_density")
    return float(out[0]), float(out[1])


def full_selection(H: int, n_q: int, BQ: int, length, BK: int):
    """Selection that lists every live key block (the dense limit)."""
    length = np.asarray(length, np.int32)
    n_qb = (n_q + BQ - 1) // BQ
    n_kb = int((int(length.max()) + BK - 1) // BK) if length.size else 0
    n_sel = max(n_kb, 1)
    sel = np.full((H, n_qb, n_sel), -1, np.int32)
    nsel = np.zeros((H, n_qb), np.int32)
    for h in range(H):
        m = int((int(length[h]) + BK - 1) // BK)
        sel[h, :, :m] = np.arange(m, dtype=np.int32)
        nsel[h, :] = m
    return sel, nsel


# ---------------------------------------------------------------------------------------------- fp8 K/V


def fp8_encode(x: np.ndarray) -> np.ndarray:
    """float32 values -> E4M3 codes (uint8), nearest with ties to even, saturating at 448."""
    x = _c(x, np.float32)
    code = np.empty(x.shape, np.uint8)
    _check(_load().oracle_fp8_encode(_p(x), ctypes.c_int64(x.size), _p(code)), "oracle_fp8_encode")
    return code


def fp8_decode(code: np.ndarray) -> np.ndarray:
    """E4M3 codes -> their exact values (float64)."""
    code = _c(code, np.uint8)
    x = np.empty(code.shape, np.float64)
    _check(_load().oracle_fp8_decode(_p(code), ctypes.c_int64(code.size), _p(x)), "oracle_fp8_decode")
    return x


def kv8_empty(H: int, C: int, d: int):
    """Zero-filled (K8 [H,Cp,d], V8T [H,Cp/64,d,64]) for a cache of capacity C."""
    n_blk = (C + 63) // 64
    return np.zeros((H, n_blk * 64, d), np.uint8), np.zeros((H, n_blk, d, 64), np.uint8)


def kv_to_fp8(cache: Cache, K8: np.ndarray, V8T: np.ndarray, stamp_lo: int = -2 ** 31):
    """(Re)write in place the blocks of the 8-bit cache copy that hold a live slot with stamp >= stamp_lo."""
    H, C, d = cache.K.shape
    n_blk = (C + 63) // 64
    assert K8.shape == (H, n_blk * 64, d) and V8T.shape == (H, n_blk, d, 64)
    assert K8.dtype == np.uint8 and V8T.dtype == np.uint8 and K8.flags.c_contiguous and V8T.flags.c_contiguous
    rc = _load().oracle_kv_to_fp8(_p(_c(cache.K)), _p(_c(cache.V)), _p(_c(cache.stamp, np.int32)),
                                  _p(_c(cache.len, np.int32)), H, C, d, _dtype_code(cache.K), ctypes.c_int32(stamp_lo),
                                  _p(K8), _p(V8T))
    _check(rc, "oracle_kv_to_fp8")


def sparse_attn_fwd_fp8(Q, K8, V8T, cnt, length, C: int, sel, nsel, BQ: int, BK: int, scale: float):
    """Attention over the 8-bit cache copy: (O [H,n_q,d] float64, lse [H,n_q] float64)."""
    Q = _c(Q)
    H, n_q, d = Q.shape
    sel = _c(sel, np.int32)
    nsel = _c(nsel, np.int32)
    n_sel = sel.shape[2]
    O = np.empty((H, n_q, d), np.float64)
    lse = np.empty((H, n_q), np.float64)
    rc = _load().oracle_sparse_attn_fwd_fp8(_p(Q), n_q, _p(_c(K8, np.uint8)), _p(_c(V8T, np.uint8)),
                                            _p(None if cnt is None else _c(cnt, np.int32)), _p(_c(length, np.int32)), H, C,
                                            d, _dtype_code(Q), _p(sel), _p(nsel), BQ, BK, n_sel, ctypes.c_double(scale),
                                            _p(O), _p(lse))
    _check(rc, "oracle_sparse_attn_fwd_fp8")
    return O, lse
