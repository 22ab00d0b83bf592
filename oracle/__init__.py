"""CPU oracle for lossless sparse weight synchronisation -- TEST INFRASTRUCTURE.

Thin numpy/ctypes front end of ``srs_oracle.c`` (a plain single-threaded C
statement of Alg. 1's changed-index set, Alg. 2's ``V = W[I]`` and Alg. 3's
scatter, with bit-pattern comparison as goal G1 requires).  Only the tests,
the smoke check and the benchmark's CPU-baseline leg may import this package;
it shares nothing with the GPU library and never imports it.

All weights are numpy ``uint16`` arrays (BF16 bit patterns); indices are
``int32``; counts are ``uint32``.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import List, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "srs_oracle.c")
_LIB = os.path.join(_HERE, "libsrs_oracle.so")

OK = 0
BAD_ARG = -1
BAD_INDEX = -2


def build(force: bool = False) -> str:
    """Compile ``srs_oracle.c`` with gcc (plain -O2, no OpenMP, no tuning)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        subprocess.check_call(["gcc", "-O2", "-Wall", "-Wextra", "-shared", "-fPIC", "-o", _LIB, _SRC])
    return _LIB


def build_sanitized(out: str) -> str:
    """The same source under AddressSanitizer and UndefinedBehaviorSanitizer (gcc), for a run of the CPU tests with
    SRS_ORACLE_LIBRARY pointing at it and gcc's libasan.so preloaded into the interpreter."""
    subprocess.check_call(["gcc", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=undefined", "-Wall", "-Wextra", "-shared", "-fPIC", "-o", out, _SRC])
    return out


_lib = None


def _load():
    global _lib
    if _lib is None:
        # SRS_ORACLE_LIBRARY: another build of the same srs_oracle.c (e.g. with -fsanitize=address,undefined)
        lib = C.CDLL(os.environ.get("SRS_ORACLE_LIBRARY") or build())
        u16p, i32p, u32p, u64p = (C.POINTER(C.c_uint16), C.POINTER(C.c_int32),
                                  C.POINTER(C.c_uint32), C.POINTER(C.c_uint64))
        lib.srs_oracle_extract.restype = C.c_int
        lib.srs_oracle_extract.argtypes = [u16p, u16p, C.c_uint64, C.c_uint64, i32p, u16p, u32p, C.c_uint64, C.c_int]
        lib.srs_oracle_apply.restype = C.c_int
        lib.srs_oracle_apply.argtypes = [u16p, C.c_uint64, C.c_uint64, i32p, u16p, u32p, C.c_uint64]
        pp = C.POINTER(u16p)
        lib.srs_oracle_extract_multi.restype = C.c_int
        lib.srs_oracle_extract_multi.argtypes = [pp, pp, u64p, C.c_uint32, C.c_uint64, C.c_uint64, C.c_uint64,
                                                 i32p, u16p, u32p, C.c_uint64, C.c_int]
        lib.srs_oracle_apply_multi.restype = C.c_int
        lib.srs_oracle_apply_multi.argtypes = [pp, u64p, C.c_uint32, C.c_uint64, C.c_uint64, C.c_uint64,
                                               i32p, u16p, u32p, C.c_uint64]
        u16p_ = C.POINTER(C.c_uint16)
        lib.srs_oracle_encode_indices.restype = C.c_int
        lib.srs_oracle_encode_indices.argtypes = [i32p, u32p, C.c_uint64, C.c_uint64, C.c_uint64, C.c_uint64,
                                                  u16p_, u32p, i32p]
        lib.srs_oracle_decode_indices.restype = C.c_int
        lib.srs_oracle_decode_indices.argtypes = [u16p_, i32p, u32p, u32p, C.c_uint64, C.c_uint64, C.c_uint64, i32p]
        lib.srs_oracle_route.restype = C.c_int
        lib.srs_oracle_route.argtypes = [u32p, C.c_uint64, C.c_uint64, C.c_uint64, C.c_uint64, C.c_uint32, C.c_uint32,
                                         i32p, u32p, i32p, u32p]
        lib.srs_oracle_copy_dense_multi.restype = C.c_int
        lib.srs_oracle_copy_dense_multi.argtypes = [pp, u64p, C.c_uint32, C.c_uint64, i32p, C.c_uint32, u16p_, C.c_int]
        lib.srs_oracle_round_bf16_array.restype = None
        lib.srs_oracle_round_bf16_array.argtypes = [u32p, C.c_uint64, u16p_]
        lib.srs_oracle_extract_cast.restype = C.c_int
        lib.srs_oracle_extract_cast.argtypes = [u16p_, u32p, C.c_uint64, C.c_uint64, i32p, u16p_, u32p, C.c_uint64]
        lib.srs_oracle_extract_cast_multi.restype = C.c_int
        lib.srs_oracle_extract_cast_multi.argtypes = [pp, C.POINTER(u32p), u64p, C.c_uint32, C.c_uint64,
                                                      i32p, u16p_, u32p, C.c_uint64]
        lib.srs_oracle_mark_multi.restype = C.c_int
        lib.srs_oracle_mark_multi.argtypes = [pp, pp, u64p, C.c_uint32, u32p]
        lib.srs_oracle_cast_mark_multi.restype = C.c_int
        lib.srs_oracle_cast_mark_multi.argtypes = [pp, C.POINTER(u32p), u64p, C.c_uint32, u32p]
        lib.srs_oracle_extract_marked_multi.restype = C.c_int
        lib.srs_oracle_extract_marked_multi.argtypes = [pp, u64p, C.c_uint32, C.c_uint64, u32p, i32p, u16p_, u32p,
                                                        C.c_uint64]
        u8p = C.POINTER(C.c_uint8)
        lib.srs_oracle_vc_chunks.restype = C.c_uint64
        lib.srs_oracle_vc_chunks.argtypes = [C.c_uint64]
        lib.srs_oracle_encode_values.restype = C.c_int
        lib.srs_oracle_encode_values.argtypes = [u16p_, u32p, C.c_uint64, C.c_uint64, u8p, u8p, u32p, u32p, u16p_]
        lib.srs_oracle_decode_values.restype = C.c_int
        lib.srs_oracle_decode_values.argtypes = [u8p, u8p, u32p, u32p, C.c_uint64, C.c_uint64, u16p_]
        pp8 = C.POINTER(u8p)
        lib.srs_oracle_extract_u8.restype = C.c_int
        lib.srs_oracle_extract_u8.argtypes = [u8p, u8p, C.c_uint64, C.c_uint64, i32p, u8p, u32p, C.c_uint64, C.c_int]
        lib.srs_oracle_apply_u8.restype = C.c_int
        lib.srs_oracle_apply_u8.argtypes = [u8p, C.c_uint64, C.c_uint64, i32p, u8p, u32p, C.c_uint64]
        lib.srs_oracle_extract_multi_u8.restype = C.c_int
        lib.srs_oracle_extract_multi_u8.argtypes = [pp8, pp8, u64p, C.c_uint32, C.c_uint64, i32p, u8p, u32p, C.c_uint64,
                                                    C.c_int]
        lib.srs_oracle_apply_multi_u8.restype = C.c_int
        lib.srs_oracle_apply_multi_u8.argtypes = [pp8, u64p, C.c_uint32, C.c_uint64, i32p, u8p, u32p, C.c_uint64]
        lib.srs_oracle_tensor_indices.restype = C.c_int
        lib.srs_oracle_tensor_indices.argtypes = [i32p, u32p, u64p, C.c_uint32, C.c_uint64, C.c_uint64, u32p, i32p]
        lib.srs_oracle_num_buckets.restype = C.c_uint64
        lib.srs_oracle_num_buckets.argtypes = [u64p, C.c_uint32, C.c_uint64]
        _lib = lib
    return _lib


def _u16(a: np.ndarray, writable: bool = False) -> np.ndarray:
    if not isinstance(a, np.ndarray) or a.dtype != np.uint16 or a.ndim != 1 or not a.flags.c_contiguous:
        raise TypeError("oracle expects 1-D contiguous numpy uint16 arrays")
    if writable and not a.flags.writeable:
        raise TypeError("array must be writable")
    return a


def _p(a: np.ndarray, ct):
    return a.ctypes.data_as(C.POINTER(ct))


def num_buckets(n: int, be: int) -> int:
    return (n + be - 1) // be


def extract(old: np.ndarray, new: np.ndarray, be: int, cap: int | None = None, refresh: bool = True
            ) -> Tuple[np.ndarray, np.ndarray, np.ndarray, int]:
    """Single tensor.  Returns (I[nb, cap] int32, V[nb, cap] uint16, counts[nb] uint32, n_overflowed).

    ``old`` is refreshed in place to ``new`` when ``refresh`` is true.  Unused payload slots hold
    I = -1, V = 0xFFFF (fill values chosen by this wrapper, never by the C code)."""
    lib = _load()
    _u16(old, True), _u16(new)
    n = old.size
    if new.size != n:
        raise ValueError("size mismatch")
    cap = be if cap is None else cap
    nb = num_buckets(n, be) if be else 0
    I = np.full((nb, max(cap, 0)), -1, np.int32)
    V = np.full((nb, max(cap, 0)), 0xFFFF, np.uint16)
    counts = np.zeros(nb, np.uint32)
    rc = lib.srs_oracle_extract(_p(old, C.c_uint16), _p(new, C.c_uint16), n, be,
                                _p(I, C.c_int32), _p(V, C.c_uint16), _p(counts, C.c_uint32), cap, int(refresh))
    if rc < 0:
        raise ValueError(f"srs_oracle_extract: bad argument ({rc})")
    return I, V, counts, rc


def apply(w: np.ndarray, be: int, I: np.ndarray, V: np.ndarray, counts: np.ndarray) -> int:
    """Single tensor scatter, in place.  Returns OK or BAD_INDEX."""
    lib = _load()
    _u16(w, True)
    I = np.ascontiguousarray(I, np.int32)
    V = np.ascontiguousarray(V, np.uint16)
    counts = np.ascontiguousarray(counts, np.uint32)
    cap = I.shape[1] if I.ndim == 2 else (I.size // max(counts.size, 1))
    rc = lib.srs_oracle_apply(_p(w, C.c_uint16), w.size, be, _p(I, C.c_int32), _p(V, C.c_uint16),
                              _p(counts, C.c_uint32), cap)
    if rc == BAD_ARG:
        raise ValueError("srs_oracle_apply: bad argument")
    return rc


def _ptr_array(arrs: Sequence[np.ndarray | None]):
    T = C.POINTER(C.c_uint16)
    out = (T * max(len(arrs), 1))()
    for k, a in enumerate(arrs):
        out[k] = _p(a, C.c_uint16) if a is not None else T()
    return out


def extract_multi(old: Sequence[np.ndarray | None], new: Sequence[np.ndarray | None], numel: Sequence[int],
                  be: int, cap: int | None = None, b_lo: int = 0, b_hi: int | None = None, refresh: bool = True
                  ) -> Tuple[np.ndarray, np.ndarray, np.ndarray, int]:
    """Tensor list laid end to end; buckets b_lo <= b < b_hi.  Index = position inside the bucket.

    Tensors wholly outside the bucket range may be None."""
    lib = _load()
    nt = len(numel)
    for a in old:
        if a is not None:
            _u16(a, True)
    for a in new:
        if a is not None:
            _u16(a)
    ne = np.asarray(list(numel), np.uint64)
    for k in range(nt):
        if old[k] is not None and (old[k].size != ne[k] or new[k].size != ne[k]):
            raise ValueError("numel mismatch")
    nb = num_buckets(int(ne.sum()), be) if be else 0
    b_hi = nb if b_hi is None else b_hi
    cap = be if cap is None else cap
    m = max(b_hi - b_lo, 0)
    I = np.full((m, max(cap, 0)), -1, np.int32)
    V = np.full((m, max(cap, 0)), 0xFFFF, np.uint16)
    counts = np.zeros(m, np.uint32)
    rc = lib.srs_oracle_extract_multi(_ptr_array(old), _ptr_array(new), _p(ne, C.c_uint64), nt, be, b_lo, b_hi,
                                      _p(I, C.c_int32), _p(V, C.c_uint16), _p(counts, C.c_uint32), cap, int(refresh))
    if rc < 0:
        raise ValueError(f"srs_oracle_extract_multi: bad argument ({rc})")
    return I, V, counts, rc


def apply_multi(w: Sequence[np.ndarray | None], numel: Sequence[int], be: int,
                I: np.ndarray, V: np.ndarray, counts: np.ndarray, b_lo: int = 0, b_hi: int | None = None) -> int:
    lib = _load()
    for a in w:
        if a is not None:
            _u16(a, True)
    ne = np.asarray(list(numel), np.uint64)
    nb = num_buckets(int(ne.sum()), be) if be else 0
    b_hi = nb if b_hi is None else b_hi
    I = np.ascontiguousarray(I, np.int32)
    V = np.ascontiguousarray(V, np.uint16)
    counts = np.ascontiguousarray(counts, np.uint32)
    cap = I.shape[1] if I.ndim == 2 else (I.size // max(counts.size, 1))
    rc = lib.srs_oracle_apply_multi(_ptr_array(w), _p(ne, C.c_uint64), len(numel), be, b_lo, b_hi,
                                    _p(I, C.c_int32), _p(V, C.c_uint16), _p(counts, C.c_uint32), cap)
    if rc == BAD_ARG:
        raise ValueError("srs_oracle_apply_multi: bad argument")
    return rc


ENC_CHUNK = 2048


def encode_indices(I: np.ndarray, counts: np.ndarray, base_stride: int = 0, chunk: int = ENC_CHUNK
                   ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """First differences of each bucket's sorted indices (Sec. 3.3).  Returns (D[nb, cap] uint16,
    max_gap[nb] uint32, anchors[nb, ceil(cap/chunk)] int32); unused slots hold 0xFFFF / -1."""
    lib = _load()
    I = np.ascontiguousarray(I, np.int32)
    counts = np.ascontiguousarray(counts, np.uint32)
    nb, cap = I.shape
    D = np.full((nb, cap), 0xFFFF, np.uint16)
    max_gap = np.zeros(nb, np.uint32)
    anchors = np.full((nb, (cap + chunk - 1) // chunk), -1, np.int32)
    rc = lib.srs_oracle_encode_indices(_p(I, C.c_int32), _p(counts, C.c_uint32), nb, cap, base_stride, chunk,
                                       _p(D, C.c_uint16), _p(max_gap, C.c_uint32), _p(anchors, C.c_int32))
    if rc != OK:
        raise ValueError(f"srs_oracle_encode_indices: {rc}")
    return D, max_gap, anchors


def decode_indices(D: np.ndarray, I_wide: np.ndarray, counts: np.ndarray, max_gap: np.ndarray, base_stride: int = 0
                   ) -> np.ndarray:
    """Running sums of the differences; buckets with max_gap >= 2^15 are taken from I_wide."""
    lib = _load()
    D = np.ascontiguousarray(D, np.uint16)
    I_wide = np.ascontiguousarray(I_wide, np.int32)
    counts = np.ascontiguousarray(counts, np.uint32)
    max_gap = np.ascontiguousarray(max_gap, np.uint32)
    nb, cap = D.shape
    out = np.full((nb, cap), -1, np.int32)
    rc = lib.srs_oracle_decode_indices(_p(D, C.c_uint16), _p(I_wide, C.c_int32), _p(counts, C.c_uint32),
                                       _p(max_gap, C.c_uint32), nb, cap, base_stride, _p(out, C.c_int32))
    if rc != OK:
        raise ValueError(f"srs_oracle_decode_indices: {rc}")
    return out


def route(counts: np.ndarray, be: int, total: int, cap: int, bytes_per_pair: int = 6, max_dense: int | None = None
          ) -> Tuple[np.ndarray, np.ndarray, np.ndarray, int, int]:
    """Per-bucket sparse / dense decision (Sec. 3.4 routing with the Eq. (1) break-even).
    Returns (route_slot[nb] int32, sparse_counts[nb] uint32, dense_bucket[max_dense] int32, n_dense, n_dropped)."""
    lib = _load()
    counts = np.ascontiguousarray(counts, np.uint32)
    nb = counts.size
    max_dense = nb if max_dense is None else max_dense
    slot = np.full(nb, -9, np.int32)
    sc = np.zeros(nb, np.uint32)
    db = np.full(max(max_dense, 1), -1, np.int32)
    nd = C.c_uint32(0)
    rc = lib.srs_oracle_route(_p(counts, C.c_uint32), nb, be, total, cap, bytes_per_pair, max_dense,
                              _p(slot, C.c_int32), _p(sc, C.c_uint32), _p(db, C.c_int32), C.byref(nd))
    if rc < 0:
        raise ValueError("srs_oracle_route: bad argument")
    return slot, sc, db, nd.value, rc


def copy_dense_multi(w: Sequence[np.ndarray], numel: Sequence[int], be: int, dense_bucket: np.ndarray, n_dense: int,
                     dense: np.ndarray, pack: bool) -> None:
    """pack: dense[s] <- bucket dense_bucket[s] of the list; else the list <- dense[s]."""
    lib = _load()
    for a in w:
        _u16(a, True)
    ne = np.asarray(list(numel), np.uint64)
    db = np.ascontiguousarray(dense_bucket, np.int32)
    if dense.dtype != np.uint16 or not dense.flags.c_contiguous or dense.size < n_dense * be:
        raise TypeError("dense: contiguous uint16 of at least n_dense*be elements")
    rc = lib.srs_oracle_copy_dense_multi(_ptr_array(w), _p(ne, C.c_uint64), len(numel), be, _p(db, C.c_int32), n_dense,
                                         _p(dense, C.c_uint16), int(pack))
    if rc != OK:
        raise ValueError("srs_oracle_copy_dense_multi: bad argument")


def _f32bits(a: np.ndarray) -> np.ndarray:
    if not isinstance(a, np.ndarray) or a.dtype not in (np.float32, np.uint32) or a.ndim != 1 or not a.flags.c_contiguous:
        raise TypeError("master weights: 1-D contiguous float32 (or their uint32 bit patterns)")
    return a.view(np.uint32)


def round_bf16(master: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even binary32 -> BF16 bit patterns (NaN -> 0x7FC0)."""
    lib = _load()
    m = _f32bits(master)
    out = np.empty(m.size, np.uint16)
    lib.srs_oracle_round_bf16_array(_p(m, C.c_uint32), m.size, _p(out, C.c_uint16))
    return out


def extract_cast(w: np.ndarray, master: np.ndarray, be: int, cap: int | None = None
                 ) -> Tuple[np.ndarray, np.ndarray, np.ndarray, int]:
    """Fused cast + diff of Alg. 1 on one tensor: w (BF16 patterns, in/out) <- round_bf16(master)."""
    lib = _load()
    _u16(w, True)
    m = _f32bits(master)
    if m.size != w.size:
        raise ValueError("size mismatch")
    cap = be if cap is None else cap
    nb = num_buckets(w.size, be) if be else 0
    I = np.full((nb, max(cap, 0)), -1, np.int32)
    V = np.full((nb, max(cap, 0)), 0xFFFF, np.uint16)
    counts = np.zeros(nb, np.uint32)
    rc = lib.srs_oracle_extract_cast(_p(w, C.c_uint16), _p(m, C.c_uint32), w.size, be, _p(I, C.c_int32),
                                     _p(V, C.c_uint16), _p(counts, C.c_uint32), cap)
    if rc < 0:
        raise ValueError(f"srs_oracle_extract_cast: bad argument ({rc})")
    return I, V, counts, rc


def extract_cast_multi(w: Sequence[np.ndarray], master: Sequence[np.ndarray], numel: Sequence[int], be: int,
                       cap: int | None = None) -> Tuple[np.ndarray, np.ndarray, np.ndarray, int]:
    lib = _load()
    for a in w:
        _u16(a, True)
    ms = [_f32bits(a) for a in master]
    ne = np.asarray(list(numel), np.uint64)
    nb = num_buckets(int(ne.sum()), be) if be else 0
    cap = be if cap is None else cap
    I = np.full((nb, max(cap, 0)), -1, np.int32)
    V = np.full((nb, max(cap, 0)), 0xFFFF, np.uint16)
    counts = np.zeros(nb, np.uint32)
    T = C.POINTER(C.c_uint32)
    mp = (T * max(len(ms), 1))()
    for k, a in enumerate(ms):
        mp[k] = _p(a, C.c_uint32)
    rc = lib.srs_oracle_extract_cast_multi(_ptr_array(w), mp, _p(ne, C.c_uint64), len(numel), be, _p(I, C.c_int32),
                                           _p(V, C.c_uint16), _p(counts, C.c_uint32), cap)
    if rc < 0:
        raise ValueError(f"srs_oracle_extract_cast_multi: bad argument ({rc})")
    return I, V, counts, rc


def bitmap_words(total: int) -> int:
    return (total + 31) // 32


def _master_ptrs(ms):
    T = C.POINTER(C.c_uint32)
    mp = (T * max(len(ms), 1))()
    for k, a in enumerate(ms):
        mp[k] = _p(a, C.c_uint32)
    return mp


def mark_multi(prev: Sequence[np.ndarray], cur: Sequence[np.ndarray], numel: Sequence[int], bitmap: np.ndarray) -> None:
    """bitmap |= (cur != prev): one optimizer step of Alg. 1's index accumulation."""
    lib = _load()
    for a in list(prev) + list(cur):
        _u16(a)
    ne = np.asarray(list(numel), np.uint64)
    if bitmap.dtype != np.uint32 or bitmap.size < bitmap_words(int(ne.sum())):
        raise TypeError("bitmap: uint32 array of ceil(total/32) words")
    lib.srs_oracle_mark_multi(_ptr_array(prev), _ptr_array(cur), _p(ne, C.c_uint64), len(numel), _p(bitmap, C.c_uint32))


def cast_mark_multi(w: Sequence[np.ndarray], master: Sequence[np.ndarray], numel: Sequence[int], bitmap: np.ndarray) -> None:
    """w <- round_bf16(master); bitmap |= changed (Alg. 1 lines 4-7 without the clone)."""
    lib = _load()
    for a in w:
        _u16(a, True)
    ms = [_f32bits(a) for a in master]
    ne = np.asarray(list(numel), np.uint64)
    if bitmap.dtype != np.uint32 or bitmap.size < bitmap_words(int(ne.sum())):
        raise TypeError("bitmap: uint32 array of ceil(total/32) words")
    lib.srs_oracle_cast_mark_multi(_ptr_array(w), _master_ptrs(ms), _p(ne, C.c_uint64), len(numel), _p(bitmap, C.c_uint32))


def extract_marked_multi(w: Sequence[np.ndarray], numel: Sequence[int], be: int, bitmap: np.ndarray,
                         cap: int | None = None) -> Tuple[np.ndarray, np.ndarray, np.ndarray, int]:
    """Per-bucket payload of the marked positions with the current values (Alg. 2 over the cumulative set)."""
    lib = _load()
    for a in w:
        _u16(a)
    ne = np.asarray(list(numel), np.uint64)
    nb = num_buckets(int(ne.sum()), be) if be else 0
    cap = be if cap is None else cap
    I = np.full((nb, max(cap, 0)), -1, np.int32)
    V = np.full((nb, max(cap, 0)), 0xFFFF, np.uint16)
    counts = np.zeros(nb, np.uint32)
    rc = lib.srs_oracle_extract_marked_multi(_ptr_array(w), _p(ne, C.c_uint64), len(numel), be, _p(bitmap, C.c_uint32),
                                             _p(I, C.c_int32), _p(V, C.c_uint16), _p(counts, C.c_uint32), cap)
    if rc < 0:
        raise ValueError("srs_oracle_extract_marked_multi: bad argument")
    return I, V, counts, rc


VC_CHUNK, VC_SLOT_WORDS, VC_SUB, VC_MAXLEN = 2048, 768, 64, 12


def encode_values(V: np.ndarray, counts: np.ndarray):
    """Huffman coding of the high bytes of each bucket's values (Sec. 3.3, value entropy coding).
    Returns dict(lens[nb,256] u8, low[nb,cap] u8, bits[nb,nchunk,768] u32, chunk_words[nb,nchunk] u32,
    sub[nb,nchunk,32] u16); unused entries hold 0xFF / 0xFFFFFFFF / 0xFFFF fill."""
    lib = _load()
    V = np.ascontiguousarray(V, np.uint16)
    counts = np.ascontiguousarray(counts, np.uint32)
    nb, cap = V.shape
    nchunk = (cap + VC_CHUNK - 1) // VC_CHUNK
    out = {"lens": np.full((nb, 256), 0xFF, np.uint8), "low": np.full((nb, cap), 0xFF, np.uint8),
           "bits": np.full((nb, nchunk, VC_SLOT_WORDS), 0xFFFFFFFF, np.uint32),
           "chunk_words": np.full((nb, nchunk), 0xFFFFFFFF, np.uint32), "sub": np.full((nb, nchunk, 32), 0xFFFF, np.uint16)}
    rc = lib.srs_oracle_encode_values(_p(V, C.c_uint16), _p(counts, C.c_uint32), nb, cap, _p(out["lens"], C.c_uint8),
                                      _p(out["low"], C.c_uint8), _p(out["bits"], C.c_uint32),
                                      _p(out["chunk_words"], C.c_uint32), _p(out["sub"], C.c_uint16))
    if rc != OK:
        raise ValueError("srs_oracle_encode_values: bad argument")
    return out


def decode_values(enc: dict, counts: np.ndarray) -> np.ndarray:
    lib = _load()
    counts = np.ascontiguousarray(counts, np.uint32)
    nb, cap = enc["low"].shape
    V = np.full((nb, cap), 0xFFFF, np.uint16)
    rc = lib.srs_oracle_decode_values(_p(enc["lens"], C.c_uint8), _p(enc["low"], C.c_uint8), _p(enc["bits"], C.c_uint32),
                                      _p(counts, C.c_uint32), nb, cap, _p(V, C.c_uint16))
    if rc != OK:
        raise ValueError(f"srs_oracle_decode_values: {rc}")
    return V


# ---------------------------------------------------------------------------------------------
# one-byte elements (FP8 synchronisation precision, Sec. 2.1): uint8 patterns, V is uint8
# ---------------------------------------------------------------------------------------------
def _u8(a: np.ndarray, writable: bool = False) -> np.ndarray:
    if not isinstance(a, np.ndarray) or a.dtype != np.uint8 or a.ndim != 1 or not a.flags.c_contiguous:
        raise TypeError("oracle expects 1-D contiguous numpy uint8 arrays")
    if writable and not a.flags.writeable:
        raise TypeError("array must be writable")
    return a


def _ptr_array_u8(arrs: Sequence[np.ndarray]):
    T = C.POINTER(C.c_uint8)
    out = (T * max(len(arrs), 1))()
    for k, a in enumerate(arrs):
        out[k] = _p(a, C.c_uint8)
    return out


def extract_u8(old: np.ndarray, new: np.ndarray, be: int, cap: int | None = None, refresh: bool = True
               ) -> Tuple[np.ndarray, np.ndarray, np.ndarray, int]:
    """Single tensor of one-byte elements.  Returns (I[nb, cap] int32, V[nb, cap] uint8, counts[nb] uint32,
    n_overflowed); unused slots hold I = -1, V = 0xFF (this wrapper's fill values)."""
    lib = _load()
    _u8(old, True), _u8(new)
    n = old.size
    if new.size != n:
        raise ValueError("size mismatch")
    cap = be if cap is None else cap
    nb = num_buckets(n, be) if be else 0
    I = np.full((nb, max(cap, 0)), -1, np.int32)
    V = np.full((nb, max(cap, 0)), 0xFF, np.uint8)
    counts = np.zeros(nb, np.uint32)
    rc = lib.srs_oracle_extract_u8(_p(old, C.c_uint8), _p(new, C.c_uint8), n, be,
                                   _p(I, C.c_int32), _p(V, C.c_uint8), _p(counts, C.c_uint32), cap, int(refresh))
    if rc < 0:
        raise ValueError(f"srs_oracle_extract_u8: bad argument ({rc})")
    return I, V, counts, rc


def apply_u8(w: np.ndarray, be: int, I: np.ndarray, V: np.ndarray, counts: np.ndarray) -> int:
    lib = _load()
    _u8(w, True)
    I = np.ascontiguousarray(I, np.int32)
    V = np.ascontiguousarray(V, np.uint8)
    counts = np.ascontiguousarray(counts, np.uint32)
    cap = I.shape[1] if I.ndim == 2 else (I.size // max(counts.size, 1))
    rc = lib.srs_oracle_apply_u8(_p(w, C.c_uint8), w.size, be, _p(I, C.c_int32), _p(V, C.c_uint8),
                                 _p(counts, C.c_uint32), cap)
    if rc == BAD_ARG:
        raise ValueError("srs_oracle_apply_u8: bad argument")
    return rc


def extract_multi_u8(old: Sequence[np.ndarray], new: Sequence[np.ndarray], numel: Sequence[int], be: int,
                     cap: int | None = None, refresh: bool = True) -> Tuple[np.ndarray, np.ndarray, np.ndarray, int]:
    """Tensor list of one-byte elements laid end to end, all buckets; index = position inside the bucket."""
    lib = _load()
    for a in old:
        _u8(a, True)
    for a in new:
        _u8(a)
    ne = np.asarray(list(numel), np.uint64)
    for k in range(len(numel)):
        if old[k].size != ne[k] or new[k].size != ne[k]:
            raise ValueError("numel mismatch")
    nb = num_buckets(int(ne.sum()), be) if be else 0
    cap = be if cap is None else cap
    I = np.full((nb, max(cap, 0)), -1, np.int32)
    V = np.full((nb, max(cap, 0)), 0xFF, np.uint8)
    counts = np.zeros(nb, np.uint32)
    rc = lib.srs_oracle_extract_multi_u8(_ptr_array_u8(old), _ptr_array_u8(new), _p(ne, C.c_uint64), len(numel), be,
                                         _p(I, C.c_int32), _p(V, C.c_uint8), _p(counts, C.c_uint32), cap, int(refresh))
    if rc < 0:
        raise ValueError(f"srs_oracle_extract_multi_u8: bad argument ({rc})")
    return I, V, counts, rc


def apply_multi_u8(w: Sequence[np.ndarray], numel: Sequence[int], be: int, I: np.ndarray, V: np.ndarray,
                   counts: np.ndarray) -> int:
    lib = _load()
    for a in w:
        _u8(a, True)
    ne = np.asarray(list(numel), np.uint64)
    I = np.ascontiguousarray(I, np.int32)
    V = np.ascontiguousarray(V, np.uint8)
    counts = np.ascontiguousarray(counts, np.uint32)
    cap = I.shape[1] if I.ndim == 2 else (I.size // max(counts.size, 1))
    rc = lib.srs_oracle_apply_multi_u8(_ptr_array_u8(w), _p(ne, C.c_uint64), len(numel), be,
                                       _p(I, C.c_int32), _p(V, C.c_uint8), _p(counts, C.c_uint32), cap)
    if rc == BAD_ARG:
        raise ValueError("srs_oracle_apply_multi_u8: bad argument")
    return rc


def tensor_indices(I: np.ndarray, counts: np.ndarray, numel: Sequence[int], be: int) -> Tuple[np.ndarray, np.ndarray, int]:
    """Per-tensor view of a list payload (Alg. 2's int32 index into each tensor): returns (tensor_id[nb, cap] uint32,
    tensor_idx[nb, cap] int32, rc); unused slots hold 0xFFFFFFFF / -1 (this wrapper's fill values)."""
    lib = _load()
    I = np.ascontiguousarray(I, np.int32)
    counts = np.ascontiguousarray(counts, np.uint32)
    ne = np.asarray(list(numel), np.uint64)
    nb, cap = I.shape
    tid = np.full((nb, cap), 0xFFFFFFFF, np.uint32)
    tix = np.full((nb, cap), -1, np.int32)
    rc = lib.srs_oracle_tensor_indices(_p(I, C.c_int32), _p(counts, C.c_uint32), _p(ne, C.c_uint64), len(numel), be, cap,
                                       _p(tid, C.c_uint32), _p(tix, C.c_int32))
    if rc == BAD_ARG:
        raise ValueError("srs_oracle_tensor_indices: bad argument")
    return tid, tix, rc
