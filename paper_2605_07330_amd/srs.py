"""ctypes binding of libsrs.so -- argument marshalling only; every step runs in the HIP kernels.

The names follow include/srs.h: ``Context.extract / apply / extract_multi / apply_multi`` call
``srs_extract / srs_apply / srs_extract_multi / srs_apply_multi``.  Tensors are torch CUDA
(ROCm) tensors used purely as device memory; the current torch stream is passed through.

Importing this module fails loudly when the library has not been built
(``python -m paper_2605_07330_amd.build``): there is no CPU fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import torch  # loads the HIP runtime that libsrs.so binds to

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("SRS_LIBRARY") or os.path.join(_HERE, "libsrs.so")   # override: a build of the same ABI

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2605_07330_amd.build` "
                      "(hipcc --offload-arch=gfx950); there is no fallback path")

_lib = C.CDLL(LIB_PATH)

OK, ERR_INVALID, ERR_HIP, ERR_NOMEM, ERR_NO_DEVICE, ERR_TOO_LARGE = 0, -1, -2, -3, -4, -5
FLAG_OVERFLOW, FLAG_BAD_INDEX, FLAG_TIMEOUT = 1, 2, 4
OPT_SPIN_LIMIT, OPT_TILE_ELEMS, OPT_REFRESH_GROUP, OPT_INTERLEAVE, OPT_SNAPSHOT = 1, 2, 3, 4, 5
SNAPSHOT_REFRESH, SNAPSHOT_ROTATE, SNAPSHOT_SECOND_PASS = 0, 1, 2

EXPORTS = [
    "srs_create", "srs_destroy", "srs_set_option", "srs_strerror", "srs_version", "srs_status",
    "srs_extract", "srs_apply", "srs_plan_create", "srs_plan_info", "srs_plan_destroy",
    "srs_extract_multi", "srs_apply_multi", "srs_stream_probe", "srs_stream_probe_sink_words",
    "srs_anchor_count", "srs_encode_indices", "srs_apply_encoded", "srs_apply_multi_encoded",
    "srs_route", "srs_pack_dense_multi", "srs_unpack_dense_multi",
    "srs_extract_cast", "srs_extract_cast_multi", "srs_plan_layout",
    "srs_bitmap_words", "srs_mark_multi", "srs_cast_mark_multi", "srs_extract_marked_multi",
    "srs_value_chunks", "srs_encode_values", "srs_decode_values",
    "srs_extract_u8", "srs_apply_u8", "srs_extract_multi_u8", "srs_apply_multi_u8", "srs_tensor_indices",
    "srs_extract_noalloc",
]


class TensorPair(C.Structure):
    _fields_ = [("old_snapshot", C.c_void_p), ("new_w", C.c_void_p)]


class Tensor(C.Structure):
    _fields_ = [("weights", C.c_void_p)]


_vp, _u64, _u32p = C.c_void_p, C.c_uint64, C.POINTER(C.c_uint32)
_lib.srs_create.argtypes = [C.POINTER(_vp), C.c_int]
_lib.srs_destroy.argtypes = [_vp]
_lib.srs_set_option.argtypes = [_vp, C.c_int, _u64]
_lib.srs_strerror.argtypes = [C.c_int]
_lib.srs_strerror.restype = C.c_char_p
_lib.srs_version.argtypes = []
_lib.srs_status.argtypes = [_vp, _u32p, _vp]
_lib.srs_extract.argtypes = [_vp, _vp, _vp, _u64, _u64, _vp, _vp, _vp, _u64, _vp]
_lib.srs_apply.argtypes = [_vp, _vp, _u64, _u64, _vp, _vp, _vp, _u64, _vp]
_lib.srs_extract_noalloc.argtypes = _lib.srs_extract.argtypes
_lib.srs_plan_create.argtypes = [_vp, C.POINTER(_u64), C.c_uint32, _u64, C.POINTER(_vp)]
_lib.srs_plan_info.argtypes = [_vp, C.POINTER(_u64), _u32p, _u32p, _u32p]
_lib.srs_plan_destroy.argtypes = [_vp]
_lib.srs_extract_multi.argtypes = [_vp, _vp, C.POINTER(TensorPair), _vp, _vp, _vp, _u64, _vp]
_lib.srs_apply_multi.argtypes = [_vp, _vp, C.POINTER(Tensor), _vp, _vp, _vp, _u64, _vp]
_lib.srs_extract_u8.argtypes = _lib.srs_extract.argtypes
_lib.srs_apply_u8.argtypes = _lib.srs_apply.argtypes
_lib.srs_extract_multi_u8.argtypes = _lib.srs_extract_multi.argtypes
_lib.srs_apply_multi_u8.argtypes = _lib.srs_apply_multi.argtypes
_lib.srs_tensor_indices.argtypes = [_vp, _vp, _vp, _vp, _u64, _vp, _vp, _vp]
_lib.srs_stream_probe.argtypes = [_vp, _vp, _vp, _u64, _vp, _vp]
_lib.srs_stream_probe_sink_words.argtypes = [_u64]
_lib.srs_stream_probe_sink_words.restype = _u64
_lib.srs_anchor_count.argtypes = [C.c_uint32, _u64]
_lib.srs_anchor_count.restype = _u64
_lib.srs_encode_indices.argtypes = [_vp, _vp, _vp, C.c_uint32, _u64, _u64, _vp, _vp, _vp, _vp]
_lib.srs_apply_encoded.argtypes = [_vp, _vp, _u64, _u64, _vp, _vp, _vp, _vp, _vp, _vp, _u64, _vp]
_lib.srs_apply_multi_encoded.argtypes = [_vp, _vp, C.POINTER(Tensor), _vp, _vp, _vp, _vp, _vp, _vp, _u64, _vp]
_lib.srs_extract_cast.argtypes = [_vp, _vp, _vp, _u64, _u64, _vp, _vp, _vp, _u64, _vp]
_lib.srs_extract_cast_multi.argtypes = [_vp, _vp, C.POINTER(TensorPair), _vp, _vp, _vp, _u64, _vp]
_lib.srs_plan_layout.argtypes = [C.POINTER(_u64), C.c_uint32, _u64, C.c_uint32, C.c_uint32, _u32p, _u32p, _u32p,
                                 _vp, _vp, _vp, _vp, _vp]
_lib.srs_bitmap_words.argtypes = [_u64]
_lib.srs_bitmap_words.restype = _u64
_lib.srs_mark_multi.argtypes = [_vp, _vp, C.POINTER(TensorPair), _vp, _vp]
_lib.srs_cast_mark_multi.argtypes = [_vp, _vp, C.POINTER(TensorPair), _vp, _vp]
_lib.srs_extract_marked_multi.argtypes = [_vp, _vp, C.POINTER(Tensor), _vp, _vp, _vp, _vp, _u64, _vp]
_lib.srs_value_chunks.argtypes = [_u64]
_lib.srs_value_chunks.restype = _u64
_lib.srs_encode_values.argtypes = [_vp, _vp, _vp, C.c_uint32, _u64, _vp, _vp, _vp, _vp, _vp, _vp]
_lib.srs_decode_values.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _vp, C.c_uint32, _u64, _vp, _vp]
_lib.srs_route.argtypes = [_vp, _vp, C.c_uint32, _u64, _u64, _u64, C.c_uint32, C.c_uint32, _vp, _vp, _vp, _vp, _vp]
_lib.srs_pack_dense_multi.argtypes = [_vp, _vp, C.POINTER(TensorPair), _vp, _vp, C.c_uint32, _vp, _vp]
_lib.srs_unpack_dense_multi.argtypes = [_vp, _vp, C.POINTER(Tensor), _vp, _vp, C.c_uint32, _vp, _vp]
for _n in EXPORTS:
    if _n not in ("srs_strerror", "srs_stream_probe_sink_words", "srs_anchor_count", "srs_bitmap_words",
                  "srs_value_chunks"):
        getattr(_lib, _n).restype = C.c_int


class SrsError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {_lib.srs_strerror(code).decode()} ({code})")


def _check(rc: int, where: str) -> None:
    if rc != OK:
        raise SrsError(rc, where)


def version() -> int:
    return _lib.srs_version()


def _stream_ptr(stream: Optional[torch.cuda.Stream]) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


def _dev16(t: torch.Tensor, what: str, width: int = 2) -> None:
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.element_size() == width and t.is_contiguous()):
        raise TypeError(f"{what}: expected a contiguous {8 * width}-bit tensor on the GPU")


def _payload_ok(I: torch.Tensor, V: torch.Tensor, counts: torch.Tensor, nb: int, cap: int, width: int = 2) -> None:
    if not (I.is_cuda and I.dtype == torch.int32 and I.is_contiguous() and I.numel() >= nb * cap):
        raise TypeError("I: expected contiguous int32 GPU tensor of at least nb*cap elements")
    if not (V.is_cuda and V.element_size() == width and V.is_contiguous() and V.numel() >= nb * cap):
        raise TypeError(f"V: expected contiguous {8 * width}-bit GPU tensor of at least nb*cap elements")
    if not (counts.is_cuda and counts.element_size() == 4 and counts.is_contiguous() and counts.numel() >= nb):
        raise TypeError("counts: expected contiguous 32-bit GPU tensor of at least nb elements")


def plan_layout(numel: Sequence[int], bucket_elems: int, tile_elems: int = 32768, interleave: int = 64) -> dict:
    """Host-only view of the tables a plan holds (numpy arrays); needs no GPU."""
    import numpy as np
    numel = [int(x) for x in numel]
    arr = (_u64 * max(len(numel), 1))(*numel)
    nb, ns, nt = C.c_uint32(), C.c_uint32(), C.c_uint32()
    _check(_lib.srs_plan_layout(arr, len(numel), bucket_elems, tile_elems, interleave, C.byref(nb), C.byref(ns),
                                C.byref(nt), None, None, None, None, None), "srs_plan_layout")
    tiles = np.zeros((nt.value, 4), np.uint32); segs = np.zeros((ns.value, 4), np.uint32)
    seg_begin = np.zeros(nb.value + 1, np.uint32); bucket_first = np.zeros(nb.value + 1, np.uint32)
    wg_bucket = np.zeros(nt.value, np.uint32)
    _check(_lib.srs_plan_layout(arr, len(numel), bucket_elems, tile_elems, interleave, None, None, None,
                                tiles.ctypes.data, segs.ctypes.data, seg_begin.ctypes.data, bucket_first.ctypes.data,
                                wg_bucket.ctypes.data), "srs_plan_layout")
    return {"nbuckets": nb.value, "tiles": tiles, "segs": segs, "seg_begin": seg_begin, "bucket_first": bucket_first,
            "wg_bucket": wg_bucket}


def bitmap_words(total_elems: int) -> int:
    return int(_lib.srs_bitmap_words(total_elems))


def stream_probe_sink_words(nbytes: int) -> int:
    return int(_lib.srs_stream_probe_sink_words(nbytes))


def anchor_count(nbuckets: int, cap: int) -> int:
    return int(_lib.srs_anchor_count(nbuckets, cap))


def _encoded_ok(D: torch.Tensor, max_gap: torch.Tensor, anchors: torch.Tensor, nb: int, cap: int) -> None:
    if not (D.is_cuda and D.element_size() == 2 and D.is_contiguous() and D.numel() >= nb * cap):
        raise TypeError("D: expected contiguous 16-bit GPU tensor of at least nb*cap elements")
    if not (max_gap.is_cuda and max_gap.element_size() == 4 and max_gap.is_contiguous() and max_gap.numel() >= nb):
        raise TypeError("max_gap: expected contiguous 32-bit GPU tensor of at least nb elements")
    if not (anchors.is_cuda and anchors.dtype == torch.int32 and anchors.is_contiguous()
            and anchors.numel() >= anchor_count(nb, cap)):
        raise TypeError("anchors: expected contiguous int32 GPU tensor of srs_anchor_count(nb, cap) elements")


class Plan:
    """Bucket / segment / tile tables of one tensor list (srs_plan_*)."""

    def __init__(self, ctx: "Context", numel: Sequence[int], bucket_elems: int):
        self._h = _vp()
        self.numel = [int(x) for x in numel]
        self.bucket_elems = int(bucket_elems)
        arr = (_u64 * max(len(self.numel), 1))(*self.numel)
        _check(_lib.srs_plan_create(ctx._h, arr, len(self.numel), self.bucket_elems, C.byref(self._h)), "srs_plan_create")
        tot, nb, ns, nt = _u64(), C.c_uint32(), C.c_uint32(), C.c_uint32()
        _check(_lib.srs_plan_info(self._h, C.byref(tot), C.byref(nb), C.byref(ns), C.byref(nt)), "srs_plan_info")
        self.total, self.nbuckets, self.nsegments, self.ntiles = tot.value, nb.value, ns.value, nt.value

    def close(self) -> None:
        if self._h:
            _lib.srs_plan_destroy(self._h)
            self._h = _vp()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Context:
    """Per-stream scratch of the library (srs_create / srs_destroy)."""

    def __init__(self, device: int = 0):
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU visible: the sparse-sync hot path has no CPU fallback")
        self._h = _vp()
        self.device = int(device)
        _check(_lib.srs_create(C.byref(self._h), self.device), "srs_create")

    def close(self) -> None:
        if self._h:
            _lib.srs_destroy(self._h)
            self._h = _vp()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_option(self, option: int, value: int) -> None:
        _check(_lib.srs_set_option(self._h, option, int(value)), "srs_set_option")

    def status(self, stream: Optional[torch.cuda.Stream] = None) -> int:
        """Synchronises the stream; returns and clears the device flag word."""
        f = C.c_uint32(0)
        _check(_lib.srs_status(self._h, C.byref(f), _stream_ptr(stream)), "srs_status")
        return f.value

    # ---- single tensor --------------------------------------------------------------------
    def extract(self, old: torch.Tensor, new: torch.Tensor, bucket_elems: int, I: torch.Tensor, V: torch.Tensor,
                counts: torch.Tensor, cap: int, stream: Optional[torch.cuda.Stream] = None) -> None:
        _dev16(old, "old"), _dev16(new, "new")
        n = old.numel()
        if new.numel() != n:
            raise ValueError("old/new size mismatch")
        if bucket_elems > 0 and cap > 0:
            _payload_ok(I, V, counts, (n + bucket_elems - 1) // bucket_elems, cap)
        _check(_lib.srs_extract(self._h, old.data_ptr(), new.data_ptr(), n, bucket_elems, I.data_ptr(), V.data_ptr(),
                                counts.data_ptr(), cap, _stream_ptr(stream)), "srs_extract")

    def extract_noalloc(self, old: torch.Tensor, new: torch.Tensor, bucket_elems: int, I: torch.Tensor,
                        V: torch.Tensor, counts: torch.Tensor, cap: int,
                        stream: Optional[torch.cuda.Stream] = None) -> None:
        """srs_extract on the library's static scratch array: never allocates (see the header for its limits)."""
        _dev16(old, "old"), _dev16(new, "new")
        n = old.numel()
        if new.numel() != n:
            raise ValueError("old/new size mismatch")
        if bucket_elems > 0 and cap > 0:
            _payload_ok(I, V, counts, (n + bucket_elems - 1) // bucket_elems, cap)
        _check(_lib.srs_extract_noalloc(self._h, old.data_ptr(), new.data_ptr(), n, bucket_elems, I.data_ptr(),
                                        V.data_ptr(), counts.data_ptr(), cap, _stream_ptr(stream)),
               "srs_extract_noalloc")

    def apply(self, weights: torch.Tensor, bucket_elems: int, I: torch.Tensor, V: torch.Tensor, counts: torch.Tensor,
              cap: int, stream: Optional[torch.cuda.Stream] = None) -> None:
        _dev16(weights, "weights")
        n = weights.numel()
        if bucket_elems > 0 and cap > 0:
            _payload_ok(I, V, counts, (n + bucket_elems - 1) // bucket_elems, cap)
        _check(_lib.srs_apply(self._h, weights.data_ptr(), n, bucket_elems, I.data_ptr(), V.data_ptr(),
                              counts.data_ptr(), cap, _stream_ptr(stream)), "srs_apply")

    # ---- tensor lists ---------------------------------------------------------------------
    def plan(self, numel: Sequence[int], bucket_elems: int) -> Plan:
        return Plan(self, numel, bucket_elems)

    def bind_pairs(self, plan: Plan, old: Sequence[torch.Tensor], new: Sequence[torch.Tensor], width: int = 2):
        """Marshals (old, new) tensor lists into the srs_tensor_pair[] host array once, for callers
        that repeat the same call (the array can be passed to extract_multi as ``pairs=``)."""
        if len(old) != len(plan.numel) or len(new) != len(plan.numel):
            raise ValueError("tensor list does not match the plan")
        arr = (TensorPair * max(len(old), 1))()
        for k, (o, w) in enumerate(zip(old, new)):
            _dev16(o, f"old[{k}]", width), _dev16(w, f"new[{k}]", width)
            if o.numel() != plan.numel[k] or w.numel() != plan.numel[k]:
                raise ValueError(f"tensor {k}: numel differs from the plan")
            arr[k].old_snapshot, arr[k].new_w = o.data_ptr(), w.data_ptr()
        return arr

    def bind_weights(self, plan: Plan, weights: Sequence[torch.Tensor], width: int = 2):
        if len(weights) != len(plan.numel):
            raise ValueError("tensor list does not match the plan")
        arr = (Tensor * max(len(weights), 1))()
        for k, w in enumerate(weights):
            _dev16(w, f"weights[{k}]", width)
            if w.numel() != plan.numel[k]:
                raise ValueError(f"tensor {k}: numel differs from the plan")
            arr[k].weights = w.data_ptr()
        return arr

    def extract_multi(self, plan: Plan, old: Optional[Sequence[torch.Tensor]], new: Optional[Sequence[torch.Tensor]],
                      I: torch.Tensor, V: torch.Tensor, counts: torch.Tensor, cap: int,
                      stream: Optional[torch.cuda.Stream] = None, pairs=None) -> None:
        if pairs is None:
            pairs = self.bind_pairs(plan, old, new)
        if cap > 0:
            _payload_ok(I, V, counts, plan.nbuckets, cap)
        _check(_lib.srs_extract_multi(self._h, plan._h, pairs, I.data_ptr(), V.data_ptr(), counts.data_ptr(), cap,
                                      _stream_ptr(stream)), "srs_extract_multi")

    def apply_multi(self, plan: Plan, weights: Optional[Sequence[torch.Tensor]], I: torch.Tensor, V: torch.Tensor,
                    counts: torch.Tensor, cap: int, stream: Optional[torch.cuda.Stream] = None, tensors=None) -> None:
        if tensors is None:
            tensors = self.bind_weights(plan, weights)
        if cap > 0:
            _payload_ok(I, V, counts, plan.nbuckets, cap)
        _check(_lib.srs_apply_multi(self._h, plan._h, tensors, I.data_ptr(), V.data_ptr(), counts.data_ptr(), cap,
                                    _stream_ptr(stream)), "srs_apply_multi")

    def tensor_indices(self, plan: Plan, I: torch.Tensor, counts: torch.Tensor, cap: int, tensor_id: torch.Tensor,
                       tensor_idx: torch.Tensor, stream: Optional[torch.cuda.Stream] = None) -> None:
        """Per-tensor view of a list payload: (tensor_id, tensor_idx) laid out like I (32-bit GPU tensors)."""
        for t, what in ((I, "I"), (tensor_id, "tensor_id"), (tensor_idx, "tensor_idx")):
            if not (t.is_cuda and t.element_size() == 4 and t.is_contiguous() and t.numel() >= plan.nbuckets * cap):
                raise TypeError(f"{what}: expected contiguous 32-bit GPU tensor of at least nb*cap elements")
        if not (counts.is_cuda and counts.element_size() == 4 and counts.numel() >= plan.nbuckets):
            raise TypeError("counts: expected 32-bit GPU tensor of at least nb elements")
        _check(_lib.srs_tensor_indices(self._h, plan._h, I.data_ptr(), counts.data_ptr(), cap, tensor_id.data_ptr(),
                                       tensor_idx.data_ptr(), _stream_ptr(stream)), "srs_tensor_indices")

    # ---- one-byte elements (FP8 synchronisation precision) ----------------------------------
    def extract_u8(self, old: torch.Tensor, new: torch.Tensor, bucket_elems: int, I: torch.Tensor, V: torch.Tensor,
                   counts: torch.Tensor, cap: int, stream: Optional[torch.cuda.Stream] = None) -> None:
        _dev16(old, "old", 1), _dev16(new, "new", 1)
        n = old.numel()
        if new.numel() != n:
            raise ValueError("old/new size mismatch")
        if bucket_elems > 0 and cap > 0:
            _payload_ok(I, V, counts, (n + bucket_elems - 1) // bucket_elems, cap, 1)
        _check(_lib.srs_extract_u8(self._h, old.data_ptr(), new.data_ptr(), n, bucket_elems, I.data_ptr(),
                                   V.data_ptr(), counts.data_ptr(), cap, _stream_ptr(stream)), "srs_extract_u8")

    def apply_u8(self, weights: torch.Tensor, bucket_elems: int, I: torch.Tensor, V: torch.Tensor,
                 counts: torch.Tensor, cap: int, stream: Optional[torch.cuda.Stream] = None) -> None:
        _dev16(weights, "weights", 1)
        n = weights.numel()
        if bucket_elems > 0 and cap > 0:
            _payload_ok(I, V, counts, (n + bucket_elems - 1) // bucket_elems, cap, 1)
        _check(_lib.srs_apply_u8(self._h, weights.data_ptr(), n, bucket_elems, I.data_ptr(), V.data_ptr(),
                                 counts.data_ptr(), cap, _stream_ptr(stream)), "srs_apply_u8")

    def extract_multi_u8(self, plan: Plan, old: Optional[Sequence[torch.Tensor]],
                         new: Optional[Sequence[torch.Tensor]], I: torch.Tensor, V: torch.Tensor, counts: torch.Tensor,
                         cap: int, stream: Optional[torch.cuda.Stream] = None, pairs=None) -> None:
        if pairs is None:
            pairs = self.bind_pairs(plan, old, new, 1)
        if cap > 0:
            _payload_ok(I, V, counts, plan.nbuckets, cap, 1)
        _check(_lib.srs_extract_multi_u8(self._h, plan._h, pairs, I.data_ptr(), V.data_ptr(), counts.data_ptr(), cap,
                                         _stream_ptr(stream)), "srs_extract_multi_u8")

    def apply_multi_u8(self, plan: Plan, weights: Optional[Sequence[torch.Tensor]], I: torch.Tensor, V: torch.Tensor,
                       counts: torch.Tensor, cap: int, stream: Optional[torch.cuda.Stream] = None, tensors=None) -> None:
        if tensors is None:
            tensors = self.bind_weights(plan, weights, 1)
        if cap > 0:
            _payload_ok(I, V, counts, plan.nbuckets, cap, 1)
        _check(_lib.srs_apply_multi_u8(self._h, plan._h, tensors, I.data_ptr(), V.data_ptr(), counts.data_ptr(), cap,
                                       _stream_ptr(stream)), "srs_apply_multi_u8")

    # ---- fused cast + diff ----------------------------------------------------------------
    def extract_cast(self, weights: torch.Tensor, master: torch.Tensor, bucket_elems: int, I: torch.Tensor,
                     V: torch.Tensor, counts: torch.Tensor, cap: int, stream: Optional[torch.cuda.Stream] = None) -> None:
        _dev16(weights, "weights")
        if not (master.is_cuda and master.dtype == torch.float32 and master.is_contiguous()
                and master.numel() == weights.numel()):
            raise TypeError("master: expected contiguous float32 GPU tensor of the same numel")
        n = weights.numel()
        if bucket_elems > 0 and cap > 0:
            _payload_ok(I, V, counts, (n + bucket_elems - 1) // bucket_elems, cap)
        _check(_lib.srs_extract_cast(self._h, weights.data_ptr(), master.data_ptr(), n, bucket_elems, I.data_ptr(),
                                     V.data_ptr(), counts.data_ptr(), cap, _stream_ptr(stream)), "srs_extract_cast")

    def bind_cast_pairs(self, plan: Plan, weights: Sequence[torch.Tensor], master: Sequence[torch.Tensor]):
        if len(weights) != len(plan.numel) or len(master) != len(plan.numel):
            raise ValueError("tensor list does not match the plan")
        arr = (TensorPair * max(len(weights), 1))()
        for k, (w, m) in enumerate(zip(weights, master)):
            _dev16(w, f"weights[{k}]")
            if not (m.is_cuda and m.dtype == torch.float32 and m.is_contiguous()):
                raise TypeError(f"master[{k}]: expected contiguous float32 GPU tensor")
            if w.numel() != plan.numel[k] or m.numel() != plan.numel[k]:
                raise ValueError(f"tensor {k}: numel differs from the plan")
            arr[k].old_snapshot, arr[k].new_w = w.data_ptr(), m.data_ptr()
        return arr

    def extract_cast_multi(self, plan: Plan, weights: Optional[Sequence[torch.Tensor]],
                           master: Optional[Sequence[torch.Tensor]], I: torch.Tensor, V: torch.Tensor,
                           counts: torch.Tensor, cap: int, stream: Optional[torch.cuda.Stream] = None, pairs=None) -> None:
        if pairs is None:
            pairs = self.bind_cast_pairs(plan, weights, master)
        if cap > 0:
            _payload_ok(I, V, counts, plan.nbuckets, cap)
        _check(_lib.srs_extract_cast_multi(self._h, plan._h, pairs, I.data_ptr(), V.data_ptr(), counts.data_ptr(), cap,
                                           _stream_ptr(stream)), "srs_extract_cast_multi")

    # ---- cumulative changed-index set (Alg. 1 as printed) ----------------------------------
    @staticmethod
    def _bitmap_ok(plan: Plan, bitmap: torch.Tensor) -> None:
        if not (bitmap.is_cuda and bitmap.element_size() == 4 and bitmap.is_contiguous()
                and bitmap.numel() >= bitmap_words(plan.total)):
            raise TypeError("bitmap: expected contiguous 32-bit GPU tensor of srs_bitmap_words(total) words")

    def mark_multi(self, plan: Plan, prev: Optional[Sequence[torch.Tensor]], cur: Optional[Sequence[torch.Tensor]],
                   bitmap: torch.Tensor, stream: Optional[torch.cuda.Stream] = None, pairs=None) -> None:
        if pairs is None:
            pairs = self.bind_pairs(plan, prev, cur)
        self._bitmap_ok(plan, bitmap)
        _check(_lib.srs_mark_multi(self._h, plan._h, pairs, bitmap.data_ptr(), _stream_ptr(stream)), "srs_mark_multi")

    def cast_mark_multi(self, plan: Plan, weights: Optional[Sequence[torch.Tensor]],
                        master: Optional[Sequence[torch.Tensor]], bitmap: torch.Tensor,
                        stream: Optional[torch.cuda.Stream] = None, pairs=None) -> None:
        if pairs is None:
            pairs = self.bind_cast_pairs(plan, weights, master)
        self._bitmap_ok(plan, bitmap)
        _check(_lib.srs_cast_mark_multi(self._h, plan._h, pairs, bitmap.data_ptr(), _stream_ptr(stream)),
               "srs_cast_mark_multi")

    def extract_marked_multi(self, plan: Plan, weights: Optional[Sequence[torch.Tensor]], bitmap: torch.Tensor,
                             I: torch.Tensor, V: torch.Tensor, counts: torch.Tensor, cap: int,
                             stream: Optional[torch.cuda.Stream] = None, tensors=None) -> None:
        if tensors is None:
            tensors = self.bind_weights(plan, weights)
        self._bitmap_ok(plan, bitmap)
        if cap > 0:
            _payload_ok(I, V, counts, plan.nbuckets, cap)
        _check(_lib.srs_extract_marked_multi(self._h, plan._h, tensors, bitmap.data_ptr(), I.data_ptr(), V.data_ptr(),
                                             counts.data_ptr(), cap, _stream_ptr(stream)), "srs_extract_marked_multi")

    # ---- value entropy coding -------------------------------------------------------------
    def encode_values(self, V: torch.Tensor, counts: torch.Tensor, nbuckets: int, cap: int, enc: dict,
                      stream: Optional[torch.cuda.Stream] = None) -> None:
        """enc: the dict alloc_value_stream() returns."""
        if not (V.is_cuda and V.element_size() == 2 and V.is_contiguous() and V.numel() >= nbuckets * cap):
            raise TypeError("V: expected contiguous 16-bit GPU tensor of at least nb*cap elements")
        _value_stream_ok(enc, nbuckets, cap)
        _check(_lib.srs_encode_values(self._h, V.data_ptr(), counts.data_ptr(), nbuckets, cap, enc["lens"].data_ptr(),
                                      enc["low"].data_ptr(), enc["bits"].data_ptr(), enc["chunk_words"].data_ptr(),
                                      enc["sub"].data_ptr(), _stream_ptr(stream)), "srs_encode_values")

    def decode_values(self, enc: dict, counts: torch.Tensor, nbuckets: int, cap: int, V_out: torch.Tensor,
                      stream: Optional[torch.cuda.Stream] = None) -> None:
        if not (V_out.is_cuda and V_out.element_size() == 2 and V_out.is_contiguous() and V_out.numel() >= nbuckets * cap):
            raise TypeError("V_out: expected contiguous 16-bit GPU tensor of at least nb*cap elements")
        _value_stream_ok(enc, nbuckets, cap)
        _check(_lib.srs_decode_values(self._h, enc["lens"].data_ptr(), enc["low"].data_ptr(), enc["bits"].data_ptr(),
                                      enc["chunk_words"].data_ptr(), enc["sub"].data_ptr(), counts.data_ptr(), nbuckets,
                                      cap, V_out.data_ptr(), _stream_ptr(stream)), "srs_decode_values")

    # ---- 16-bit index coding --------------------------------------------------------------
    def encode_indices(self, I: torch.Tensor, counts: torch.Tensor, nbuckets: int, cap: int, base_stride: int,
                       D: torch.Tensor, max_gap: torch.Tensor, anchors: torch.Tensor,
                       stream: Optional[torch.cuda.Stream] = None) -> None:
        if cap > 0:
            _payload_ok(I, D, counts, nbuckets, cap)
            _encoded_ok(D, max_gap, anchors, nbuckets, cap)
        _check(_lib.srs_encode_indices(self._h, I.data_ptr(), counts.data_ptr(), nbuckets, cap, base_stride,
                                       D.data_ptr(), max_gap.data_ptr(), anchors.data_ptr(), _stream_ptr(stream)),
               "srs_encode_indices")

    def apply_encoded(self, weights: torch.Tensor, bucket_elems: int, D: torch.Tensor, I_wide: torch.Tensor,
                      V: torch.Tensor, counts: torch.Tensor, max_gap: torch.Tensor, anchors: torch.Tensor, cap: int,
                      stream: Optional[torch.cuda.Stream] = None) -> None:
        _dev16(weights, "weights")
        n = weights.numel()
        if bucket_elems > 0 and cap > 0:
            nb = (n + bucket_elems - 1) // bucket_elems
            _payload_ok(I_wide, V, counts, nb, cap)
            _encoded_ok(D, max_gap, anchors, nb, cap)
        _check(_lib.srs_apply_encoded(self._h, weights.data_ptr(), n, bucket_elems, D.data_ptr(), I_wide.data_ptr(),
                                      V.data_ptr(), counts.data_ptr(), max_gap.data_ptr(), anchors.data_ptr(), cap,
                                      _stream_ptr(stream)), "srs_apply_encoded")

    def apply_multi_encoded(self, plan: Plan, weights: Optional[Sequence[torch.Tensor]], D: torch.Tensor,
                            I_wide: torch.Tensor, V: torch.Tensor, counts: torch.Tensor, max_gap: torch.Tensor,
                            anchors: torch.Tensor, cap: int, stream: Optional[torch.cuda.Stream] = None,
                            tensors=None) -> None:
        if tensors is None:
            tensors = self.bind_weights(plan, weights)
        if cap > 0:
            _payload_ok(I_wide, V, counts, plan.nbuckets, cap)
            _encoded_ok(D, max_gap, anchors, plan.nbuckets, cap)
        _check(_lib.srs_apply_multi_encoded(self._h, plan._h, tensors, D.data_ptr(), I_wide.data_ptr(), V.data_ptr(),
                                            counts.data_ptr(), max_gap.data_ptr(), anchors.data_ptr(), cap,
                                            _stream_ptr(stream)), "srs_apply_multi_encoded")

    # ---- density routing and the dense route ----------------------------------------------
    def route(self, counts: torch.Tensor, nbuckets: int, bucket_elems: int, total_elems: int, cap: int,
              bytes_per_pair: int, max_dense: int, route_slot: torch.Tensor, sparse_counts: torch.Tensor,
              dense_bucket: torch.Tensor, n_dense: torch.Tensor, stream: Optional[torch.cuda.Stream] = None) -> None:
        for name, t, need in (("counts", counts, nbuckets), ("route_slot", route_slot, nbuckets),
                              ("sparse_counts", sparse_counts, nbuckets), ("dense_bucket", dense_bucket, max_dense),
                              ("n_dense", n_dense, 1)):
            if not (t.is_cuda and t.element_size() == 4 and t.is_contiguous() and t.numel() >= need):
                raise TypeError(f"{name}: expected contiguous 32-bit GPU tensor of at least {need} elements")
        _check(_lib.srs_route(self._h, counts.data_ptr(), nbuckets, bucket_elems, total_elems, cap, bytes_per_pair,
                              max_dense, route_slot.data_ptr(), sparse_counts.data_ptr(), dense_bucket.data_ptr(),
                              n_dense.data_ptr(), _stream_ptr(stream)), "srs_route")

    @staticmethod
    def _dense_ok(plan: Plan, dense_bucket: torch.Tensor, n_dense: torch.Tensor, max_dense: int, dense: torch.Tensor):
        if not (dense.is_cuda and dense.element_size() == 2 and dense.is_contiguous()
                and dense.numel() >= max_dense * plan.bucket_elems):
            raise TypeError("dense: expected contiguous 16-bit GPU tensor of max_dense*bucket_elems elements")
        if not (dense_bucket.is_cuda and dense_bucket.element_size() == 4 and dense_bucket.numel() >= max_dense):
            raise TypeError("dense_bucket: expected 32-bit GPU tensor of max_dense elements")
        if not (n_dense.is_cuda and n_dense.element_size() == 4 and n_dense.numel() >= 1):
            raise TypeError("n_dense: expected 32-bit GPU tensor")

    def pack_dense_multi(self, plan: Plan, old: Optional[Sequence[torch.Tensor]], new: Optional[Sequence[torch.Tensor]],
                         dense_bucket: torch.Tensor, n_dense: torch.Tensor, max_dense: int, dense: torch.Tensor,
                         stream: Optional[torch.cuda.Stream] = None, pairs=None) -> None:
        if pairs is None:
            pairs = self.bind_pairs(plan, old, new)
        self._dense_ok(plan, dense_bucket, n_dense, max_dense, dense)
        _check(_lib.srs_pack_dense_multi(self._h, plan._h, pairs, dense_bucket.data_ptr(), n_dense.data_ptr(), max_dense,
                                         dense.data_ptr(), _stream_ptr(stream)), "srs_pack_dense_multi")

    def unpack_dense_multi(self, plan: Plan, weights: Optional[Sequence[torch.Tensor]], dense_bucket: torch.Tensor,
                           n_dense: torch.Tensor, max_dense: int, dense: torch.Tensor,
                           stream: Optional[torch.cuda.Stream] = None, tensors=None) -> None:
        if tensors is None:
            tensors = self.bind_weights(plan, weights)
        self._dense_ok(plan, dense_bucket, n_dense, max_dense, dense)
        _check(_lib.srs_unpack_dense_multi(self._h, plan._h, tensors, dense_bucket.data_ptr(), n_dense.data_ptr(),
                                           max_dense, dense.data_ptr(), _stream_ptr(stream)), "srs_unpack_dense_multi")

    # ---- measurement aid ------------------------------------------------------------------
    def stream_probe(self, a: torch.Tensor, b: torch.Tensor, sink: torch.Tensor,
                     stream: Optional[torch.cuda.Stream] = None) -> None:
        nbytes = a.numel() * a.element_size()
        if b.numel() * b.element_size() != nbytes:
            raise ValueError("size mismatch")
        if sink.numel() * sink.element_size() < 4 * _lib.srs_stream_probe_sink_words(nbytes):
            raise ValueError("sink too small")
        _check(_lib.srs_stream_probe(self._h, a.data_ptr(), b.data_ptr(), nbytes, sink.data_ptr(), _stream_ptr(stream)),
               "srs_stream_probe")


def value_chunks(cap: int) -> int:
    return int(_lib.srs_value_chunks(cap))


def alloc_value_stream(nbuckets: int, cap: int, device) -> dict:
    """Device buffers of srs_encode_values' output, filled with 0xFF bytes so that tests see untouched entries."""
    nchunk = value_chunks(cap)
    return {"lens": torch.full((nbuckets, 256), -1, dtype=torch.int8, device=device).view(torch.uint8),
            "low": torch.full((nbuckets, cap), -1, dtype=torch.int8, device=device).view(torch.uint8),
            "bits": torch.full((nbuckets, nchunk, 768), -1, dtype=torch.int32, device=device),
            "chunk_words": torch.full((nbuckets, nchunk), -1, dtype=torch.int32, device=device),
            "sub": torch.full((nbuckets, nchunk, 32), -1, dtype=torch.int16, device=device)}


def _value_stream_ok(enc: dict, nb: int, cap: int) -> None:
    nchunk = value_chunks(cap)
    need = {"lens": (1, nb * 256), "low": (1, nb * cap), "bits": (4, nb * nchunk * 768), "chunk_words": (4, nb * nchunk),
            "sub": (2, nb * nchunk * 32)}
    for name, (esize, n) in need.items():
        t = enc[name]
        if not (t.is_cuda and t.element_size() == esize and t.is_contiguous() and t.numel() >= n):
            raise TypeError(f"{name}: expected contiguous GPU tensor of {n} elements of {esize} byte(s)")


def alloc_encoded(nbuckets: int, cap: int, device) -> tuple:
    """(D, max_gap, anchors) device buffers for srs_encode_indices, filled with 0xFFFF / 0 / -1."""
    D = torch.full((nbuckets, cap), -1, dtype=torch.int16, device=device)
    max_gap = torch.zeros(nbuckets, dtype=torch.int32, device=device)
    anchors = torch.full((max(anchor_count(nbuckets, cap), 1),), -1, dtype=torch.int32, device=device)
    return D, max_gap, anchors


def alloc_payload_u8(nbuckets: int, cap: int, device) -> tuple:
    """(I, V, counts) for the one-byte calls: V is uint8, filled with 0xFF."""
    I = torch.full((nbuckets, cap), -1, dtype=torch.int32, device=device)
    V = torch.full((nbuckets, cap), 0xFF, dtype=torch.uint8, device=device)
    counts = torch.zeros(nbuckets, dtype=torch.int32, device=device)
    return I, V, counts


def alloc_payload(nbuckets: int, cap: int, device) -> tuple:
    """(I, V, counts) device buffers of the layout srs.h describes.  I is filled with -1 and V with
    0xFFFF so that tests can see that slots beyond counts[b] are left untouched."""
    I = torch.full((nbuckets, cap), -1, dtype=torch.int32, device=device)
    V = torch.full((nbuckets, cap), -1, dtype=torch.int16, device=device)
    counts = torch.zeros(nbuckets, dtype=torch.int32, device=device)
    return I, V, counts
