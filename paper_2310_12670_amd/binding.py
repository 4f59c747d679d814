"""ctypes binding of ``include/reft.h``: the same entry points, arguments marshalled from Python.

Pointers may be given as ``torch.Tensor`` (its ``data_ptr()`` is used), as ``int`` addresses or as
``None``; pointer arrays as sequences of those or as a ctypes array made with :func:`ptr_array`
(worth it when the same list is passed many times).  Streams may be ``torch.cuda.Stream``,
``int`` (a ``hipStream_t``) or ``None`` (the default stream).  Every failing call raises
:class:`ReftError` carrying the library's code and message.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

__all__ = [
    "ReftError", "REFT_OK", "REFT_EINVAL", "REFT_ESIZE", "REFT_EHIP", "REFT_EUNRECOVERABLE",
    "REFT_MAX_K", "lib_path", "ptr_array",
    "reft_plan_create", "reft_plan_destroy", "reft_plan_stream_bytes", "reft_plan_num_spans",
    "reft_plan_num_buckets", "reft_plan_max_bucket_bytes", "reft_plan_staging_slot_bytes",
    "reft_plan_bucket_range", "reft_plan_split", "reft_plan_span_offset", "reft_plan_tile_info",
    "reft_plan_tile_first_span",
    "reft_snapshot_pack", "reft_snapshot_pack_range", "reft_plan_bucket_of", "reft_snapshot_wait",
    "reft_snapshot_query", "reft_ckpt_create", "reft_ckpt_destroy", "reft_ckpt_begin",
    "reft_ckpt_commit", "reft_ckpt_latest", "reft_ckpt_wait", "REFT_EBUSY",
    "reft_plan_staged_work", "reft_plan_burst_stats", "reft_recovery_plan",
    "REFT_RECOVER_COPY", "REFT_RECOVER_DECODE",
    "reft_pack_device", "reft_unpack_device", "reft_parity_encode", "reft_parity_encode_noalloc",
    "reft_parity_encode_pack", "reft_reconstruct",
    "reft_reconstruct_spans", "reft_segment_bytes", "reft_parity_encode_rotated",
    "reft_reconstruct_rotated", "reft_restore", "reft_restore_wait",
    "reft_set_tunable", "reft_get_tunable", "reft_last_error", "reft_version",
]

REFT_OK, REFT_EINVAL, REFT_ESIZE, REFT_EHIP, REFT_EUNRECOVERABLE, REFT_EBUSY = 0, -1, -2, -3, -4, -5
REFT_MAX_K = 32
REFT_RECOVER_COPY, REFT_RECOVER_DECODE = 1, 2

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libreft.so")
_lib = None


class ReftError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"libreft error {code}: {message}")
        self.code = code
        self.message = message


def lib_path() -> str:
    return _LIB_PATH


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            f"{_LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'` "
            "(there is no fallback path)")
    lib = ctypes.CDLL(_LIB_PATH)
    u64, u32, vp, i = ctypes.c_uint64, ctypes.c_uint32, ctypes.c_void_p, ctypes.c_int
    pu64 = ctypes.POINTER(ctypes.c_uint64)
    sig = {
        "reft_plan_create": (i, [vp, u64, vp, u64, u64, ctypes.POINTER(vp)]),
        "reft_plan_destroy": (None, [vp]),
        "reft_plan_stream_bytes": (u64, [vp]),
        "reft_plan_num_spans": (u64, [vp]),
        "reft_plan_num_buckets": (u64, [vp]),
        "reft_plan_max_bucket_bytes": (u64, [vp]),
        "reft_plan_staging_slot_bytes": (u64, [vp]),
        "reft_plan_bucket_range": (i, [vp, u64, pu64, pu64]),
        "reft_plan_span_offset": (i, [vp, u64, pu64]),
        "reft_plan_tile_info": (i, [vp, pu64, pu64]),
        "reft_plan_tile_first_span": (i, [vp, u64, pu64]),
        "reft_plan_split": (i, [vp, ctypes.c_double, ctypes.c_double, pu64]),
        "reft_snapshot_pack": (i, [vp, vp, vp, u64, vp, u64, vp, vp]),
        "reft_snapshot_pack_range": (i, [vp, vp, vp, u64, vp, u64, u64, u64, vp, vp]),
        "reft_plan_bucket_of": (i, [vp, u64, pu64]),
        "reft_ckpt_create": (i, [vp, vp, vp, u64, ctypes.POINTER(vp)]),
        "reft_ckpt_destroy": (None, [vp]),
        "reft_ckpt_begin": (i, [vp, ctypes.POINTER(vp), pu64]),
        "reft_ckpt_commit": (i, [vp, vp]),
        "reft_ckpt_latest": (i, [vp, ctypes.POINTER(vp), pu64]),
        "reft_snapshot_wait": (i, [vp]),
        "reft_snapshot_query": (i, [vp]),
        "reft_pack_device": (i, [vp, vp, vp, u64, vp]),
        "reft_unpack_device": (i, [vp, vp, u64, vp, vp]),
        "reft_parity_encode": (i, [vp, vp, u32, vp, vp]),
        "reft_parity_encode_noalloc": (i, [vp, vp, u32, vp, vp]),
        "reft_parity_encode_pack": (i, [vp, vp, u32, u32, vp, vp, u64, vp]),
        "reft_plan_staged_work": (i, [vp, pu64, pu64]),
        "reft_plan_burst_stats": (i, [vp, pu64]),
        "reft_ckpt_wait": (i, [vp]),
        "reft_recovery_plan": (i, [u32, vp, u32, i, vp, vp, ctypes.POINTER(u32)]),
        "reft_reconstruct": (i, [vp, u32, vp, u64, vp, ctypes.POINTER(u32), vp]),
        "reft_reconstruct_spans": (i, [vp, vp, u32, u32, vp, vp, vp]),
        "reft_segment_bytes": (u64, [vp, u32]),
        "reft_parity_encode_rotated": (i, [vp, vp, u32, u32, vp, vp]),
        "reft_reconstruct_rotated": (i, [vp, vp, vp, u32, u32, vp, vp]),
        "reft_restore": (i, [vp, vp, u64, vp, u64, vp, vp, vp]),
        "reft_restore_wait": (i, [vp]),
        "reft_set_tunable": (i, [ctypes.c_char_p, u64]),
        "reft_get_tunable": (i, [ctypes.c_char_p, pu64]),
        "reft_last_error": (ctypes.c_char_p, []),
        "reft_version": (ctypes.c_char_p, []),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    return lib


# ------------------------------------------------------------------------------------------------
# marshalling
# ------------------------------------------------------------------------------------------------
def _addr(x) -> Optional[int]:
    if x is None:
        return None
    if isinstance(x, int):
        return x or None
    if hasattr(x, "data_ptr"):
        return x.data_ptr() or None
    if hasattr(x, "ctypes"):          # numpy array (host memory)
        return x.ctypes.data or None
    raise TypeError(f"cannot take the address of {type(x).__name__}")


def _nbytes(x) -> int:
    if hasattr(x, "element_size"):
        return x.numel() * x.element_size()
    return x.nbytes


def ptr_array(items: Sequence):
    """ctypes ``void*[]`` holding the addresses of ``items`` (tensors, ints or None)."""
    if isinstance(items, ctypes.Array):
        return items
    return (ctypes.c_void_p * max(1, len(items)))(*[_addr(x) for x in items])


def _u64s(vals: Optional[Sequence[int]]):
    if vals is None:
        return None, 0
    return (ctypes.c_uint64 * max(1, len(vals)))(*[int(v) for v in vals]), len(vals)


def _stream(s) -> Optional[int]:
    if s is None:
        return None
    if isinstance(s, int):
        return s or None
    return s.cuda_stream or None


def _check(rc: int) -> int:
    if rc < 0:
        raise ReftError(rc, (_load().reft_last_error() or b"").decode())
    return rc


# ------------------------------------------------------------------------------------------------
# entry points (same names and argument order as include/reft.h)
# ------------------------------------------------------------------------------------------------
def reft_plan_create(span_nbytes: Sequence[int], bucket_nbytes: Optional[Sequence[int]] = None,
                     uniform_bucket: int = 0) -> int:
    """Returns the plan handle (an opaque address).  Destroy with :func:`reft_plan_destroy`."""
    lib = _load()
    spans, T = _u64s(span_nbytes)
    buckets, NB = _u64s(bucket_nbytes)
    out = ctypes.c_void_p()
    _check(lib.reft_plan_create(spans, T, buckets, NB, int(uniform_bucket), ctypes.byref(out)))
    return out.value


def reft_plan_destroy(plan) -> None:
    _load().reft_plan_destroy(plan)


def reft_plan_stream_bytes(plan) -> int:
    return int(_load().reft_plan_stream_bytes(plan))


def reft_plan_num_spans(plan) -> int:
    return int(_load().reft_plan_num_spans(plan))


def reft_plan_num_buckets(plan) -> int:
    return int(_load().reft_plan_num_buckets(plan))


def reft_plan_max_bucket_bytes(plan) -> int:
    return int(_load().reft_plan_max_bucket_bytes(plan))


def reft_plan_staging_slot_bytes(plan) -> int:
    return int(_load().reft_plan_staging_slot_bytes(plan))


def reft_plan_bucket_range(plan, b: int):
    lo, hi = ctypes.c_uint64(), ctypes.c_uint64()
    _check(_load().reft_plan_bucket_range(plan, int(b), ctypes.byref(lo), ctypes.byref(hi)))
    return lo.value, hi.value


def reft_plan_span_offset(plan, t: int) -> int:
    v = ctypes.c_uint64()
    _check(_load().reft_plan_span_offset(plan, int(t), ctypes.byref(v)))
    return v.value


def reft_plan_tile_info(plan):
    """(tile_bytes, ntiles)"""
    a, b = ctypes.c_uint64(), ctypes.c_uint64()
    _check(_load().reft_plan_tile_info(plan, ctypes.byref(a), ctypes.byref(b)))
    return a.value, b.value


def reft_plan_tile_first_span(plan, t: int) -> int:
    v = ctypes.c_uint64()
    _check(_load().reft_plan_tile_first_span(plan, int(t), ctypes.byref(v)))
    return v.value


def reft_plan_split(plan, t_bubble: float, t_ss: float) -> int:
    cut = ctypes.c_uint64()
    _check(_load().reft_plan_split(plan, float(t_bubble), float(t_ss), ctypes.byref(cut)))
    return cut.value


def reft_snapshot_pack(plan, span_ptrs, staging, host_dst, pack_stream=None, copy_stream=None,
                       staging_bytes: Optional[int] = None, host_cap: Optional[int] = None) -> None:
    _check(_load().reft_snapshot_pack(
        plan, ptr_array(span_ptrs), _addr(staging),
        (0 if staging is None else _nbytes(staging)) if staging_bytes is None else int(staging_bytes),
        _addr(host_dst), _nbytes(host_dst) if host_cap is None else int(host_cap),
        _stream(pack_stream), _stream(copy_stream)))


def reft_snapshot_pack_range(plan, span_ptrs, staging, host_dst, bucket_begin: int, bucket_end: int,
                             pack_stream=None, copy_stream=None,
                             staging_bytes: Optional[int] = None,
                             host_cap: Optional[int] = None) -> None:
    _check(_load().reft_snapshot_pack_range(
        plan, ptr_array(span_ptrs), _addr(staging),
        (0 if staging is None else _nbytes(staging)) if staging_bytes is None else int(staging_bytes),
        _addr(host_dst), _nbytes(host_dst) if host_cap is None else int(host_cap),
        int(bucket_begin), int(bucket_end), _stream(pack_stream), _stream(copy_stream)))


def reft_plan_bucket_of(plan, offset: int) -> int:
    b = ctypes.c_uint64()
    _check(_load().reft_plan_bucket_of(plan, int(offset), ctypes.byref(b)))
    return b.value


def reft_ckpt_create(plan, host_buf0, host_buf1, cap: Optional[int] = None) -> int:
    out = ctypes.c_void_p()
    _check(_load().reft_ckpt_create(plan, _addr(host_buf0), _addr(host_buf1),
                                    min(_nbytes(host_buf0), _nbytes(host_buf1)) if cap is None
                                    else int(cap), ctypes.byref(out)))
    return out.value


def reft_ckpt_destroy(ckpt) -> None:
    _load().reft_ckpt_destroy(ckpt)


def reft_ckpt_begin(ckpt):
    """(address of the ongoing host buffer, generation)"""
    dst, gen = ctypes.c_void_p(), ctypes.c_uint64()
    _check(_load().reft_ckpt_begin(ckpt, ctypes.byref(dst), ctypes.byref(gen)))
    return dst.value, gen.value


def reft_ckpt_commit(ckpt, stream=None) -> None:
    _check(_load().reft_ckpt_commit(ckpt, _stream(stream)))


def reft_ckpt_latest(ckpt):
    """(address of the newest complete host snapshot or None, its generation or 0)"""
    src, gen = ctypes.c_void_p(), ctypes.c_uint64()
    _check(_load().reft_ckpt_latest(ckpt, ctypes.byref(src), ctypes.byref(gen)))
    return src.value, gen.value


def reft_ckpt_wait(ckpt) -> None:
    _check(_load().reft_ckpt_wait(ckpt))


def reft_plan_staged_work(plan):
    """(gather kernel launches, copies) of a staged snapshot of the whole stream"""
    a, b = ctypes.c_uint64(), ctypes.c_uint64()
    _check(_load().reft_plan_staged_work(plan, ctypes.byref(a), ctypes.byref(b)))
    return a.value, b.value


def reft_plan_burst_stats(plan):
    """(rounds met, rounds timed out, rounds not waited, group completions) of the last burst launch"""
    v = (ctypes.c_uint64 * 4)()
    _check(_load().reft_plan_burst_stats(plan, v))
    return tuple(int(x) for x in v)


def reft_recovery_plan(k: int, copy_offsets: Sequence[int], parity_units: bool, lost: Sequence[int]):
    """``lost``: the lost members' indices.  Returns (steps, recoverable) with steps a list of
    (member, how, source, which); ``recoverable`` is False where the library answers
    REFT_EUNRECOVERABLE (the steps of the members that can be recovered still come back)."""
    lib = _load()
    flags = (ctypes.c_uint8 * max(1, k))(*[1 if x in set(lost) else 0 for x in range(k)])
    offs = (ctypes.c_uint32 * max(1, len(copy_offsets)))(*[int(d) for d in copy_offsets])
    steps = (ctypes.c_uint32 * (4 * max(1, k)))()
    n = ctypes.c_uint32()
    rc = lib.reft_recovery_plan(int(k), offs, len(copy_offsets), 1 if parity_units else 0, flags,
                                steps, ctypes.byref(n))
    if rc not in (REFT_OK, REFT_EUNRECOVERABLE):
        _check(rc)
    out = [tuple(steps[4 * j:4 * j + 4]) for j in range(n.value)]
    return out, rc == REFT_OK


def reft_snapshot_wait(plan) -> None:
    _check(_load().reft_snapshot_wait(plan))


def reft_snapshot_query(plan) -> bool:
    return bool(_check(_load().reft_snapshot_query(plan)))


def reft_pack_device(plan, span_ptrs, dst_dev, stream=None, dst_cap: Optional[int] = None) -> None:
    _check(_load().reft_pack_device(plan, ptr_array(span_ptrs), _addr(dst_dev),
                                    _nbytes(dst_dev) if dst_cap is None else int(dst_cap),
                                    _stream(stream)))


def reft_unpack_device(plan, src_dev, span_ptrs, stream=None,
                       src_bytes: Optional[int] = None) -> None:
    _check(_load().reft_unpack_device(plan, _addr(src_dev),
                                      _nbytes(src_dev) if src_bytes is None else int(src_bytes),
                                      ptr_array(span_ptrs), _stream(stream)))


def reft_parity_encode(plan, shard_span_ptrs, k: int, parity_dev, stream=None) -> None:
    """``shard_span_ptrs``: k*T entries, row-major (entry s*T + t = span t of shard s)."""
    _check(_load().reft_parity_encode(plan, ptr_array(shard_span_ptrs), int(k), _addr(parity_dev),
                                      _stream(stream)))


def reft_parity_encode_pack(plan, shard_span_ptrs, k: int, own: int, parity_dev, packed_dev,
                            stream=None, packed_cap: Optional[int] = None) -> None:
    _check(_load().reft_parity_encode_pack(plan, ptr_array(shard_span_ptrs), int(k), int(own),
                                           _addr(parity_dev), _addr(packed_dev),
                                           _nbytes(packed_dev) if packed_cap is None else int(packed_cap),
                                           _stream(stream)))


def reft_parity_encode_noalloc(plan, shard_span_ptrs, k: int, parity_dev, stream=None) -> None:
    _check(_load().reft_parity_encode_noalloc(plan, ptr_array(shard_span_ptrs), int(k),
                                              _addr(parity_dev), _stream(stream)))


def reft_reconstruct(shards, parity, L: int, out_dev, stream=None) -> int:
    """``shards``: the k packed streams with ``None`` for the lost one.  Returns the lost index."""
    lost = ctypes.c_uint32(0xFFFFFFFF)
    _check(_load().reft_reconstruct(ptr_array(shards), len(shards), _addr(parity), int(L),
                                    _addr(out_dev), ctypes.byref(lost), _stream(stream)))
    return lost.value


def reft_reconstruct_spans(plan, shard_span_ptrs, k: int, lost: int, parity_dev, out_span_ptrs,
                           stream=None) -> None:
    _check(_load().reft_reconstruct_spans(plan, ptr_array(shard_span_ptrs), int(k), int(lost),
                                          _addr(parity_dev), ptr_array(out_span_ptrs),
                                          _stream(stream)))


def reft_segment_bytes(plan, k: int) -> int:
    return int(_load().reft_segment_bytes(plan, int(k)))


def reft_parity_encode_rotated(plan, shard_span_ptrs, k: int, member: int, parity_dev,
                               stream=None) -> None:
    _check(_load().reft_parity_encode_rotated(plan, ptr_array(shard_span_ptrs), int(k), int(member),
                                              _addr(parity_dev), _stream(stream)))


def reft_reconstruct_rotated(plan, shard_span_ptrs, parity_ptrs, k: int, lost: int, out_span_ptrs,
                             stream=None) -> None:
    _check(_load().reft_reconstruct_rotated(plan, ptr_array(shard_span_ptrs), ptr_array(parity_ptrs),
                                            int(k), int(lost), ptr_array(out_span_ptrs),
                                            _stream(stream)))


def reft_restore(plan, host_src, staging, span_ptrs, copy_stream=None, unpack_stream=None,
                 host_bytes: Optional[int] = None, staging_bytes: Optional[int] = None) -> None:
    _check(_load().reft_restore(
        plan, _addr(host_src), _nbytes(host_src) if host_bytes is None else int(host_bytes),
        _addr(staging),
        (0 if staging is None else _nbytes(staging)) if staging_bytes is None else int(staging_bytes),
        ptr_array(span_ptrs), _stream(copy_stream), _stream(unpack_stream)))


def reft_restore_wait(plan) -> None:
    _check(_load().reft_restore_wait(plan))


def reft_set_tunable(name: str, value: int) -> None:
    _check(_load().reft_set_tunable(name.encode(), int(value)))


def reft_get_tunable(name: str) -> int:
    v = ctypes.c_uint64()
    _check(_load().reft_get_tunable(name.encode(), ctypes.byref(v)))
    return v.value


def reft_last_error() -> str:
    return (_load().reft_last_error() or b"").decode()


def reft_version() -> str:
    return _load().reft_version().decode()
