"""Python access to the CPU oracle (``reft_oracle.c``).  TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may import
this package.  The product package never does, and this package imports nothing of the product.

The wrapper only marshals numpy ``uint8`` arrays into the C functions; all of the method's
arithmetic is in the C file, which cites the passages of the paper it follows.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "reft_oracle.c")
_LIB = os.path.join(_HERE, "libreft_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C, -O2, OpenMP for the optional outer-range split)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared",
                               "-Wall", "-Wextra", "-o", _LIB, _SRC])
    return _LIB



class Oracle:
    """One loaded build of the oracle's C file.  The module-level functions use the default build;
    the tests also load deliberately broken builds (planted mistakes) to show that the pins fail."""

    def __init__(self, libpath: str):
        lib = ctypes.CDLL(libpath)
        u64, u32, p = ctypes.c_uint64, ctypes.c_uint32, ctypes.c_void_p
        lib.oracle_set_threads.argtypes = [ctypes.c_int]
        lib.oracle_set_threads.restype = None
        lib.oracle_get_threads.restype = ctypes.c_int
        lib.oracle_max_threads.restype = ctypes.c_int
        lib.oracle_stream_bytes.argtypes = [p, u64]
        lib.oracle_stream_bytes.restype = u64
        lib.oracle_pack.argtypes = [p, p, u64, p, u64]
        lib.oracle_pack_bucketed.argtypes = [p, p, u64, p, u64, p, u64]
        lib.oracle_unpack.argtypes = [p, u64, p, u64, p]
        lib.oracle_encode.argtypes = [p, u32, u64, p]
        lib.oracle_encode_padded.argtypes = [p, p, u32, p, u64]
        lib.oracle_reconstruct.argtypes = [p, u32, p, u64, p]
        lib.oracle_segment_bytes.argtypes = [u64, u32]
        lib.oracle_segment_bytes.restype = u64
        lib.oracle_encode_rotated.argtypes = [p, u32, u64, u32, p]
        lib.oracle_reconstruct_rotated.argtypes = [p, p, u32, u64, u32, p]
        lib.oracle_collab_recover.argtypes = [p, p, p, u32, p, u32, u64, p, p, p]
        self.lib = lib

    # -- threads for the optional outer-range split ------------------------------------------
    def set_threads(self, n: int) -> None:
        self.lib.oracle_set_threads(int(n))

    def get_threads(self) -> int:
        return int(self.lib.oracle_get_threads())

    def max_threads(self) -> int:
        return int(self.lib.oracle_max_threads())

    # -- the operations ------------------------------------------------------------------------
    def pack(self, spans: Sequence[np.ndarray]) -> np.ndarray:
        """Stream = the spans' bytes end to end."""
        sizes = [a.size for a in spans]
        out = np.empty(sum(sizes), dtype=np.uint8)
        _check(self.lib.oracle_pack(_ptr_array(spans), _u64_array(sizes), len(spans),
                                    out.ctypes.data, out.size), "pack")
        return out

    def pack_bucketed(self, spans: Sequence[np.ndarray], bucket_nbytes: Sequence[int],
                      host: Optional[np.ndarray] = None) -> np.ndarray:
        """Bucket by bucket, byte by byte, into ``host`` (allocated here if None)."""
        sizes = [a.size for a in spans]
        if host is None:
            host = np.empty(sum(sizes), dtype=np.uint8)
        _check(self.lib.oracle_pack_bucketed(_ptr_array(spans), _u64_array(sizes), len(spans),
                                             _u64_array(bucket_nbytes), len(bucket_nbytes),
                                             host.ctypes.data, host.size), "pack_bucketed")
        return host

    def unpack(self, stream: np.ndarray, span_nbytes: Sequence[int]) -> List[np.ndarray]:
        outs = [np.empty(int(n), dtype=np.uint8) for n in span_nbytes]
        _check(self.lib.oracle_unpack(stream.ctypes.data, stream.size, _u64_array(span_nbytes),
                                      len(span_nbytes), _ptr_array(outs)), "unpack")
        return outs

    def encode(self, shards: Sequence[np.ndarray]) -> np.ndarray:
        L = shards[0].size
        if any(s.size != L for s in shards):
            raise ValueError("oracle: encode needs equal-length shards (see encode_padded)")
        out = np.empty(L, dtype=np.uint8)
        _check(self.lib.oracle_encode(_ptr_array(shards), len(shards), L, out.ctypes.data),
               "encode")
        return out

    def encode_padded(self, shards: Sequence[np.ndarray]) -> np.ndarray:
        lens = [s.size for s in shards]
        out = np.empty(max(lens), dtype=np.uint8)
        _check(self.lib.oracle_encode_padded(_ptr_array(shards), _u64_array(lens), len(shards),
                                             out.ctypes.data, out.size), "encode_padded")
        return out

    def reconstruct(self, survivors: Sequence[np.ndarray], parity: np.ndarray) -> np.ndarray:
        L = parity.size
        if any(s.size != L for s in survivors):
            raise ValueError("oracle: reconstruct needs survivors of the parity's length")
        out = np.empty(L, dtype=np.uint8)
        _check(self.lib.oracle_reconstruct(_ptr_array(survivors), len(survivors),
                                           parity.ctypes.data, L, out.ctypes.data),
               "reconstruct")
        return out


    # -- rotated placement of the parity (section 4.2) ------------------------------------------
    def segment_bytes(self, L: int, k: int) -> int:
        return int(self.lib.oracle_segment_bytes(int(L), int(k)))

    def encode_rotated(self, shards: Sequence[np.ndarray], member: int) -> np.ndarray:
        L, k = shards[0].size, len(shards)
        if any(s.size != L for s in shards):
            raise ValueError("oracle: encode_rotated needs equal-length shards")
        out = np.empty(self.segment_bytes(L, k) if k >= 2 else 0, dtype=np.uint8)
        _check(self.lib.oracle_encode_rotated(_ptr_array(shards), k, L, int(member),
                                              out.ctypes.data), "encode_rotated")
        return out

    def reconstruct_rotated(self, shards: Sequence[Optional[np.ndarray]],
                            parities: Sequence[Optional[np.ndarray]], lost: int, L: int) -> np.ndarray:
        """``shards[lost]`` and ``parities[lost]`` may be None: they are never read."""
        k = len(shards)
        dummy = np.zeros(1, dtype=np.uint8)
        sh = [dummy if (a is None) else a for a in shards]
        pa = [dummy if (a is None) else a for a in parities]
        out = np.empty(L, dtype=np.uint8)
        _check(self.lib.oracle_reconstruct_rotated(_ptr_array(sh), _ptr_array(pa), k, int(L),
                                                   int(lost), out.ctypes.data),
               "reconstruct_rotated")
        return out


    # -- collaborative protection (section 4.2, last paragraph) ------------------------------------
    def collab_recover(self, shards: Sequence[Optional[np.ndarray]],
                       dups: Sequence[Sequence[Optional[np.ndarray]]], arc_offsets: Sequence[int],
                       units: Optional[Sequence[Optional[np.ndarray]]], lost: Sequence[int], L: int):
        """``shards[i]`` / ``dups[a][i]`` / ``units[i]`` of lost members may be None (never read).
        Returns (recovered, unknown, seg_known): the recovered shards by lost member, the number
        of segments that stay unknown, and the k x (k-1) table of known segments."""
        k = len(shards)
        lost_flags = np.zeros(k, dtype=np.uint8)
        lost_flags[list(lost)] = 1
        dummy = np.zeros(1, dtype=np.uint8)
        sh = [dummy if a is None else a for a in shards]
        du = [dummy if a is None else a for row in dups for a in row]
        un = None if units is None else [dummy if a is None else a for a in units]
        out = [np.full(int(L), 0xEE, dtype=np.uint8) if lost_flags[i] else dummy for i in range(k)]
        seg = np.zeros(k * (k - 1), dtype=np.uint8)
        rc = self.lib.oracle_collab_recover(
            _ptr_array(sh), _ptr_array(du), _u32_array(arc_offsets), len(arc_offsets),
            None if un is None else _ptr_array(un), k, int(L), lost_flags.ctypes.data,
            _ptr_array(out), seg.ctypes.data)
        if rc < 0:
            raise ValueError("oracle: collab_recover rejected its arguments")
        return {i: out[i] for i in range(k) if lost_flags[i]}, int(rc), seg.reshape(k, k - 1)


# ------------------------------------------------------------------------------------------------
# marshalling helpers (no arithmetic)
# ------------------------------------------------------------------------------------------------
def as_bytes(x) -> np.ndarray:
    """A flat, C-contiguous uint8 view of a numpy array or a CPU torch tensor (any dtype)."""
    if isinstance(x, np.ndarray):
        return np.ascontiguousarray(x).reshape(-1).view(np.uint8)
    import torch  # only for tensor inputs
    assert x.device.type == "cpu"
    return x.contiguous().reshape(-1).view(torch.uint8).numpy()


def _ptr_array(arrays: Sequence[np.ndarray]):
    for a in arrays:
        assert a.dtype == np.uint8 and a.flags["C_CONTIGUOUS"]
    return (ctypes.c_void_p * max(1, len(arrays)))(*[a.ctypes.data for a in arrays])


def _u32_array(vals: Sequence[int]):
    return (ctypes.c_uint32 * max(1, len(vals)))(*[int(v) for v in vals])


def _u64_array(vals: Sequence[int]):
    return (ctypes.c_uint64 * max(1, len(vals)))(*[int(v) for v in vals])


def _check(rc: int, what: str):
    if rc != 0:
        raise ValueError(f"oracle: {what} rejected its arguments (rc={rc})")


_default: Optional[Oracle] = None


def default() -> Oracle:
    global _default
    if _default is None:
        _default = Oracle(build())
    return _default


def set_threads(n):          default().set_threads(n)
def get_threads():           return default().get_threads()
def max_threads():           return default().max_threads()
def pack(spans):             return default().pack(spans)
def pack_bucketed(spans, bucket_nbytes, host=None):
    return default().pack_bucketed(spans, bucket_nbytes, host)
def unpack(stream, sizes):   return default().unpack(stream, sizes)
def encode(shards):          return default().encode(shards)
def encode_padded(shards):   return default().encode_padded(shards)
def reconstruct(surv, par):  return default().reconstruct(surv, par)
def segment_bytes(L, k):     return default().segment_bytes(L, k)
def encode_rotated(shards, member):
    return default().encode_rotated(shards, member)
def reconstruct_rotated(shards, parities, lost, L):
    return default().reconstruct_rotated(shards, parities, lost, L)
def collab_recover(shards, dups, arc_offsets, units, lost, L):
    return default().collab_recover(shards, dups, arc_offsets, units, lost, L)
