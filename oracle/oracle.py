"""ctypes front end of the CPU oracle (oracle/reshard_oracle.cpp).

TEST INFRASTRUCTURE ONLY.  Importable from tests/, the smoke check and the bench's
cpu_baseline leg -- never from the product package.  It loads nothing but its own shared
library (built with g++ from the one C++ file beside it) and shares no code with the HIP path.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "reshard_oracle.cpp")
_LIB = os.path.join(_HERE, "libreshard_oracle.so")

MAX_DIMS = 8

PART_DTYPE = np.dtype([
    ("fqn", "<i8"), ("ndim", "<i4"), ("pad_", "<i4"),
    ("global_shape", "<i8", (MAX_DIMS,)), ("offsets", "<i8", (MAX_DIMS,)), ("lengths", "<i8", (MAX_DIMS,)),
], align=True)
SHARD_DTYPE = np.dtype([
    ("part_begin", "<i8"), ("part_count", "<i8"), ("flat_begin", "<i8"), ("flat_end", "<i8"),
    ("byte_offset", "<i8"), ("strides", "<i8", (MAX_DIMS,)),
    ("itemsize", "<i4"), ("buf", "<i4"), ("has_strides", "<i4"), ("pad_", "<i4"),
], align=True)

ERRORS = {0: "ok", 1: "invalid", 2: "saved_overlap", 3: "uncovered", 4: "mismatch", 5: "bounds"}


class OracleError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"oracle: {ERRORS.get(code, code)}: {msg}")
        self.code = code
        self.kind = ERRORS.get(code, str(code))


def build(force: bool = False) -> str:
    """Compile the oracle with g++ (host only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["g++", "-O2", "-std=c++17", "-Wall", "-Wextra", "-shared", "-fPIC", "-pthread",
                               _SRC, "-o", _LIB])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.orc_reshard.restype = ctypes.c_int
        _lib.orc_reshard.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_char_p, ctypes.c_int]
        assert _lib.orc_max_dims() == MAX_DIMS
    return _lib


def _marshal(layout):
    """Layout (paper_2407_20143_amd.synth) -> (parts array, shards array).  A group's shared part
    list is emitted once."""
    n_parts = 0
    seen = {}
    for sh in layout.shards:
        key = id(sh.parts) if sh.group >= 0 else None
        if key is None or key not in seen:
            if key is not None:
                seen[key] = n_parts
            n_parts += len(sh.parts)
    parts = np.zeros(max(n_parts, 1), dtype=PART_DTYPE)
    shards = np.zeros(max(len(layout.shards), 1), dtype=SHARD_DTYPE)
    seen = {}
    cur = 0
    for i, sh in enumerate(layout.shards):
        key = id(sh.parts) if sh.group >= 0 else None
        if key is not None and key in seen:
            begin = seen[key]
        else:
            begin = cur
            if key is not None:
                seen[key] = begin
            for p in sh.parts:
                r = parts[cur]
                n = len(p.global_shape)
                r["fqn"], r["ndim"] = p.fqn, n
                r["global_shape"][:n] = p.global_shape
                r["offsets"][:n] = p.offsets
                r["lengths"][:n] = p.lengths
                cur += 1
        s = shards[i]
        s["part_begin"], s["part_count"] = begin, len(sh.parts)
        s["flat_begin"], s["flat_end"] = sh.flat_begin, sh.flat_end
        s["byte_offset"], s["itemsize"], s["buf"] = sh.byte_offset, sh.itemsize, sh.buf
        if sh.strides is not None:
            s["has_strides"] = 1
            s["strides"][:len(sh.strides)] = sh.strides
    return parts, shards


def _ptr_array(bufs: Sequence[np.ndarray]):
    arr = (ctypes.c_void_p * max(len(bufs), 1))()
    for i, b in enumerate(bufs):
        arr[i] = b.ctypes.data
    return arr


def _as_np(t) -> np.ndarray:
    if isinstance(t, torch.Tensor):
        assert t.device.type == "cpu" and t.dtype == torch.uint8 and t.is_contiguous()
        return t.numpy()
    return t


def reshard(saved, target, src_blobs, dst_init: Optional[List] = None, poison: int = 0xA5,
            allow_uncovered: bool = False, threads: Optional[int] = None, want_written: bool = False):
    """Run the oracle.  saved/target: synth.Layout.  src_blobs: CPU uint8 buffers (torch or numpy).
    Returns the destination buffers as numpy uint8 arrays (bytes no target shard covers keep
    `poison`), and with want_written also per-byte write counters."""
    lib = _load()
    sparts, sshards = _marshal(saved)
    tparts, tshards = _marshal(target)
    src = [np.ascontiguousarray(_as_np(b)) for b in src_blobs]
    if dst_init is None:
        dst = [np.full(n, poison, dtype=np.uint8) for n in target.buf_bytes]
    else:
        dst = [np.array(_as_np(b), copy=True) for b in dst_init]
    written = [np.zeros(len(d), dtype=np.uint8) for d in dst] if want_written else None
    src_sizes = np.array([len(b) for b in src] or [0], dtype=np.int64)
    dst_sizes = np.array([len(b) for b in dst] or [0], dtype=np.int64)
    sp, dp = _ptr_array(src), _ptr_array(dst)
    wp = _ptr_array(written) if want_written else None
    err = ctypes.create_string_buffer(512)
    if threads is None:
        threads = min(os.cpu_count() or 1, 16)
    rc = lib.orc_reshard(sparts.ctypes.data, sshards.ctypes.data, len(saved.shards), sp, src_sizes.ctypes.data,
                         tparts.ctypes.data, tshards.ctypes.data, len(target.shards), dp, dst_sizes.ctypes.data,
                         wp, int(allow_uncovered), int(threads), err, len(err))
    if rc != 0:
        raise OracleError(rc, err.value.decode())
    return (dst, written) if want_written else dst
