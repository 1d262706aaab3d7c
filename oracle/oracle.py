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
        # ORACLE_LIB_OVERRIDE: the mutation test (tests/test_oracle_mutants.py) runs the pins against
        # deliberately broken builds of the oracle to show that they notice
        path = os.environ.get("ORACLE_LIB_OVERRIDE")
        if not path:
            build()
            path = _LIB
        _lib = ctypes.CDLL(path)
        _lib.orc_reshard.restype = ctypes.c_int
        _lib.orc_reshard.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_int64,
            ctypes.c_int, ctypes.c_char_p, ctypes.c_int]
        _lib.orc_f32_to_bf16.restype = None
        _lib.orc_f32_to_bf16.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64]
        assert _lib.orc_max_dims() == MAX_DIMS
    return _lib


def _pad(t):
    return tuple(t) + (0,) * (MAX_DIMS - len(t))


def _marshal(layout):
    """Layout (paper_2407_20143_amd.synth) -> (parts array, shards array).  A group's shared part
    list is emitted once.  Filled column-wise: a million shards take about a second."""
    part_list = []
    begins = []
    seen = {}
    for sh in layout.shards:
        key = id(sh.parts) if sh.group >= 0 else None
        if key is not None and key in seen:
            begins.append(seen[key])
            continue
        if key is not None:
            seen[key] = len(part_list)
        begins.append(len(part_list))
        part_list.extend(sh.parts)
    parts = np.zeros(max(len(part_list), 1), dtype=PART_DTYPE)
    k = len(part_list)
    if k:
        parts["fqn"][:k] = [p.fqn for p in part_list]
        parts["ndim"][:k] = [len(p.global_shape) for p in part_list]
        parts["global_shape"][:k] = [_pad(p.global_shape) for p in part_list]
        parts["offsets"][:k] = [_pad(p.offsets) for p in part_list]
        parts["lengths"][:k] = [_pad(p.lengths) for p in part_list]
    n = len(layout.shards)
    shards = np.zeros(max(n, 1), dtype=SHARD_DTYPE)
    if n:
        shards["part_begin"][:n] = begins
        shards["part_count"][:n] = [len(sh.parts) for sh in layout.shards]
        shards["flat_begin"][:n] = [sh.flat_begin for sh in layout.shards]
        shards["flat_end"][:n] = [sh.flat_end for sh in layout.shards]
        shards["byte_offset"][:n] = [sh.byte_offset for sh in layout.shards]
        shards["itemsize"][:n] = [sh.itemsize for sh in layout.shards]
        shards["buf"][:n] = [sh.buf for sh in layout.shards]
        for i, sh in enumerate(layout.shards):
            if sh.strides is not None:
                shards["has_strides"][i] = 1
                shards["strides"][i, :len(sh.strides)] = sh.strides
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
            allow_uncovered: bool = False, threads: Optional[int] = None, want_written: bool = False,
            only_fqns: Optional[Sequence[int]] = None, dst_inplace: Optional[List[np.ndarray]] = None,
            convert: int = 0):
    """Run the oracle.  saved/target: synth.Layout.  src_blobs: CPU uint8 buffers (torch or numpy).
    Returns the destination buffers as numpy uint8 arrays (bytes no target shard covers keep
    `poison`), and with want_written also per-byte write counters.  only_fqns: produce just these
    tensors (everything else in the destination keeps its initial bytes).  dst_inplace: write into
    these numpy buffers instead of fresh ones (large sparse checks).  convert=1: tensors saved with
    4-byte elements and asked for with 2-byte elements are narrowed binary32 -> bfloat16."""
    lib = _load()
    sparts, sshards = _marshal(saved)
    tparts, tshards = _marshal(target)
    src = [np.ascontiguousarray(_as_np(b)) for b in src_blobs]
    if dst_inplace is not None:
        dst = dst_inplace
    elif dst_init is None:
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
    only = np.array(list(only_fqns), dtype=np.int64) if only_fqns is not None else None
    rc = lib.orc_reshard(sparts.ctypes.data, sshards.ctypes.data, len(saved.shards), sp, src_sizes.ctypes.data,
                         tparts.ctypes.data, tshards.ctypes.data, len(target.shards), dp, dst_sizes.ctypes.data,
                         wp, int(allow_uncovered), int(threads),
                         only.ctypes.data if only is not None else None, len(only) if only is not None else 0,
                         int(convert), err, len(err))
    if rc != 0:
        raise OracleError(rc, err.value.decode())
    return (dst, written) if want_written else dst


def f32_to_bf16(bits: np.ndarray) -> np.ndarray:
    """The oracle's binary32 -> bfloat16 narrowing on an array of uint32 bit patterns -> uint16 patterns."""
    lib = _load()
    src = np.ascontiguousarray(bits, dtype=np.uint32)
    out = np.empty(src.shape, dtype=np.uint16)
    lib.orc_f32_to_bf16(src.ctypes.data, out.ctypes.data, src.size)
    return out
