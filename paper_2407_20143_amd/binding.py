"""Thin ctypes binding of libbcp.so (include/bcp.h).  Argument marshalling only: every step of
the reshard path runs inside the library's kernels.  PyTorch appears here only as the owner of
device memory and streams; there is no CPU fallback -- a missing library is an ImportError-like
failure at first use.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

import numpy as np

MAX_DIMS = 8
_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbcp.so")

SHARD_META = np.dtype([
    ("fqn_id", "<i8"), ("ndim", "<i4"), ("itemsize", "<i4"),
    ("global_shape", "<i8", (MAX_DIMS,)), ("offsets", "<i8", (MAX_DIMS,)), ("lengths", "<i8", (MAX_DIMS,)),
    ("flat_begin", "<i8"), ("flat_end", "<i8"), ("strides", "<i8", (MAX_DIMS,)),
    ("byte_offset", "<i8"), ("buf", "<i4"), ("reserved", "<i4"),
], align=True)

STATS = np.dtype([
    ("n_saved_boxes", "<i8"), ("n_target_boxes", "<i8"), ("n_pairs", "<i8"), ("n_regions", "<i8"),
    ("n_tiles", "<i8"), ("payload_bytes", "<i8"), ("n_transposed", "<i8"), ("max_src_buf", "<i8"),
    ("max_dst_buf", "<i8"), ("region_dims_hist", "<i8", (MAX_DIMS + 1,)),
    ("plan_device_ms", "<f8"), ("plan_wall_ms", "<f8"), ("n_batches", "<i8"), ("src_bytes", "<i8"),
], align=True)

REGION_INFO = np.dtype([
    ("src_base", "<i8"), ("dst_base", "<i8"), ("run_bytes", "<i8"),
    ("len", "<i8", (MAX_DIMS,)), ("src_pitch", "<i8", (MAX_DIMS,)), ("dst_pitch", "<i8", (MAX_DIMS,)),
    ("ndim", "<i4"), ("src_buf", "<i4"), ("dst_buf", "<i4"), ("kind", "<i4"),
    ("target_index", "<i8"), ("saved_index", "<i8"),
], align=True)

BCP_OK = 0
BCP_ALLOW_UNCOVERED = 1
BCP_SKIP_OVERLAP_CHECK = 2
BCP_ORDER_BY_SOURCE = 4
BCP_META_ON_DEVICE = 8
BCP_CONVERT_F32_TO_BF16 = 16
NOALLOC_MAX_BUFFERS = 8192

# entry points that need no GPU (csrc/bcp_host.cpp) ...
HOST_EXPORTS = [
    "bcp_meta_from_flat_slice", "bcp_decompose", "bcp_dedup_worst_fit", "bcp_validate_meta", "bcp_last_error",
    "bcp_status_name", "bcp_abi_version", "bcp_sizeof_shard_meta",
]
# ... and the rest of include/bcp.h
EXPORTS = HOST_EXPORTS + [
    "bcp_plan", "bcp_reshard", "bcp_reshard_checked", "bcp_reshard_noalloc", "bcp_reshard_arrived",
    "bcp_reshard_from_host", "bcp_plan_stats", "bcp_plan_regions", "bcp_plan_buffer_extents", "bcp_plan_destroy",
    "bcp_configure", "bcp_release_workspace",
]


class BcpError(RuntimeError):
    def __init__(self, status: int, name: str, msg: str):
        super().__init__(f"{name}: {msg}")
        self.status = status
        self.name = name


_lib = None


def _signatures():
    vp, i64, i32, u32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_uint32
    p64 = ctypes.POINTER(i64)
    return {
        "bcp_meta_from_flat_slice": [vp, i64, i64, i64, i32, i64, vp, p64],
        "bcp_decompose": [vp, vp, p64],
        "bcp_dedup_worst_fit": [vp, vp, i64, i32, vp, vp],
        "bcp_validate_meta": [vp, i64, vp, i64, u32],
        "bcp_plan": [vp, i64, vp, i64, u32, vp, ctypes.POINTER(vp)],
        "bcp_reshard": [vp, vp, i32, vp, i32, vp],
        "bcp_reshard_checked": [vp, vp, vp, i32, vp, vp, i32, vp],
        "bcp_reshard_noalloc": [vp, vp, i32, vp, i32, vp],
        "bcp_reshard_arrived": [vp, vp, i32, vp, i32, i32, i64, i64, vp],
        "bcp_reshard_from_host": [vp, vp, vp, vp, i32, vp, i32, i64, vp, vp],
        "bcp_plan_stats": [vp, vp],
        "bcp_plan_regions": [vp, vp, i64, p64],
        "bcp_plan_buffer_extents": [vp, vp, i32, vp, i32],
        "bcp_plan_destroy": [vp],
        "bcp_configure": [i64, i32, i32, i32],
        "bcp_release_workspace": [p64],
        "bcp_status_name": [ctypes.c_int],
    }


def lib():
    """Load libbcp.so (built beforehand by paper_2407_20143_amd.build / __graft_entry__.build).

    BCP_HOST_LIB_OVERRIDE names a build of the host-only part alone (csrc/bcp_host.cpp compiled with a
    plain C++ compiler, e.g. with sanitizers, for the CPU tests): then only HOST_EXPORTS exist."""
    global _lib
    if _lib is None:
        host_only = os.environ.get("BCP_HOST_LIB_OVERRIDE")
        path = host_only or LIB_PATH
        if not os.path.exists(path):
            raise RuntimeError(f"{path} is missing: build it first (python -m paper_2407_20143_amd.build); "
                               "there is no fallback path")
        L = ctypes.CDLL(path)
        sig = _signatures()
        for f in (HOST_EXPORTS if host_only else EXPORTS):
            fn = getattr(L, f)
            fn.restype = ctypes.c_int
            if f in sig:
                fn.argtypes = sig[f]
        L.bcp_last_error.restype = ctypes.c_char_p
        L.bcp_status_name.restype = ctypes.c_char_p
        L.bcp_sizeof_shard_meta.restype = ctypes.c_int64
        if L.bcp_sizeof_shard_meta() != SHARD_META.itemsize:
            raise RuntimeError("bcp_shard_meta layout mismatch between binding and library")
        _lib = L
    return _lib


def _check(status: int):
    if status != BCP_OK:
        L = lib()
        raise BcpError(status, L.bcp_status_name(status).decode(), L.bcp_last_error().decode())


# ---- metadata marshalling ---------------------------------------------------------------------
def _fill_record(r, part, itemsize, flat_begin, flat_end, buf, byte_offset, strides=None):
    n = len(part.global_shape)
    r["fqn_id"], r["ndim"], r["itemsize"] = part.fqn, n, itemsize
    r["global_shape"][:n] = part.global_shape
    r["offsets"][:n] = part.offsets
    r["lengths"][:n] = part.lengths
    r["flat_begin"], r["flat_end"] = flat_begin, flat_end
    r["buf"], r["byte_offset"] = buf, byte_offset
    if strides is not None:
        r["strides"][:n] = strides


def meta_from_flat_slice(params: np.ndarray, a: int, b: int, buf: int, byte_offset: int) -> np.ndarray:
    """bcp_meta_from_flat_slice: records for slice [a, b) of the concatenation of `params`."""
    L = lib()
    n = ctypes.c_int64(0)
    st = L.bcp_meta_from_flat_slice(params.ctypes.data, len(params), a, b, buf, byte_offset, None, ctypes.byref(n))
    if st != BCP_OK and n.value == 0:
        _check(st)
    out = np.zeros(max(n.value, 1), dtype=SHARD_META)
    cap = ctypes.c_int64(len(out))
    _check(L.bcp_meta_from_flat_slice(params.ctypes.data, len(params), a, b, buf, byte_offset, out.ctypes.data,
                                      ctypes.byref(cap)))
    return out[:cap.value]


def decompose(rec: np.ndarray) -> np.ndarray:
    """bcp_decompose of one record (a length-1 SHARD_META array or a scalar of it)."""
    L = lib()
    rec = np.ascontiguousarray(np.atleast_1d(rec))
    out = np.zeros(2 * MAX_DIMS, dtype=SHARD_META)
    n = ctypes.c_int64(len(out))
    _check(L.bcp_decompose(rec.ctypes.data, out.ctypes.data, ctypes.byref(n)))
    return out[:n.value]


def _pad(t, fill=0):
    return tuple(t) + (fill,) * (MAX_DIMS - len(t))


def _records_bulk(shards) -> np.ndarray:
    """Field-by-field copy of single-part shards into a bcp_shard_meta array (column-wise, so a
    million records take about a second)."""
    arr = np.zeros(len(shards), dtype=SHARD_META)
    if not len(shards):
        return arr
    parts = [sh.parts[0] for sh in shards]
    arr["fqn_id"] = [p.fqn for p in parts]
    arr["ndim"] = [len(p.global_shape) for p in parts]
    arr["itemsize"] = [sh.itemsize for sh in shards]
    arr["global_shape"] = [_pad(p.global_shape) for p in parts]
    arr["offsets"] = [_pad(p.offsets) for p in parts]
    arr["lengths"] = [_pad(p.lengths) for p in parts]
    arr["flat_begin"] = [sh.flat_begin for sh in shards]
    arr["flat_end"] = [sh.flat_end for sh in shards]
    arr["buf"] = [sh.buf for sh in shards]
    arr["byte_offset"] = [sh.byte_offset for sh in shards]
    strided = [i for i, sh in enumerate(shards) if sh.strides is not None]
    for i in strided:
        arr["strides"][i, :len(shards[i].strides)] = shards[i].strides
    return arr


def dedup_worst_fit(meta: np.ndarray, rank_of, n_ranks: int):
    """bcp_dedup_worst_fit -> (keep mask, bytes assigned per rank)."""
    meta = np.ascontiguousarray(meta, dtype=SHARD_META)
    ranks = np.ascontiguousarray(rank_of, dtype=np.int32)
    assert len(ranks) == len(meta)
    keep = np.zeros(max(len(meta), 1), dtype=np.uint8)
    load = np.zeros(n_ranks, dtype=np.int64)
    _check(lib().bcp_dedup_worst_fit(meta.ctypes.data if len(meta) else None, ranks.ctypes.data if len(meta) else None,
                                     len(meta), n_ranks, keep.ctypes.data, load.ctypes.data))
    return keep[:len(meta)].astype(bool), load


def validate_meta(saved_meta: np.ndarray, target_meta: np.ndarray, flags: int = 0) -> None:
    """bcp_validate_meta: the metadata checks of bcp_plan on the host, without a GPU (raises BcpError)."""
    saved_meta = np.ascontiguousarray(saved_meta, dtype=SHARD_META)
    target_meta = np.ascontiguousarray(target_meta, dtype=SHARD_META)
    _check(lib().bcp_validate_meta(saved_meta.ctypes.data if len(saved_meta) else None, len(saved_meta),
                                   target_meta.ctypes.data if len(target_meta) else None, len(target_meta), flags))


def pinned_meta(meta: np.ndarray) -> np.ndarray:
    """A copy of a bcp_shard_meta array in pinned host memory (bcp_plan uploads 304 bytes per record;
    from pinned memory that runs at the full host-to-device rate).  Without a GPU: the array itself."""
    import torch
    if not torch.cuda.is_available() or len(meta) == 0:
        return meta
    raw = np.ascontiguousarray(meta, dtype=SHARD_META).view(np.uint8).reshape(-1)
    t = torch.empty(raw.size, dtype=torch.uint8, pin_memory=True)
    out = t.numpy()  # keeps the tensor alive
    out[:] = raw
    return out.view(SHARD_META)


def layout_to_meta(layout, pinned: bool = True) -> np.ndarray:
    """synth.Layout -> array of bcp_shard_meta (in pinned host memory when there is a GPU).
    Multi-part (flat ZeRO) shards go through bcp_meta_from_flat_slice; everything else is a
    field-by-field copy."""
    meta = _layout_to_meta(layout)
    return pinned_meta(meta) if pinned else meta


def _layout_to_meta(layout) -> np.ndarray:
    chunks: List[np.ndarray] = [_records_bulk([sh for sh in layout.shards if len(sh.parts) == 1])]
    cache = {}
    for sh in layout.shards:
        if len(sh.parts) == 1:
            continue
        key = id(sh.parts)
        if key not in cache:
            params = np.zeros(len(sh.parts), dtype=SHARD_META)
            for r, p in zip(params, sh.parts):
                _fill_record(r, p, sh.itemsize, 0, p.volume, 0, 0)
            cache[key] = params
        chunks.append(meta_from_flat_slice(cache[key], sh.flat_begin, sh.flat_end, sh.buf, sh.byte_offset))
    return np.concatenate(chunks) if chunks else np.zeros(0, dtype=SHARD_META)


# ---- plan / reshard ----------------------------------------------------------------------------
class Plan:
    def __init__(self, handle):
        self._h = handle

    def buffer_extents(self):
        """(src, dst): per buffer, one past the highest byte the plan touches."""
        st = self.stats()
        ns, nd = st["max_src_buf"] + 1, st["max_dst_buf"] + 1
        s = np.zeros(max(ns, 1), dtype=np.int64)
        d = np.zeros(max(nd, 1), dtype=np.int64)
        _check(lib().bcp_plan_buffer_extents(self._h, s.ctypes.data, ns, d.ctypes.data, nd))
        return s[:ns], d[:nd]

    def stats(self) -> dict:
        out = np.zeros(1, dtype=STATS)
        _check(lib().bcp_plan_stats(self._h, out.ctypes.data))
        return {k: (out[0][k].tolist()) for k in STATS.names}

    def regions(self) -> np.ndarray:
        n = ctypes.c_int64(0)
        _check(lib().bcp_plan_regions(self._h, None, 0, ctypes.byref(n)))
        out = np.zeros(max(n.value, 1), dtype=REGION_INFO)
        _check(lib().bcp_plan_regions(self._h, out.ctypes.data, len(out), ctypes.byref(n)))
        return out[:n.value]

    def destroy(self):
        if self._h:
            lib().bcp_plan_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def _stream_ptr(stream) -> int:
    if stream is None:
        import torch
        return int(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return stream
    return int(stream.cuda_stream)


def meta_to_device(meta: np.ndarray):
    """Upload a bcp_shard_meta array once (for plans built with BCP_META_ON_DEVICE)."""
    import torch
    raw = np.ascontiguousarray(meta, dtype=SHARD_META).view(np.uint8)
    return torch.from_numpy(raw.copy()).cuda(), len(meta)


def plan_from_device_meta(saved_dev, n_saved: int, target_dev, n_target: int, flags: int = 0, stream=None) -> Plan:
    """bcp_plan with BCP_META_ON_DEVICE: the records are byte tensors in device memory."""
    h = ctypes.c_void_p()
    _check(lib().bcp_plan(saved_dev.data_ptr() if n_saved else None, n_saved,
                          target_dev.data_ptr() if n_target else None, n_target,
                          flags | BCP_META_ON_DEVICE, _stream_ptr(stream), ctypes.byref(h)))
    return Plan(h)


def plan(saved_meta: np.ndarray, target_meta: np.ndarray, flags: int = 0, stream=None) -> Plan:
    """bcp_plan(saved_meta, target_meta) -> plan"""
    saved_meta = np.ascontiguousarray(saved_meta, dtype=SHARD_META)
    target_meta = np.ascontiguousarray(target_meta, dtype=SHARD_META)
    h = ctypes.c_void_p()
    _check(lib().bcp_plan(saved_meta.ctypes.data if len(saved_meta) else None, len(saved_meta),
                          target_meta.ctypes.data if len(target_meta) else None, len(target_meta),
                          flags, _stream_ptr(stream), ctypes.byref(h)))
    return Plan(h)


def _ptrs(bufs: Sequence) -> "ctypes.Array":
    arr = (ctypes.c_void_p * max(len(bufs), 1))()
    for i, b in enumerate(bufs):
        arr[i] = b if isinstance(b, int) else b.data_ptr()
    return arr


def _sizes(bufs: Sequence):
    return (ctypes.c_int64 * max(len(bufs), 1))(*[b.numel() * b.element_size() for b in bufs])


def reshard(p: Plan, src_blobs: Sequence, dst_buffers: Sequence, stream=None, check_sizes: bool = True) -> None:
    """bcp_reshard(plan, src_blobs, dst_buffers, stream): asynchronous on `stream` (default: torch's current).
    check_sizes (the buffers are tensors): go through bcp_reshard_checked, which refuses buffers smaller
    than what the plan touches -- an undersized buffer would otherwise be a GPU memory fault."""
    if check_sizes and not any(isinstance(b, int) for b in list(src_blobs) + list(dst_buffers)):
        _check(lib().bcp_reshard_checked(p._h, _ptrs(src_blobs), _sizes(src_blobs), len(src_blobs),
                                         _ptrs(dst_buffers), _sizes(dst_buffers), len(dst_buffers), _stream_ptr(stream)))
        return
    _check(lib().bcp_reshard(p._h, _ptrs(src_blobs), len(src_blobs), _ptrs(dst_buffers), len(dst_buffers),
                             _stream_ptr(stream)))


def reshard_noalloc(p: Plan, src_blobs: Sequence, dst_buffers: Sequence, stream=None) -> None:
    """bcp_reshard_noalloc: bcp_reshard with the queue words and the pointer table in the library's
    static device array (no allocation of any kind; at most BCP_NOALLOC_MAX_BUFFERS buffers)."""
    _check(lib().bcp_reshard_noalloc(p._h, _ptrs(src_blobs), len(src_blobs), _ptrs(dst_buffers), len(dst_buffers),
                                     _stream_ptr(stream)))


def reshard_arrived(p: Plan, src_blobs: Sequence, dst_buffers: Sequence, src_buf: int, byte_begin: int,
                    byte_end: int, stream=None) -> None:
    """bcp_reshard_arrived: the work whose last source byte lies in [byte_begin, byte_end) of blob src_buf."""
    _check(lib().bcp_reshard_arrived(p._h, _ptrs(src_blobs), len(src_blobs), _ptrs(dst_buffers), len(dst_buffers),
                                     src_buf, byte_begin, byte_end, _stream_ptr(stream)))


def reshard_from_host(p: Plan, host_blobs: Sequence, src_blobs: Sequence, dst_buffers: Sequence, chunk_bytes: int,
                      copy_stream, stream=None) -> None:
    """bcp_reshard_from_host: chunked host-to-device arrival overlapped with the reshard."""
    sizes = _sizes(host_blobs)
    if len(host_blobs) < len(src_blobs):
        raise ValueError("fewer host blobs than device blobs")
    for h, d in zip(host_blobs, src_blobs):
        if d.numel() * d.element_size() < h.numel() * h.element_size():
            raise ValueError("device blob smaller than its host blob")
    _check(lib().bcp_reshard_from_host(p._h, _ptrs(host_blobs), sizes, _ptrs(src_blobs), len(src_blobs),
                                       _ptrs(dst_buffers), len(dst_buffers), chunk_bytes,
                                       _stream_ptr(copy_stream), _stream_ptr(stream)))


def configure(tile_bytes: int = 0, persistent: int = -1, wg_per_cu: int = 0, threads: int = 0) -> None:
    _check(lib().bcp_configure(tile_bytes, persistent, wg_per_cu, threads))


def release_workspace() -> int:
    """bcp_release_workspace: free the planner's grow-only device workspace; returns the bytes released."""
    n = ctypes.c_int64(0)
    _check(lib().bcp_release_workspace(ctypes.byref(n)))
    return n.value


DEFAULT_CONFIG = dict(tile_bytes=65536, persistent=1, wg_per_cu=1, threads=1024)
