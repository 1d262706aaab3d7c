"""Malformed and well-formed shard metadata with the status each must get -- shared by the CPU test of
bcp_validate_meta and the GPU test that asserts bcp_plan gives the same verdict."""
import numpy as np
import torch

from paper_2407_20143_amd import binding, synth
from paper_2407_20143_amd.synth import Layout, Part, regular

FULL = Part(0, (8, 4), (0, 0), (8, 4))


def _meta(layout):
    return binding.layout_to_meta(layout, pinned=False).copy()


def _ok_pair():
    return _meta(Layout([regular(FULL, 4, 0, 0)], [128])), _meta(Layout([regular(FULL, 4, 0, 0)], [128]))


def _mutated(fn):
    sm, tm = _ok_pair()
    fn(sm, tm)
    return sm, tm


def _set(side, field, value, idx=None):
    def fn(sm, tm):
        m = sm if side == "s" else tm
        if idx is None:
            m[field][0] = value
        else:
            m[field][0, idx] = value
    return fn


def _huge_volume(sm, tm):
    for m in (sm, tm):
        m["global_shape"][0, :2] = (1 << 30, 1 << 30)
        m["lengths"][0, :2] = (1 << 30, 1 << 30)
        m["flat_end"][0] = 1 << 60


def _huge_stride(sm, tm):
    tm["strides"][0, 0] = 1 << 58
    tm["strides"][0, 1] = 1


def cases():
    """(name, saved meta, target meta, flags, expected status name)"""
    over = Layout([regular(Part(0, (8, 4), (0, 0), (5, 4)), 4, 0, 0), regular(Part(0, (8, 4), (4, 0), (4, 4)), 4, 1, 0)], [80, 64])
    half = Layout([regular(Part(0, (8, 4), (0, 0), (4, 4)), 4, 0, 0)], [64])
    two_saved_disagree = Layout([regular(Part(0, (8, 4), (0, 0), (4, 4)), 4, 0, 0), regular(Part(0, (8, 5), (4, 0), (4, 4)), 4, 0, 64)], [128])
    ok_t = Layout([regular(FULL, 4, 0, 0)], [128])
    out = [
        ("ok", *_ok_pair(), 0, "BCP_OK"),
        ("saved overlap", _meta(over), _meta(ok_t), 0, "BCP_ERR_SAVED_OVERLAP"),
        ("saved overlap unchecked -> target covered twice", _meta(over), _meta(ok_t), binding.BCP_SKIP_OVERLAP_CHECK,
         "BCP_ERR_SAVED_OVERLAP"),
        ("shape mismatch", _ok_pair()[0], _meta(Layout([regular(Part(0, (4, 8), (0, 0), (4, 8)), 4, 0, 0)], [128])), 0,
         "BCP_ERR_SHAPE_MISMATCH"),
        ("saved records disagree on the shape", _meta(two_saved_disagree), _meta(ok_t), 0, "BCP_ERR_SHAPE_MISMATCH"),
        ("dtype mismatch", _ok_pair()[0], _meta(Layout([regular(FULL, 2, 0, 0)], [64])), 0, "BCP_ERR_DTYPE_MISMATCH"),
        ("4 -> 2 bytes with the conversion flag", _ok_pair()[0], _meta(Layout([regular(FULL, 2, 0, 0)], [64])),
         binding.BCP_CONVERT_F32_TO_BF16, "BCP_OK"),
        ("2 -> 4 bytes is no conversion", _meta(Layout([regular(FULL, 2, 0, 0)], [64])), _ok_pair()[1],
         binding.BCP_CONVERT_F32_TO_BF16, "BCP_ERR_DTYPE_MISMATCH"),
        ("8 -> 2 bytes is no conversion", _meta(Layout([regular(FULL, 8, 0, 0)], [256])), _meta(Layout([regular(FULL, 2, 0, 0)], [64])),
         binding.BCP_CONVERT_F32_TO_BF16, "BCP_ERR_DTYPE_MISMATCH"),
        ("offsets beyond the shape", *_mutated(_set("t", "offsets", 4, 0)), 0, "BCP_ERR_OUT_OF_BOUNDS"),
        ("too many dims", *_mutated(_set("t", "ndim", 9)), 0, "BCP_ERR_TOO_MANY_DIMS"),
        ("negative ndim", *_mutated(_set("s", "ndim", -1)), 0, "BCP_ERR_INVALID_ARG"),
        ("itemsize 3", *_mutated(_set("s", "itemsize", 3)), 0, "BCP_ERR_INVALID_ARG"),
        ("flat range beyond the box", *_mutated(_set("t", "flat_end", 33)), 0, "BCP_ERR_OUT_OF_BOUNDS"),
        ("flat range backwards", *_mutated(_set("t", "flat_begin", 40)), 0, "BCP_ERR_INVALID_ARG"),
        ("negative fqn", *_mutated(_set("t", "fqn_id", -2)), 0, "BCP_ERR_INVALID_ARG"),
        ("negative buffer index", *_mutated(_set("s", "buf", -1)), 0, "BCP_ERR_INVALID_ARG"),
        ("reserved field set", *_mutated(_set("s", "reserved", 1)), 0, "BCP_ERR_INVALID_ARG"),
        ("stride that leaves the address range", *_mutated(_huge_stride), 0, "BCP_ERR_INVALID_ARG"),
        ("byte offset that leaves the address range", *_mutated(_set("s", "byte_offset", 1 << 61)), 0, "BCP_ERR_INVALID_ARG"),
        ("volume that leaves the address range", *_mutated(_huge_volume), 0, "BCP_ERR_INVALID_ARG"),
        ("uncovered", _meta(half), _meta(ok_t), 0, "BCP_ERR_UNCOVERED"),
        ("uncovered allowed", _meta(half), _meta(ok_t), binding.BCP_ALLOW_UNCOVERED, "BCP_OK"),
        ("no target records", _ok_pair()[0], np.zeros(0, dtype=binding.SHARD_META), 0, "BCP_OK"),
    ]
    # well-formed model-shaped and random layouts, flat (irregular) shards on either side
    for c in (synth.cfg4(layers=1, hidden=32, ffn=48, vocab=64, dp_s=16, dp_t=12, n_states=1),
              synth.cfg5(layers=1, hidden=64, experts=8, ffn=24, n_small=300),
              synth.random_case(41, saved_mode="flat", target_mode="grid", p_strided=0.3),
              synth.random_case(42, saved_mode="grid", target_mode="flat")):
        out.append((c.name, _meta(c.saved), _meta(c.target), 0, "BCP_OK"))
    c = synth.eval_load_case(layers=1, hidden=32, ffn=48, vocab=64, zero_saved=True)
    out.append((c.name, _meta(c.saved), _meta(c.target), binding.BCP_CONVERT_F32_TO_BF16, "BCP_OK"))
    out.append((c.name + " without the flag", _meta(c.saved), _meta(c.target), 0, "BCP_ERR_DTYPE_MISMATCH"))
    # a flat saved slice dropped: the elements it held are uncovered; the same slice twice: overlap
    c = synth.cfg4(layers=1, hidden=32, ffn=48, vocab=64, dp_s=4, dp_t=3, n_states=1)
    sm = _meta(c.saved)
    drop = sm[sm["buf"] != 2]
    out.append(("flat slice missing", drop, _meta(c.target), 0, "BCP_ERR_UNCOVERED"))
    twice = np.concatenate([sm, sm[sm["buf"] == 1]])
    out.append(("flat slice saved twice", twice, _meta(c.target), 0, "BCP_ERR_SAVED_OVERLAP"))
    return out


def host_verdict(sm, tm, flags):
    try:
        binding.validate_meta(sm, tm, flags)
        return "BCP_OK", ""
    except binding.BcpError as e:
        return e.name, str(e)


def device_verdict(sm, tm, flags):
    try:
        binding.plan(sm, tm, flags=flags).destroy()
        return "BCP_OK", ""
    except binding.BcpError as e:
        return e.name, str(e)
