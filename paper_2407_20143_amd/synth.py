"""Seeded synthetic checkpoints: tensor lists, shard layouts and values.

This module only *describes* workloads.  A stored shard is written down the way the
paper's checkpoint representation does (Sec. 3.2, "Decoupled Checkpoint Representation"):
a tensor is named by an integer FQN id and a global shape, and a shard is the box
(nD offsets, nD lengths) it holds.  A ZeRO-style irregular shard (Sec. 3.2, "Decomposing
irregular tensors"; Appendix A on hybrid 3-D parallelism) is written as a slice
[flat_begin, flat_end) of the concatenation of several row-major-flattened boxes.

Nothing here intersects boxes, decomposes flat ranges or moves bytes by index arithmetic:
blob contents are produced with library slicing / concatenation of the seeded global
tensors, so the same routine, applied to the *target* layout, yields the expected result
of a reshard independently of both the HIP path and the CPU oracle.
"""
from __future__ import annotations

import math
from collections import defaultdict
from dataclasses import dataclass, field
from typing import Dict, List, NamedTuple, Optional, Sequence, Tuple

import numpy as np
import torch

BASE_SEED = 20143
BLOB_ALIGN = 256  # tensors are packed back-to-back at 256-byte aligned offsets


# ----------------------------------------------------------------------------------------
# descriptions
# ----------------------------------------------------------------------------------------
@dataclass(frozen=True)
class TensorSpec:
    fqn: int
    name: str
    shape: Tuple[int, ...]
    dtype: torch.dtype
    dist: Tuple  # ("uniform", lo, hi) | ("normal", mean, std) | ("normal_sq", std) | ("bits",)


class Part(NamedTuple):
    """One box of one tensor: offsets/lengths along the axes of the global shape."""
    fqn: int
    global_shape: Tuple[int, ...]
    offsets: Tuple[int, ...]
    lengths: Tuple[int, ...]

    @property
    def volume(self) -> int:
        return math.prod(self.lengths)


@dataclass(slots=True)
class Shard:
    """Stored shard = elements [flat_begin, flat_end) of concat(flatten(part) for part in parts).

    Packed at `byte_offset` of buffer `buf` unless `strides` (element strides, one per
    dimension of the single part) is given.
    """
    parts: Tuple[Part, ...]
    flat_begin: int
    flat_end: int
    itemsize: int
    buf: int
    byte_offset: int
    strides: Optional[Tuple[int, ...]] = None
    group: int = -1  # >= 0: shards with the same group share one `parts` tuple (a flat buffer)

    @property
    def numel(self) -> int:
        return self.flat_end - self.flat_begin


@dataclass
class Layout:
    shards: List[Shard] = field(default_factory=list)
    buf_bytes: List[int] = field(default_factory=list)

    def payload_bytes(self) -> int:
        return sum(s.numel * s.itemsize for s in self.shards)


@dataclass
class Case:
    name: str
    seed: int
    tensors: Dict[int, TensorSpec]
    saved: Layout
    target: Layout
    convert: int = 0  # 1: the target asks for fp32 tensors as bf16 (2-byte elements), see narrowed()


def regular(part: Part, itemsize: int, buf: int, byte_offset: int, strides=None) -> Shard:
    return Shard((part,), 0, part.volume, itemsize, buf, byte_offset, strides)


def _align_up(x: int, a: int) -> int:
    return (x + a - 1) // a * a


class _Packer:
    """Running byte cursor per buffer."""

    def __init__(self, n_bufs: int, align: int = BLOB_ALIGN):
        self.cur = [0] * n_bufs
        self.align = align

    def take(self, buf: int, nbytes: int) -> int:
        off = _align_up(self.cur[buf], self.align)
        self.cur[buf] = off + nbytes
        return off

    def sizes(self) -> List[int]:
        return [max(c, 1) for c in self.cur]


# ----------------------------------------------------------------------------------------
# values
# ----------------------------------------------------------------------------------------
def global_tensor(spec: TensorSpec, seed: int, device="cpu") -> torch.Tensor:
    """Seeded contents of one whole (unsharded) tensor."""
    gen = torch.Generator(device=device)
    gen.manual_seed((seed * 1000003 + spec.fqn * 7919 + 12345) & 0x7FFFFFFFFFFFFFFF)
    shape = tuple(spec.shape)
    kind = spec.dist[0]
    if kind == "uniform":
        lo, hi = spec.dist[1], spec.dist[2]
        t = torch.rand(shape, generator=gen, device=device, dtype=torch.float32) * (hi - lo) + lo
    elif kind == "normal":
        t = torch.randn(shape, generator=gen, device=device, dtype=torch.float32) * spec.dist[2] + spec.dist[1]
    elif kind == "normal_sq":
        t = (torch.randn(shape, generator=gen, device=device, dtype=torch.float32) * spec.dist[1]) ** 2
    elif kind == "bits":  # arbitrary bit patterns (NaN payloads, -0.0, denormals all occur)
        n = max(1, math.prod(shape)) * spec.dtype.itemsize
        raw = torch.randint(0, 256, (n,), generator=gen, device=device, dtype=torch.uint8)
        return raw.view(spec.dtype).reshape(shape)
    elif kind == "bits_no_nan":  # float32 only: arbitrary bit patterns with every NaN turned into an infinity
        assert spec.dtype == torch.float32
        n = max(1, math.prod(shape))
        raw = torch.randint(0, 256, (4 * n,), generator=gen, device=device, dtype=torch.uint8).view(torch.int32)
        nan = (raw & 0x7FFFFFFF) > 0x7F800000
        raw = torch.where(nan, raw & -8388608, raw)   # keep sign and exponent: +-infinity
        return raw.view(torch.float32).reshape(shape)
    elif kind == "fill":  # every byte == dist[1] (coverage masks)
        n = max(1, math.prod(shape)) * spec.dtype.itemsize
        return torch.full((n,), spec.dist[1], device=device, dtype=torch.uint8).view(spec.dtype).reshape(shape)
    elif kind == "iota":  # element value == its global row-major index
        t = torch.arange(max(1, math.prod(shape)), device=device, dtype=torch.float64).reshape(shape)
    else:
        raise ValueError(kind)
    return t.to(spec.dtype)


def _box(G: torch.Tensor, p: Part) -> torch.Tensor:
    return G[tuple(slice(o, o + l) for o, l in zip(p.offsets, p.lengths))]


def _store(buf: torch.Tensor, sh: Shard, vals: torch.Tensor, dtype: torch.dtype) -> None:
    if vals.dtype == torch.float32 and sh.itemsize == 2:
        # a dtype-converting load: the shard holds the fp32 tensor as bf16 (the library's own cast)
        vals, dtype = vals.to(torch.bfloat16), torch.bfloat16
    assert vals.element_size() == sh.itemsize, (vals.dtype, sh.itemsize)
    if sh.strides is None:
        n = vals.numel() * sh.itemsize
        if n:
            buf[sh.byte_offset:sh.byte_offset + n] = vals.contiguous().view(-1).view(torch.uint8)
        return
    lens = sh.parts[0].lengths
    if math.prod(lens) == 0:
        return
    span = 1 + sum((l - 1) * s for l, s in zip(lens, sh.strides))
    typed = buf[sh.byte_offset:sh.byte_offset + span * sh.itemsize].view(dtype)
    torch.as_strided(typed, lens, sh.strides).copy_(vals.reshape(lens))


def coverage_mask(layout: Layout, tensors: Dict[int, TensorSpec], device="cpu") -> List[torch.Tensor]:
    """Per buffer: 1 where some shard of `layout` stores a byte, else 0 (library slicing only)."""
    ones = {f: TensorSpec(f, s.name, s.shape, s.dtype, ("fill", 1)) for f, s in tensors.items()}
    return materialize(layout, ones, 0, device, poison=0)


def materialize(layout: Layout, tensors: Dict[int, TensorSpec], seed: int, device="cpu",
                poison: Optional[int] = None, only_bufs=None) -> List[Optional[torch.Tensor]]:
    """Byte buffers of `layout` holding the seeded values (library slicing only).

    Applied to a saved layout this gives the source blobs; applied to a target layout it
    gives what a correct reshard must leave in the destination buffers (bytes no shard
    covers keep `poison`, or are unspecified when poison is None).  only_bufs: build just these
    buffers (the others come back as None) -- full-size checks go through the layout piecewise.
    """
    bufs = []
    for i, n in enumerate(layout.buf_bytes):
        if only_bufs is not None and i not in only_bufs:
            bufs.append(None)
            continue
        if poison is None:
            bufs.append(torch.zeros(n, dtype=torch.uint8, device=device))
        else:
            bufs.append(torch.full((n,), poison, dtype=torch.uint8, device=device))
    by_fqn = defaultdict(list)
    groups = defaultdict(list)
    for sh in layout.shards:
        if only_bufs is not None and sh.buf not in only_bufs:
            continue
        if sh.group >= 0:
            groups[sh.group].append(sh)
        else:
            assert len(sh.parts) == 1
            by_fqn[sh.parts[0].fqn].append(sh)
    for fqn, shs in by_fqn.items():
        spec = tensors[fqn]
        G = global_tensor(spec, seed, device)
        for sh in shs:
            box = _box(G, sh.parts[0])
            if sh.strides is not None:
                _store(bufs[sh.buf], sh, box, spec.dtype)
            else:
                _store(bufs[sh.buf], sh, box.reshape(-1)[sh.flat_begin:sh.flat_end], spec.dtype)
    for _, shs in groups.items():
        parts = shs[0].parts
        flat = torch.cat([_box(global_tensor(tensors[p.fqn], seed, device), p).reshape(-1) for p in parts])
        for sh in shs:
            assert sh.parts is parts or sh.parts == parts
            _store(bufs[sh.buf], sh, flat[sh.flat_begin:sh.flat_end], tensors[parts[0].fqn].dtype)
        del flat
    return bufs


# ----------------------------------------------------------------------------------------
# model tensor lists
# ----------------------------------------------------------------------------------------
@dataclass(frozen=True)
class _ModelTensor:
    name: str
    shape: Tuple[int, ...]
    tp_dim: Optional[int]  # None: replicated under tensor parallelism
    layer: int             # -1: first pipeline stage, -2: last pipeline stage, else layer index


def llama_tensors(layers: int, hidden: int, ffn: int, vocab: int) -> List[_ModelTensor]:
    """Decoder in model-definition order: embedding, per layer [ln1,q,k,v,o,ln2,gate,up,down],
    final norm, lm_head (untied).  Column-parallel GEMMs split dim 0 of [out,in], row-parallel
    ones dim 1, norms are replicated (Appendix A)."""
    ts = [_ModelTensor("embed.weight", (vocab, hidden), 0, -1)]
    for i in range(layers):
        p = f"layers.{i}."
        ts += [
            _ModelTensor(p + "ln1.weight", (hidden,), None, i),
            _ModelTensor(p + "attn.q.weight", (hidden, hidden), 0, i),
            _ModelTensor(p + "attn.k.weight", (hidden, hidden), 0, i),
            _ModelTensor(p + "attn.v.weight", (hidden, hidden), 0, i),
            _ModelTensor(p + "attn.o.weight", (hidden, hidden), 1, i),
            _ModelTensor(p + "ln2.weight", (hidden,), None, i),
            _ModelTensor(p + "mlp.gate.weight", (ffn, hidden), 0, i),
            _ModelTensor(p + "mlp.up.weight", (ffn, hidden), 0, i),
            _ModelTensor(p + "mlp.down.weight", (hidden, ffn), 1, i),
        ]
    ts += [_ModelTensor("final_norm.weight", (hidden,), None, -2),
           _ModelTensor("lm_head.weight", (vocab, hidden), 0, -2)]
    return ts


# state sets: (suffix, dtype, distribution)
STATE_BF16_WEIGHT = ("", torch.bfloat16, ("normal", 0.0, 0.02))
STATE_FP32_MASTER = (".master", torch.float32, ("normal", 0.0, 0.02))
STATE_FP32_EXP_AVG = (".exp_avg", torch.float32, ("normal", 0.0, 1e-3))
STATE_FP32_EXP_AVG_SQ = (".exp_avg_sq", torch.float32, ("normal_sq", 1e-3))


def _specs(model: Sequence[_ModelTensor], states) -> Dict[int, TensorSpec]:
    out = {}
    for si, (suffix, dtype, dist) in enumerate(states):
        for ti, mt in enumerate(model):
            fqn = si * len(model) + ti
            out[fqn] = TensorSpec(fqn, mt.name + suffix, mt.shape, dtype, dist)
    return out


def _stage_of(mt: _ModelTensor, layers: int, pp: int) -> int:
    if mt.layer == -1:
        return 0
    if mt.layer == -2:
        return pp - 1
    return mt.layer * pp // layers


def _tp_box(shape, tp_dim, tp, r):
    off = [0] * len(shape)
    ln = list(shape)
    if tp_dim is not None:
        assert shape[tp_dim] % tp == 0, (shape, tp_dim, tp)
        ln[tp_dim] = shape[tp_dim] // tp
        off[tp_dim] = r * ln[tp_dim]
    return tuple(off), tuple(ln)


def megatron_layout(model: Sequence[_ModelTensor], states, layers: int, tp: int, pp: int,
                    replicate_norms: bool, only_ranks=None) -> Layout:
    """One buffer per (pp_rank, tp_rank).  Replicated tensors are stored once (lowest TP rank)
    when `replicate_norms` is False -- the saved side, where every element has exactly one
    saver -- and on every TP rank otherwise (the target side).  `only_ranks`: keep just these
    (pp_rank, tp_rank) pairs (one target rank's share); buffers are renumbered densely."""
    ranks = [(p, t) for p in range(pp) for t in range(tp)]
    if only_ranks is not None:
        ranks = [r for r in ranks if r in set(only_ranks)]
    buf_of = {r: i for i, r in enumerate(ranks)}
    pk = _Packer(len(ranks))
    lay = Layout()
    for si, (_, dtype, _) in enumerate(states):
        e = dtype.itemsize
        for ti, mt in enumerate(model):
            fqn = si * len(model) + ti
            stage = _stage_of(mt, layers, pp)
            for r in range(tp):
                if (stage, r) not in buf_of:
                    continue
                if mt.tp_dim is None and not replicate_norms and r != 0:
                    continue
                off, ln = _tp_box(mt.shape, mt.tp_dim, tp, r)
                part = Part(fqn, tuple(mt.shape), off, ln)
                b = buf_of[(stage, r)]
                lay.shards.append(regular(part, e, b, pk.take(b, part.volume * e)))
    lay.buf_bytes = pk.sizes()
    return lay


def replicated_live_layout(model: Sequence[_ModelTensor], states, layers: int, tp: int, pp: int, dp: int):
    """Training-time ("live") layout with data parallelism: every DP rank of a (pp, tp) group holds
    the same shards, replicated tensors are on every TP rank as well.  One buffer per rank
    (rank = (pp_rank * tp + tp_rank) * dp + dp_rank).  Returns (layout, holder rank per shard)."""
    n_ranks = pp * tp * dp
    pk = _Packer(n_ranks)
    lay = Layout()
    rank_of: List[int] = []
    for si, (_, dtype, _) in enumerate(states):
        e = dtype.itemsize
        for ti, mt in enumerate(model):
            stage = _stage_of(mt, layers, pp)
            for r in range(tp):
                off, ln = _tp_box(mt.shape, mt.tp_dim, tp, r)
                part = Part(si * len(model) + ti, tuple(mt.shape), off, ln)
                for d in range(dp):
                    rank = (stage * tp + r) * dp + d
                    lay.shards.append(regular(part, e, rank, pk.take(rank, part.volume * e)))
                    rank_of.append(rank)
    lay.buf_bytes = pk.sizes()
    return lay, rank_of


def packed_layout(shards: Sequence[Shard], buf_of: Sequence[int], n_bufs: int, align: int = BLOB_ALIGN) -> Layout:
    """The given shards, each stored packed in buffer buf_of[i], back to back (a save-blob layout)."""
    pk = _Packer(n_bufs, align)
    lay = Layout()
    for sh, b in zip(shards, buf_of):
        lay.shards.append(Shard(sh.parts, sh.flat_begin, sh.flat_end, sh.itemsize, b,
                                pk.take(b, sh.numel * sh.itemsize), None, sh.group))
    lay.buf_bytes = pk.sizes()
    return lay


def zero_layout(model: Sequence[_ModelTensor], states, tp: int, dp: int, replicate_norms: bool,
                only=None) -> Layout:
    """ZeRO-style flat sharding: per state and TP rank the TP-local shards are flattened and
    concatenated in parameter order, then cut evenly into `dp` slices of ceil(N/dp) elements
    (the last ones short or empty).  One buffer per (state, tp_rank, dp_rank).  `only`:
    optional predicate (state, tp_rank, dp_rank) -> keep."""
    lay = Layout()
    gid = 0
    for si, (_, dtype, _) in enumerate(states):
        e = dtype.itemsize
        for r in range(tp):
            parts = []
            for ti, mt in enumerate(model):
                if mt.tp_dim is None and not replicate_norms and r != 0:
                    continue
                off, ln = _tp_box(mt.shape, mt.tp_dim, tp, r)
                parts.append(Part(si * len(model) + ti, tuple(mt.shape), off, ln))
            parts = tuple(parts)
            n = sum(p.volume for p in parts)
            chunk = -(-n // dp)
            for d in range(dp):
                if only is not None and not only(si, r, d):
                    continue
                a, b = min(n, d * chunk), min(n, (d + 1) * chunk)
                lay.shards.append(Shard(parts, a, b, e, len(lay.buf_bytes), 0, None, gid))
                lay.buf_bytes.append(max(1, (b - a) * e))
            gid += 1
    return lay


def flat_units_layout(model: Sequence[_ModelTensor], states, units: Sequence[Sequence[int]], dp: int,
                      tp: int = 1, tp_rank: int = 0) -> Layout:
    """FSDP / Megatron-distributed-optimizer style flat sharding: per state and per unit (a list of
    tensor indices, e.g. one transformer block) the TP-local shards are flattened and concatenated
    and cut evenly into `dp` slices.  One buffer per DP rank holding its slice of every unit and
    state, back to back at 256-byte aligned offsets."""
    pk = _Packer(dp)
    lay = Layout()
    gid = 0
    for si, (_, dtype, _) in enumerate(states):
        e = dtype.itemsize
        for unit in units:
            parts = []
            for ti in unit:
                mt = model[ti]
                off, ln = _tp_box(mt.shape, mt.tp_dim, tp, tp_rank)
                parts.append(Part(si * len(model) + ti, tuple(mt.shape), off, ln))
            parts = tuple(parts)
            n = sum(p.volume for p in parts)
            chunk = -(-n // dp)
            for d in range(dp):
                a, b = min(n, d * chunk), min(n, (d + 1) * chunk)
                lay.shards.append(Shard(parts, a, b, e, d, pk.take(d, (b - a) * e), None, gid))
            gid += 1
    lay.buf_bytes = pk.sizes()
    return lay


def dit_tensors(layers: int, hidden: int, text_dim: int = 4096) -> Tuple[List[_ModelTensor], List[List[int]]]:
    """A video-DiT-shaped parameter list (spatial + temporal self-attention, cross-attention to
    text, adaLN modulation, 4x MLP) and its FSDP units: one per block plus one for the rest."""
    h = hidden
    ts: List[_ModelTensor] = []
    units: List[List[int]] = []

    def add(unit, name, shape):
        unit.append(len(ts))
        ts.append(_ModelTensor(name, tuple(shape), None, 0))

    root: List[int] = []
    add(root, "x_embedder.proj.weight", (h, 16 * 2 * 2 * 2))
    add(root, "x_embedder.proj.bias", (h,))
    add(root, "t_embedder.mlp.0.weight", (h, 256))
    add(root, "t_embedder.mlp.0.bias", (h,))
    add(root, "t_embedder.mlp.2.weight", (h, h))
    add(root, "t_embedder.mlp.2.bias", (h,))
    add(root, "y_embedder.proj.weight", (h, text_dim))
    add(root, "y_embedder.proj.bias", (h,))
    for i in range(layers):
        u: List[int] = []
        p = f"blocks.{i}."
        add(u, p + "adaLN_modulation.weight", (6 * h, h))
        add(u, p + "adaLN_modulation.bias", (6 * h,))
        for attn in ("attn", "attn_temp"):
            add(u, p + attn + ".qkv.weight", (3 * h, h))
            add(u, p + attn + ".qkv.bias", (3 * h,))
            add(u, p + attn + ".proj.weight", (h, h))
            add(u, p + attn + ".proj.bias", (h,))
        add(u, p + "cross_attn.q.weight", (h, h))
        add(u, p + "cross_attn.q.bias", (h,))
        add(u, p + "cross_attn.kv.weight", (2 * h, h))
        add(u, p + "cross_attn.kv.bias", (2 * h,))
        add(u, p + "cross_attn.proj.weight", (h, h))
        add(u, p + "cross_attn.proj.bias", (h,))
        add(u, p + "mlp.fc1.weight", (4 * h, h))
        add(u, p + "mlp.fc1.bias", (4 * h,))
        add(u, p + "mlp.fc2.weight", (h, 4 * h))
        add(u, p + "mlp.fc2.bias", (h,))
        units.append(u)
    add(root, "final_layer.adaLN_modulation.weight", (2 * h, h))
    add(root, "final_layer.adaLN_modulation.bias", (2 * h,))
    add(root, "final_layer.linear.weight", (16 * 2 * 2 * 2, h))
    add(root, "final_layer.linear.bias", (16 * 2 * 2 * 2,))
    units.append(root)
    return ts, units


def gpt_stage_tensors(layers: int, hidden: int, vocab: int, first_stage: bool) -> Tuple[List[_ModelTensor], List[List[int]]]:
    """One pipeline stage of a GPT-3 style decoder (fused qkv, 4x MLP, biases, LayerNorm with bias)
    as Megatron lays it out; a single flat unit (the distributed optimizer's buffer)."""
    h = hidden
    ts: List[_ModelTensor] = []
    if first_stage:
        ts.append(_ModelTensor("embedding.word_embeddings.weight", (vocab, h), 0, 0))
    for i in range(layers):
        p = f"layers.{i}."
        ts += [
            _ModelTensor(p + "input_layernorm.weight", (h,), None, i),
            _ModelTensor(p + "input_layernorm.bias", (h,), None, i),
            _ModelTensor(p + "attention.qkv.weight", (3 * h, h), 0, i),
            _ModelTensor(p + "attention.qkv.bias", (3 * h,), 0, i),
            _ModelTensor(p + "attention.dense.weight", (h, h), 1, i),
            _ModelTensor(p + "attention.dense.bias", (h,), None, i),
            _ModelTensor(p + "post_attention_layernorm.weight", (h,), None, i),
            _ModelTensor(p + "post_attention_layernorm.bias", (h,), None, i),
            _ModelTensor(p + "mlp.fc1.weight", (4 * h, h), 0, i),
            _ModelTensor(p + "mlp.fc1.bias", (4 * h,), 0, i),
            _ModelTensor(p + "mlp.fc2.weight", (h, 4 * h), 1, i),
            _ModelTensor(p + "mlp.fc2.bias", (h,), None, i),
        ]
    return ts, [list(range(len(ts)))]


def moe_tensors(layers: int, hidden: int, experts: int, ffn: int):
    """Stacked expert weights: gate, up [E, ffn, h]; down [E, h, ffn].  EP splits dim 0, TP splits
    dim 1 of gate/up and dim 2 of down."""
    ts = []
    for i in range(layers):
        p = f"layers.{i}.experts."
        ts += [(p + "gate", (experts, ffn, hidden), 1),
               (p + "up", (experts, ffn, hidden), 1),
               (p + "down", (experts, hidden, ffn), 2)]
    return ts


def moe_layout(ts, ep: int, tp: int, itemsize: int, fqn_base: int = 0) -> Layout:
    pk = _Packer(ep * tp)
    lay = Layout()
    for ti, (_, shape, tp_dim) in enumerate(ts):
        for er in range(ep):
            for tr in range(tp):
                off = [0, 0, 0]
                ln = list(shape)
                ln[0] = shape[0] // ep
                off[0] = er * ln[0]
                ln[tp_dim] = shape[tp_dim] // tp
                off[tp_dim] = tr * ln[tp_dim]
                part = Part(fqn_base + ti, tuple(shape), tuple(off), tuple(ln))
                b = er * tp + tr
                lay.shards.append(regular(part, itemsize, b, pk.take(b, part.volume * itemsize)))
    lay.buf_bytes = pk.sizes()
    return lay


def _random_shapes(rng: np.random.Generator, count: int, lo: int, hi: int) -> List[Tuple[int, ...]]:
    """`count` shapes of rank 1..3 with about lo..hi elements (all draws vectorised)."""
    n = rng.integers(lo, hi + 1, size=count)
    rank = rng.integers(1, 4, size=count)
    u0, u1 = rng.random(count), rng.random(count)
    shapes = []
    for i in range(count):
        ni = int(n[i])
        if rank[i] == 1:
            shapes.append((ni,))
            continue
        d0 = 1 + int(u0[i] * max(1, int(round(ni ** 0.5))))
        rest = max(1, ni // d0)
        if rank[i] == 2:
            shapes.append((d0, rest))
            continue
        d1 = 1 + int(u1[i] * max(1, int(round(rest ** 0.5))))
        shapes.append((d0, d1, max(1, rest // d1)))
    return shapes


def _random_1d_shardings(rng: np.random.Generator, shapes, max_shards: int):
    """Per shape: one random dimension cut at sorted random points (empty shards can occur)."""
    count = len(shapes)
    udim = rng.random(count)
    ns = rng.integers(1, max_shards + 1, size=count)
    ucut = rng.random((count, max(max_shards - 1, 0)))
    out = []
    for i, shape in enumerate(shapes):
        dim = int(udim[i] * len(shape))
        ln_d = shape[dim]
        k = int(ns[i]) - 1
        cuts = sorted(int(c * (ln_d + 1)) for c in ucut[i, :k])
        edges = [0] + cuts + [ln_d]
        boxes = []
        for a, b in zip(edges[:-1], edges[1:]):
            off = [0] * len(shape)
            ln = list(shape)
            off[dim], ln[dim] = a, b - a
            boxes.append((tuple(off), tuple(ln)))
        out.append(boxes)
    return out


def small_tensor_case(n_tensors: int, seed: int, n_bufs: int = 64, max_shards: int = 16,
                      lo: int = 4, hi: int = 4096, fqn_base: int = 0,
                      dtype: torch.dtype = torch.float32, granule: int = 4,
                      buf_base: Tuple[int, int] = (0, 0)):
    """Many small random-shape tensors under independent random 1-D shardings on the saved
    and the target side, packed at `granule`-byte granularity into `n_bufs` buffers each."""
    rng = np.random.default_rng(seed)
    e = dtype.itemsize
    specs: Dict[int, TensorSpec] = {}
    saved, target = Layout(), Layout()
    pks = _Packer(n_bufs, granule), _Packer(n_bufs, granule)
    shapes = _random_shapes(rng, n_tensors, lo, hi)
    for i, shape in enumerate(shapes):
        specs[fqn_base + i] = TensorSpec(fqn_base + i, f"small.{i}", shape, dtype, ("normal", 0.0, 1.0))
    for lay, pk, base in ((saved, pks[0], buf_base[0]), (target, pks[1], buf_base[1])):
        shardings = _random_1d_shardings(rng, shapes, max_shards)
        bufs = rng.integers(0, n_bufs, size=sum(len(b) for b in shardings))
        j = 0
        for i, boxes in enumerate(shardings):
            for off, ln in boxes:
                part = Part(fqn_base + i, shapes[i], off, ln)
                b = int(bufs[j])
                j += 1
                lay.shards.append(regular(part, e, base + b, pk.take(b, part.volume * e)))
    saved.buf_bytes = pks[0].sizes()
    target.buf_bytes = pks[1].sizes()
    return specs, saved, target


# ----------------------------------------------------------------------------------------
# the five benchmark configurations (full size by default; every builder takes smaller
# dimensions so tests can run the same structure at sizes a CPU finishes in seconds)
# ----------------------------------------------------------------------------------------
def cfg1(n: int = 1024, m: int = 1024, strided_target: bool = False) -> Case:
    """One fp32 [n,m] tensor, uniform[-1,1); saved as 2 row shards, loaded as 4 column shards.
    strided_target: each target buffer holds its [n, m/4] shard column-major (a transposed view)."""
    spec = TensorSpec(0, "w", (n, m), torch.float32, ("uniform", -1.0, 1.0))
    saved, target = Layout(), Layout()
    for r in range(2):
        part = Part(0, (n, m), (r * (n // 2), 0), (n // 2, m))
        saved.shards.append(regular(part, 4, r, 0))
        saved.buf_bytes.append(part.volume * 4)
    for c in range(4):
        part = Part(0, (n, m), (0, c * (m // 4)), (n, m // 4))
        strides = (1, n) if strided_target else None
        target.shards.append(regular(part, 4, c, 0, strides))
        target.buf_bytes.append(part.volume * 4)
    return Case("cfg1" + ("_strided" if strided_target else ""), BASE_SEED + 1, {0: spec}, saved, target)


def transpose_case(n: int = 16384, m: int = 16384, dtype: torch.dtype = torch.float32, shards: int = 4) -> Case:
    """A [n, m] tensor saved row-major in `shards` row blocks and loaded as `shards` column blocks whose
    buffers hold them column-major (a transposed view: BasicMeta strides (1, n)): every region takes
    the LDS-staged path."""
    e = dtype.itemsize
    spec = TensorSpec(0, "w", (n, m), dtype, ("bits",))
    saved, target = Layout(), Layout()
    for r in range(shards):
        part = Part(0, (n, m), (r * (n // shards), 0), (n // shards, m))
        saved.shards.append(regular(part, e, r, 0))
        saved.buf_bytes.append(part.volume * e)
    for c in range(shards):
        part = Part(0, (n, m), (0, c * (m // shards)), (n, m // shards))
        target.shards.append(regular(part, e, c, 0, (1, n)))
        target.buf_bytes.append(part.volume * e)
    return Case(f"transpose_{n}x{m}", BASE_SEED + 9, {0: spec}, saved, target)


def column_blocks_case(n: int = 16384, m: int = 16384, cols: int = 128, strided_side: str = "read",
                       dtype: torch.dtype = torch.float32) -> Case:
    """A [n, m] tensor held whole (row-major) on one side and as m/cols column blocks [n, cols], packed
    one after the other into a single buffer, on the other: a plain row copy with runs of cols elements
    at a pitch of m elements on the strided side and none on the other -- the access pattern of
    `transpose_case` without the transposition.  strided_side "read": the whole tensor is the source."""
    e = dtype.itemsize
    spec = TensorSpec(0, "w", (n, m), dtype, ("bits",))
    whole = Layout([regular(Part(0, (n, m), (0, 0), (n, m)), e, 0, 0)], [n * m * e])
    split = Layout()
    off = 0
    for c in range(m // cols):
        part = Part(0, (n, m), (0, c * cols), (n, cols))
        split.shards.append(regular(part, e, 0, off))
        off += part.volume * e
    split.buf_bytes.append(off)
    saved, target = (whole, split) if strided_side == "read" else (split, whole)
    return Case(f"column_blocks_{strided_side}_{cols}", BASE_SEED + 10, {0: spec}, saved, target)


def copy_case(nbytes: int = 8 << 30, src_shift: int = 0, dst_shift: int = 0) -> Case:
    """One byte tensor saved whole and loaded whole: the reshard degenerates to a plain copy
    (the practical bandwidth ceiling of the copy kernel).  Shifts move the shard inside its
    buffer to give source and destination different alignments."""
    spec = TensorSpec(0, "bytes", (nbytes,), torch.uint8, ("bits",))
    part = Part(0, (nbytes,), (0,), (nbytes,))
    return Case(f"copy_{src_shift}_{dst_shift}", BASE_SEED, {0: spec},
                Layout([regular(part, 1, 0, src_shift)], [nbytes + src_shift]),
                Layout([regular(part, 1, 0, dst_shift)], [nbytes + dst_shift]))


def regions_case(size: int, src_gap: int = 0, dst_gap: int = 0, jitter: int = 0, total: int = 6 << 30) -> Case:
    """About `total` bytes as byte tensors of `size` (+ up to `jitter`, drawn per tensor) bytes, packed into one
    buffer on either side with `src_gap` / `dst_gap` bytes before each: a plain copy cut into regions, to
    show what the region size (partial tiles at both ends of a region) and the alignment of the two sides cost."""
    rng = np.random.default_rng(BASE_SEED + 12)
    specs: Dict[int, TensorSpec] = {}
    sv, tg, so, to, f = [], [], src_gap, dst_gap, 0
    while so + size + jitter <= total:
        n = size + (int(rng.integers(0, jitter)) if jitter else 0)
        specs[f] = TensorSpec(f, f"r{f}", (n,), torch.uint8, ("bits",))
        part = Part(f, (n,), (0,), (n,))
        sv.append(regular(part, 1, 0, so))
        tg.append(regular(part, 1, 0, to))
        so += n + src_gap
        to += n + dst_gap
        f += 1
    return Case(f"regions_{size}_{src_gap}_{dst_gap}_{jitter}", BASE_SEED + 12, specs, Layout(sv, [so]), Layout(tg, [to]))


def llama_case(name: str, seed: int, layers: int, hidden: int, ffn: int, vocab: int, states,
               tp_s: int, pp_s: int, tp_t: int, pp_t: int, only_target_ranks=None) -> Case:
    model = llama_tensors(layers, hidden, ffn, vocab)
    return Case(name, seed, _specs(model, states),
                megatron_layout(model, states, layers, tp_s, pp_s, replicate_norms=False),
                megatron_layout(model, states, layers, tp_t, pp_t, replicate_norms=True,
                                only_ranks=only_target_ranks))


def narrowed(layout: Layout) -> Layout:
    """The same layout asked for with 2-byte elements instead of 4-byte ones (an evaluation job that
    loads fp32 master weights as bf16, Sec. 2.2): same boxes, flat ranges and element strides, every
    byte offset and buffer size halved (shards that were disjoint stay disjoint)."""
    shards = []
    for sh in layout.shards:
        assert sh.itemsize == 4
        shards.append(Shard(sh.parts, sh.flat_begin, sh.flat_end, 2, sh.buf, sh.byte_offset // 2, sh.strides, sh.group))
    return Layout(shards, [max(1, (n + 1) // 2) for n in layout.buf_bytes])


def eval_load_case(layers: int = 32, hidden: int = 4096, ffn: int = 11008, vocab: int = 32000,
                   zero_saved: bool = False) -> Case:
    """An evaluation job loads the model only (Sec. 2.2): the fp32 master weights of the 7B-shaped
    decoder, saved TP4 PP2 (or, zero_saved, as a ZeRO flat buffer cut over DP16), are loaded as bf16
    weights under TP2 PP4.  Every tensor is converted on the way."""
    model = llama_tensors(layers, hidden, ffn, vocab)
    states = [STATE_FP32_MASTER]
    saved = (zero_layout(model, states, 1, 16, replicate_norms=False) if zero_saved
             else megatron_layout(model, states, layers, 4, 2, replicate_norms=False))
    target = narrowed(megatron_layout(model, states, layers, 2, 4, replicate_norms=True))
    return Case("eval_load" + ("_zero" if zero_saved else ""), BASE_SEED + 6, _specs(model, states), saved, target, convert=1)


def cfg2(layers: int = 24, hidden: int = 2048, ffn: int = 5504, vocab: int = 32000) -> Case:
    """bf16 decoder saved TP4 PP2, loaded TP2 PP4, all target shards."""
    return llama_case("cfg2", BASE_SEED + 2, layers, hidden, ffn, vocab, [STATE_BF16_WEIGHT], 4, 2, 2, 4)


CFG3_STATES = [STATE_BF16_WEIGHT, STATE_FP32_MASTER, STATE_FP32_EXP_AVG, STATE_FP32_EXP_AVG_SQ]


def cfg3(layers: int = 32, hidden: int = 4096, ffn: int = 11008, vocab: int = 32000,
         rank_share: bool = False) -> Case:
    """7B-shaped decoder, bf16 weights + three fp32 Adam states, TP4 PP2 -> TP2 PP4.
    rank_share: only target rank (pp 0, tp 0)."""
    return llama_case("cfg3" + ("_rank0" if rank_share else ""), BASE_SEED + 3, layers, hidden, ffn, vocab,
                      CFG3_STATES, 4, 2, 2, 4, only_target_ranks=[(0, 0)] if rank_share else None)


CFG4_STATES = [STATE_FP32_MASTER, STATE_FP32_EXP_AVG, STATE_FP32_EXP_AVG_SQ]


def cfg4(layers: int = 32, hidden: int = 4096, ffn: int = 11008, vocab: int = 32000,
         dp_s: int = 16, dp_t: int = 12, tp_t: int = 2, n_states: int = 3) -> Case:
    """fp32 optimizer states flattened in parameter order: saved TP1 DP16, loaded TP2 DP12."""
    model = llama_tensors(layers, hidden, ffn, vocab)
    states = CFG4_STATES[:n_states]
    return Case("cfg4", BASE_SEED + 4, _specs(model, states),
                zero_layout(model, states, 1, dp_s, replicate_norms=False),
                zero_layout(model, states, tp_t, dp_t, replicate_norms=True))


ADAM_FP32_STATES = [STATE_FP32_MASTER, STATE_FP32_EXP_AVG, STATE_FP32_EXP_AVG_SQ]


def table3_vdit(dp_s: int = 32, dp_t: int = 64, layers: int = 48, hidden: int = 1664, text_dim: int = 4096) -> Case:
    """Shaped like the paper's vDiT rows of Table 3 (hidden 1664, 48 layers, FSDP ZeRO-2, 32 -> 64 and
    128 -> 64 GPUs): bf16 flat parameters and fp32 Adam states, one FSDP unit per block, every unit
    cut evenly over the DP ranks.  The model itself is internal to the paper; this is a DiT-style
    stand-in of the same width and depth (about 3.5 B parameters)."""
    model, units = dit_tensors(layers, hidden, text_dim)
    states = [STATE_BF16_WEIGHT] + ADAM_FP32_STATES
    return Case(f"vdit_dp{dp_s}to{dp_t}", BASE_SEED + 6, _specs(model, states),
                flat_units_layout(model, states, units, dp_s), flat_units_layout(model, states, units, dp_t))


def table3_tgpt_group(dp_s: int = 75, dp_t: int = 150, layers: int = 10, hidden: int = 8192, vocab: int = 51200,
                      tp: int = 4, first_stage: bool = True) -> Case:
    """Shaped like the paper's tGPT 70B rows of Table 3 (hidden 8192, 80 layers, TP4 PP8, DP 75 <-> 150):
    ONE (tp rank 0, pp stage) group -- 10 of the 80 layers, plus the vocab-parallel embedding on the
    first stage -- whose fp32 Adam states sit in Megatron's distributed-optimizer buffer cut over the
    DP ranks.  All target DP ranks of the group are built on one GPU (26 GB one way)."""
    model, units = gpt_stage_tensors(layers, hidden, vocab, first_stage)
    return Case(f"tgpt_dp{dp_s}to{dp_t}", BASE_SEED + 7, _specs(model, ADAM_FP32_STATES),
                flat_units_layout(model, ADAM_FP32_STATES, units, dp_s, tp=tp, tp_rank=0),
                flat_units_layout(model, ADAM_FP32_STATES, units, dp_t, tp=tp, tp_rank=0))


def fused_qkv_case(layers: int = 32, hidden: int = 4096, n_heads: int = 32, n_kv: int = 8, tp_s: int = 4,
                   tp_t: int = 2, dtype: torch.dtype = torch.bfloat16) -> Case:
    """The layout change Appendix A names as a pain point of resharding scripts: grouped-query
    attention stored as ONE fused, group-interleaved QKV weight per TP rank (per KV group: its query
    heads, then its key head, then its value head) is loaded as separate q, k, v tensors under a
    different TP degree.  No special support is needed: the fused blob is described by one record
    per (group, q|k|v) block, each a box of the q, k or v tensor with its byte offset in the blob."""
    d = hidden // n_heads
    qpg = n_heads // n_kv
    assert n_kv % tp_s == 0 and n_heads % tp_t == 0 and n_kv % tp_t == 0
    e = dtype.itemsize
    specs: Dict[int, TensorSpec] = {}
    saved, target = Layout(), Layout()
    pks, pkt = _Packer(tp_s), _Packer(tp_t)
    for l in range(layers):
        fq, fk, fv = 3 * l, 3 * l + 1, 3 * l + 2
        shapes = {fq: (n_heads * d, hidden), fk: (n_kv * d, hidden), fv: (n_kv * d, hidden)}
        for f, nm in ((fq, "q"), (fk, "k"), (fv, "v")):
            specs[f] = TensorSpec(f, f"layers.{l}.attn.{nm}.weight", shapes[f], dtype, ("normal", 0.0, 0.02))
        gps = n_kv // tp_s
        for r in range(tp_s):
            base = pks.take(r, gps * (qpg + 2) * d * hidden * e)  # one fused block per layer and rank
            off = base
            for g in range(r * gps, (r + 1) * gps):
                for f, row0, rows in ((fq, g * qpg * d, qpg * d), (fk, g * d, d), (fv, g * d, d)):
                    part = Part(f, shapes[f], (row0, 0), (rows, hidden))
                    saved.shards.append(regular(part, e, r, off))
                    off += rows * hidden * e
        for r in range(tp_t):
            for f in (fq, fk, fv):
                rows = shapes[f][0] // tp_t
                part = Part(f, shapes[f], (r * rows, 0), (rows, hidden))
                target.shards.append(regular(part, e, r, pkt.take(r, part.volume * e)))
    saved.buf_bytes, target.buf_bytes = pks.sizes(), pkt.sizes()
    return Case(f"fused_qkv_tp{tp_s}to{tp_t}", BASE_SEED + 8, specs, saved, target)


def cfg5(layers: int = 16, hidden: int = 4096, experts: int = 64, ffn: int = 1408,
         n_small: int = 100_000, include_experts: bool = True) -> Case:
    """bf16 stacked expert weights EP8 TP2 -> EP4 TP4 (16 buffers each side) plus `n_small`
    small fp32 tensors under random 1-D shardings in 64 further buffers each side."""
    seed = BASE_SEED + 5
    specs: Dict[int, TensorSpec] = {}
    saved, target = Layout(), Layout()
    nb = 0
    if include_experts:
        ts = moe_tensors(layers, hidden, experts, ffn)
        for i, (nm, shape, _) in enumerate(ts):
            specs[i] = TensorSpec(i, nm, shape, torch.bfloat16, ("normal", 0.0, 0.02))
        saved = moe_layout(ts, 8, 2, 2)
        target = moe_layout(ts, 4, 4, 2)
        nb = 16
    if n_small:
        sp, s2, t2 = small_tensor_case(n_small, seed, fqn_base=len(specs), buf_base=(nb, nb))
        specs.update(sp)
        saved.shards += s2.shards
        saved.buf_bytes += s2.buf_bytes
        target.shards += t2.shards
        target.buf_bytes += t2.buf_bytes
    return Case("cfg5", seed, specs, saved, target)


# ----------------------------------------------------------------------------------------
# randomised small cases (parity tests)
# ----------------------------------------------------------------------------------------
def _random_cuts(rng, n: int, max_cuts: int) -> List[int]:
    k = int(rng.integers(0, max_cuts + 1))
    return [0] + sorted(int(c) for c in rng.integers(0, n + 1, size=k)) + [n]


def _grid_boxes(rng, shape, max_cuts: int):
    """Partition a shape into a grid of boxes by cutting every dimension at random points."""
    edges = [_random_cuts(rng, n, max_cuts) for n in shape]
    boxes = [((), ())]
    for e in edges:
        boxes = [(o + (a,), l + (b - a,)) for (o, l) in boxes for a, b in zip(e[:-1], e[1:])]
    return boxes


def _permuted_strides(rng, lengths, pad: bool):
    """Element strides of a buffer that stores the box with its dimensions in a random order
    (optionally with padding between rows)."""
    order = list(rng.permutation(len(lengths)))  # order[0] slowest ... order[-1] fastest
    strides = [0] * len(lengths)
    s = 1
    for d in reversed(order):
        strides[d] = s
        s *= max(1, lengths[d]) + (int(rng.integers(0, 3)) if pad else 0)
    return tuple(strides), s


def _random_grid_layout(rng, specs, n_bufs: int, granule: int, max_cuts: int, p_strided: float) -> Layout:
    pk = _Packer(n_bufs, granule)
    lay = Layout()
    for fqn, spec in specs.items():
        e = spec.dtype.itemsize
        for off, ln in _grid_boxes(rng, spec.shape, max_cuts):
            part = Part(fqn, tuple(spec.shape), off, ln)
            b = int(rng.integers(0, n_bufs))
            if len(ln) >= 1 and part.volume > 0 and rng.random() < p_strided:
                strides, span = _permuted_strides(rng, ln, pad=bool(rng.integers(0, 2)))
                pk.align = max(granule, e)  # typed strided views need itemsize-aligned storage
                lay.shards.append(regular(part, e, b, pk.take(b, span * e), strides))
                pk.align = granule
            else:
                lay.shards.append(regular(part, e, b, pk.take(b, part.volume * e)))
    lay.buf_bytes = pk.sizes()
    return lay


def _random_flat_layout(rng, specs, tp: int, dp: int, granule: int, pack_bufs: int) -> Layout:
    """ZeRO-like: every tensor is first cut along one random dimension into `tp` (possibly
    uneven) pieces; per piece index the pieces are flattened and concatenated in FQN order and
    the concatenation is cut into `dp` even slices.  Slices are packed into `pack_bufs` buffers."""
    pk = _Packer(pack_bufs, granule)
    lay = Layout()
    cuts = {}
    for fqn, spec in specs.items():
        if len(spec.shape) == 0:
            cuts[fqn] = None
            continue
        d = int(rng.integers(0, len(spec.shape)))
        n = spec.shape[d]
        edges = [0] + sorted(int(c) for c in rng.integers(0, n + 1, size=tp - 1)) + [n]
        cuts[fqn] = (d, edges)
    e = next(iter(specs.values())).dtype.itemsize
    for r in range(tp):
        parts = []
        for fqn, spec in specs.items():
            if cuts[fqn] is None:
                if r == 0:
                    parts.append(Part(fqn, (), (), ()))
                continue
            d, edges = cuts[fqn]
            off = [0] * len(spec.shape)
            ln = list(spec.shape)
            off[d], ln[d] = edges[r], edges[r + 1] - edges[r]
            parts.append(Part(fqn, tuple(spec.shape), tuple(off), tuple(ln)))
        parts = tuple(parts)
        n = sum(p.volume for p in parts)
        chunk = max(1, -(-n // dp))
        for k in range(dp):
            a, b = min(n, k * chunk), min(n, (k + 1) * chunk)
            buf = int(rng.integers(0, pack_bufs))
            lay.shards.append(Shard(parts, a, b, e, buf, pk.take(buf, (b - a) * e), None, r))
    lay.buf_bytes = pk.sizes()
    return lay


RANDOM_DTYPES = (torch.uint8, torch.bfloat16, torch.float32, torch.float64, torch.complex128)  # 1..16 bytes


def random_case(seed: int, n_tensors: int = 5, max_elems: int = 3000, saved_mode: str = "grid",
                target_mode: str = "grid", max_rank: int = 4, granules=(1, 2, 4, 8, 16, 256),
                p_strided: float = 0.0, dtype: Optional[torch.dtype] = None, narrow_target: bool = False) -> Case:
    """Small random tensors (rank 0..max_rank, arbitrary bit patterns) under random saved and
    target layouts.  'grid': boxes from random cuts in every dimension; 'flat': ZeRO-like slices
    of concatenated pieces (single dtype for the whole case).  narrow_target (dtype float32 only):
    the target asks for every tensor as bf16."""
    assert not narrow_target or dtype == torch.float32
    rng = np.random.default_rng(seed)
    flat = "flat" in (saved_mode, target_mode)
    one_dtype = dtype if dtype is not None else (RANDOM_DTYPES[int(rng.integers(0, len(RANDOM_DTYPES)))] if flat else None)
    specs: Dict[int, TensorSpec] = {}
    for i in range(n_tensors):
        rank = int(rng.integers(0, max_rank + 1))
        total = int(rng.integers(1, max_elems + 1))
        shape = []
        rest = total
        for k in range(rank):
            if k == rank - 1:
                shape.append(max(1, rest))
            else:
                d = int(rng.integers(1, max(2, int(round(rest ** (1.0 / (rank - k)))) * 2)))
                shape.append(d)
                rest = max(1, rest // d)
        rng.shuffle(shape)
        dt = one_dtype or RANDOM_DTYPES[int(rng.integers(0, len(RANDOM_DTYPES)))]
        specs[i] = TensorSpec(i, f"t{i}", tuple(int(s) for s in shape), dt, ("bits",))

    def side(mode):
        g = int(granules[int(rng.integers(0, len(granules)))])
        if mode == "grid":
            return _random_grid_layout(rng, specs, int(rng.integers(1, 5)), g, 3, p_strided)
        return _random_flat_layout(rng, specs, int(rng.integers(1, 4)), int(rng.integers(1, 7)), g,
                                   int(rng.integers(1, 4)))

    saved, target = side(saved_mode), side(target_mode)
    if narrow_target:
        return Case(f"random{seed}_narrow", seed, specs, saved, narrowed(target), convert=1)
    return Case(f"random{seed}", seed, specs, saved, target)
