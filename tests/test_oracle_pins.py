"""Pins for the CPU oracle: it is checked against things other than itself.

* the paper's worked example of an irregular shard (Sec. 3.2, "Decomposing irregular tensors"),
  values from tests/golden/paper_irregular_example.txt;
* a closed form that involves neither the oracle nor the HIP path: blobs of any layout are cut out
  of seeded global tensors with library slicing (synth.materialize), so resharding saved->target
  must reproduce materialize(target);
* invariants: reassembly into the whole tensor, A->B->A identity, every target byte written exactly
  once and nothing else touched;
* brute force on tiny tensors: for each target element, search all saved shards for the one that
  contains its global coordinates (numpy ravel/unravel as the library routine);
* special cases that are textbook routines: identity layout == memcpy, row shards -> column shards
  == numpy concatenate + slice.
"""
import math

import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2407_20143_amd import synth
from paper_2407_20143_amd.synth import Case, Layout, Part, Shard, TensorSpec, regular

POISON = 0xA5


def run(case: Case, **kw):
    src = synth.materialize(case.saved, case.tensors, case.seed)
    return src, oracle.reshard(case.saved, case.target, src, poison=POISON, **kw)


def expect(case: Case):
    return [b.numpy() for b in synth.materialize(case.target, case.tensors, case.seed, poison=POISON)]


def assert_bufs_equal(got, want):
    assert len(got) == len(want)
    for i, (g, w) in enumerate(zip(got, want)):
        assert g.shape == w.shape
        if not np.array_equal(g, w):
            bad = np.flatnonzero(g != w)
            raise AssertionError(f"buffer {i}: {bad.size} bytes differ, first at {bad[0]}")


# ------------------------------------------------------------------------------------------
# the paper's example
# ------------------------------------------------------------------------------------------
def _ints(s):
    return [int(v) for v in s.split()]


def _paper_layout():
    A = Part(0, (2,), (0,), (2,))
    B = Part(1, (3, 2), (0, 0), (3, 2))
    C = Part(2, (2,), (0,), (2,))
    parts = (A, B, C)
    saved = Layout([Shard(parts, 0, 5, 4, 0, 0, None, 0), Shard(parts, 5, 10, 4, 1, 0, None, 0)], [20, 20])
    return parts, saved


def test_paper_irregular_example(golden_irregular):
    g = golden_irregular
    assert int(g["flat_cut"]) == 5
    _, saved = _paper_layout()
    src = [np.array(_ints(g["rank0_flat"]), dtype=np.float32).view(np.uint8),
           np.array(_ints(g["rank1_flat"]), dtype=np.float32).view(np.uint8)]
    B = lambda off, ln: Part(1, (3, 2), off, ln)
    # whole B; two column shards; three row shards -- each in its own buffer
    target = Layout([regular(B((0, 0), (3, 2)), 4, 0, 0),
                     regular(B((0, 0), (3, 1)), 4, 1, 0), regular(B((0, 1), (3, 1)), 4, 2, 0),
                     regular(B((0, 0), (1, 2)), 4, 3, 0), regular(B((1, 0), (1, 2)), 4, 3, 8),
                     regular(B((2, 0), (1, 2)), 4, 3, 16)], [24, 12, 12, 24])
    dst = oracle.reshard(saved, target, src)
    f = lambda b: list(dst[b].view(np.float32).astype(int))
    assert f(0) == _ints(g["B_full"])
    assert f(1) == _ints(g["B_col0"])
    assert f(2) == _ints(g["B_col1"])
    assert f(3) == _ints(g["B_row_shards"].replace("|", " "))
    # the neighbours A and C come back whole
    t2 = Layout([regular(Part(0, (2,), (0,), (2,)), 4, 0, 0), regular(Part(2, (2,), (0,), (2,)), 4, 0, 8)], [16])
    d2 = oracle.reshard(saved, t2, src)
    assert list(d2[0].view(np.float32).astype(int)) == [0, 1, 200, 201]


def test_paper_example_boxes_as_saved_layout(golden_irregular):
    """The decomposition the fixture lists for B (two boxes per rank) describes the same bytes:
    feeding those boxes to the oracle as regular saved shards gives the same result."""
    g = golden_irregular

    def boxes(s):
        out = []
        for tok in s.split():
            o, l = tok.split("+")
            out.append((tuple(int(v) for v in o.strip("()").split(",")), tuple(int(v) for v in l.strip("()").split(","))))
        return out

    b0, b1 = boxes(g["B_rank0_boxes"]), boxes(g["B_rank1_boxes"])
    assert len(b0) == int(g["B_rank0_box_count"]) == 2
    src = [np.array(_ints(g["rank0_flat"]), dtype=np.float32).view(np.uint8),
           np.array(_ints(g["rank1_flat"]), dtype=np.float32).view(np.uint8)]
    shards = []
    # rank 0's blob: A (2 elements) then B's boxes; rank 1's blob: B's boxes then C
    off = 8
    for o, l in b0:
        shards.append(regular(Part(1, (3, 2), o, l), 4, 0, off))
        off += 4 * math.prod(l)
    assert off == 20
    off = 0
    for o, l in b1:
        shards.append(regular(Part(1, (3, 2), o, l), 4, 1, off))
        off += 4 * math.prod(l)
    assert off == 12
    target = Layout([regular(Part(1, (3, 2), (0, 0), (3, 2)), 4, 0, 0)], [24])
    dst = oracle.reshard(Layout(shards, [20, 20]), target, src)
    assert list(dst[0].view(np.float32).astype(int)) == _ints(g["B_full"])


# ------------------------------------------------------------------------------------------
# closed form: library slicing of the seeded global tensors
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("modes", [("grid", "grid"), ("grid", "flat"), ("flat", "grid"), ("flat", "flat")])
@pytest.mark.parametrize("seed", range(6))
def test_closed_form_random(seed, modes):
    case = synth.random_case(1000 + seed, saved_mode=modes[0], target_mode=modes[1])
    _, got = run(case)
    assert_bufs_equal(got, expect(case))


@pytest.mark.parametrize("seed", range(6))
def test_closed_form_strided(seed):
    case = synth.random_case(2000 + seed, p_strided=0.6, granules=(4, 8, 16))
    _, got = run(case)
    assert_bufs_equal(got, expect(case))


def test_closed_form_model_shapes():
    """Scaled-down versions of the five benchmark layouts."""
    cases = [synth.cfg1(64, 48), synth.cfg1(64, 48, strided_target=True),
             synth.cfg2(layers=4, hidden=32, ffn=88, vocab=64),
             synth.cfg3(layers=4, hidden=32, ffn=88, vocab=64),
             synth.cfg3(layers=4, hidden=32, ffn=88, vocab=64, rank_share=True),
             synth.cfg4(layers=2, hidden=24, ffn=40, vocab=52, dp_s=16, dp_t=12),
             synth.cfg5(layers=1, hidden=16, experts=8, ffn=12, n_small=50),
             synth.fused_qkv_case(layers=2, hidden=32, n_heads=8, n_kv=4, tp_s=4, tp_t=2),
             synth.fused_qkv_case(layers=1, hidden=48, n_heads=12, n_kv=6, tp_s=2, tp_t=3, dtype=torch.float32),
             synth.table3_vdit(8, 16, layers=2, hidden=24, text_dim=40),
             synth.table3_vdit(16, 8, layers=2, hidden=24, text_dim=40),
             synth.table3_tgpt_group(5, 10, layers=2, hidden=32, vocab=128),
             synth.table3_tgpt_group(10, 5, layers=1, hidden=32, vocab=128, first_stage=False),
             synth.regions_case(700, 4, 12, 90, total=40_000), synth.copy_case(5000, 3, 9),
             synth.column_blocks_case(40, 96, 8, "write")]
    for case in cases:
        _, got = run(case)
        assert_bufs_equal(got, expect(case))


# ------------------------------------------------------------------------------------------
# invariants
# ------------------------------------------------------------------------------------------
def _whole_tensor_target(case: Case) -> Layout:
    lay = Layout()
    for fqn, spec in case.tensors.items():
        part = Part(fqn, tuple(spec.shape), (0,) * len(spec.shape), tuple(spec.shape))
        lay.shards.append(regular(part, spec.dtype.itemsize, len(lay.buf_bytes), 0))
        lay.buf_bytes.append(max(1, part.volume * spec.dtype.itemsize))
    return lay


@pytest.mark.parametrize("seed", range(4))
def test_reassembly_is_layout_independent(seed):
    """Reassembling the whole tensors from two different shardings of the same data is identical
    (and equals the data)."""
    a = synth.random_case(3000 + seed, saved_mode="grid")
    b = synth.random_case(3000 + seed, saved_mode="flat", dtype=torch.float32)
    for case in (a, b):
        whole = _whole_tensor_target(case)
        src = synth.materialize(case.saved, case.tensors, case.seed)
        got = oracle.reshard(case.saved, whole, src, poison=0)
        # a second, different sharding of the same tensors
        other = case.target
        mid = oracle.reshard(case.saved, other, src, poison=0)
        got2 = oracle.reshard(other, whole, mid, poison=0)
        assert_bufs_equal(got, got2)
        for (fqn, spec), buf in zip(case.tensors.items(), got):
            G = synth.global_tensor(spec, case.seed).contiguous().view(-1).view(torch.uint8).numpy()
            assert np.array_equal(buf[:G.size], G)


@pytest.mark.parametrize("modes", [("grid", "grid"), ("flat", "grid"), ("grid", "flat")])
@pytest.mark.parametrize("seed", range(3))
def test_round_trip_identity(seed, modes):
    case = synth.random_case(4000 + seed, saved_mode=modes[0], target_mode=modes[1])
    src = synth.materialize(case.saved, case.tensors, case.seed, poison=POISON)
    mid = oracle.reshard(case.saved, case.target, src, poison=0x11)
    back = oracle.reshard(case.target, case.saved, mid, poison=POISON)
    assert_bufs_equal(back, [b.numpy() for b in src])


@pytest.mark.parametrize("seed", range(4))
def test_every_target_byte_written_exactly_once(seed):
    case = synth.random_case(5000 + seed, saved_mode="flat", target_mode="grid", p_strided=0.3, granules=(4, 8))
    src = synth.materialize(case.saved, case.tensors, case.seed)
    dst, written = oracle.reshard(case.saved, case.target, src, poison=POISON, want_written=True)
    cover = synth.coverage_mask(case.target, case.tensors)
    for w, c, d in zip(written, cover, dst):
        covered = c.numpy() == 1
        assert np.all(w[covered] == 1)
        assert np.all(w[~covered] == 0)
        assert np.all(d[~covered] == POISON)


# ------------------------------------------------------------------------------------------
# brute force
# ------------------------------------------------------------------------------------------
def _brute(case: Case, src):
    dst = [np.full(n, POISON, dtype=np.uint8) for n in case.target.buf_bytes]

    def elements(sh: Shard):
        """(stored byte position, fqn, global coords) of every stored element of a packed shard."""
        pos = 0
        for p in sh.parts:
            for local in range(p.volume):
                ci = pos + local
                if sh.flat_begin <= ci < sh.flat_end:
                    y = np.unravel_index(local, p.lengths) if p.lengths else ()
                    x = tuple(int(o + v) for o, v in zip(p.offsets, y))
                    yield sh.byte_offset + sh.itemsize * (ci - sh.flat_begin), p.fqn, x
            pos += p.volume

    def find(fqn, x):
        hits = []
        for sh in case.saved.shards:
            pos = 0
            for p in sh.parts:
                if p.fqn == fqn and all(o <= v < o + l for o, v, l in zip(p.offsets, x, p.lengths)):
                    local = int(np.ravel_multi_index(tuple(v - o for v, o in zip(x, p.offsets)), p.lengths)) if p.lengths else 0
                    ci = pos + local
                    if sh.flat_begin <= ci < sh.flat_end:
                        hits.append((sh, sh.byte_offset + sh.itemsize * (ci - sh.flat_begin)))
                pos += p.volume
        assert len(hits) == 1, (fqn, x, len(hits))
        return hits[0]

    for sh in case.target.shards:
        for byte, fqn, x in elements(sh):
            ssh, sbyte = find(fqn, x)
            dst[sh.buf][byte:byte + sh.itemsize] = src[ssh.buf].numpy()[sbyte:sbyte + sh.itemsize]
    return dst


@pytest.mark.parametrize("modes", [("grid", "grid"), ("grid", "flat"), ("flat", "grid"), ("flat", "flat")])
@pytest.mark.parametrize("seed", range(3))
def test_brute_force_tiny(seed, modes):
    case = synth.random_case(6000 + seed, n_tensors=3, max_elems=60, saved_mode=modes[0], target_mode=modes[1],
                             max_rank=3)
    src, got = run(case)
    assert_bufs_equal(got, _brute(case, src))


# ------------------------------------------------------------------------------------------
# special cases that are library routines
# ------------------------------------------------------------------------------------------
def test_identity_layout_is_memcpy():
    case = synth.random_case(7000, saved_mode="grid")
    src = synth.materialize(case.saved, case.tensors, case.seed, poison=POISON)
    got = oracle.reshard(case.saved, case.saved, src, poison=POISON)
    assert_bufs_equal(got, [b.numpy() for b in src])


def test_rows_to_columns_is_concatenate_and_slice():
    case = synth.cfg1(128, 96)
    src, got = run(case)
    rows = np.concatenate([b.numpy().view(np.float32).reshape(64, 96) for b in src], axis=0)
    for c in range(4):
        want = np.ascontiguousarray(rows[:, 24 * c:24 * (c + 1)])
        assert np.array_equal(got[c].view(np.float32).reshape(128, 24), want)
    # values are uniform in [-1, 1)
    assert rows.min() >= -1.0 and rows.max() < 1.0


def test_flat_rechunk_is_array_split():
    """ZeRO DP a -> DP b at TP=1 only re-chunks one flat array."""
    model = synth.llama_tensors(2, 8, 12, 20)
    states = [synth.STATE_FP32_MASTER]
    specs = synth._specs(model, states)
    a = synth.zero_layout(model, states, 1, 16, replicate_norms=False)
    b = synth.zero_layout(model, states, 1, 12, replicate_norms=True)
    case = Case("rechunk", 9, specs, a, b)
    src, got = run(case)
    flat = np.concatenate([s.numpy() for s in src])
    n = sum(sh.numel for sh in a.shards)
    assert flat.size == n * 4
    chunk = -(-n // 12) * 4
    for k in range(12):
        want = flat[k * chunk:(k + 1) * chunk]
        assert np.array_equal(got[k][:want.size], want)


# ------------------------------------------------------------------------------------------
# error behaviour
# ------------------------------------------------------------------------------------------
def _simple(n=8):
    spec = TensorSpec(0, "w", (n, 4), torch.float32, ("normal", 0.0, 1.0))
    full = Part(0, (n, 4), (0, 0), (n, 4))
    return spec, full


def test_saved_overlap_is_an_error():
    spec, full = _simple()
    half = Part(0, (8, 4), (0, 0), (5, 4))
    half2 = Part(0, (8, 4), (4, 0), (4, 4))
    saved = Layout([regular(half, 4, 0, 0), regular(half2, 4, 1, 0)], [80, 64])
    target = Layout([regular(full, 4, 0, 0)], [128])
    src = synth.materialize(saved, {0: spec}, 1)
    with pytest.raises(oracle.OracleError) as e:
        oracle.reshard(saved, target, src)
    assert e.value.kind == "saved_overlap"


def test_uncovered_target_is_an_error_unless_allowed():
    spec, full = _simple()
    half = Part(0, (8, 4), (0, 0), (4, 4))
    saved = Layout([regular(half, 4, 0, 0)], [64])
    target = Layout([regular(full, 4, 0, 0)], [128])
    src = synth.materialize(saved, {0: spec}, 1)
    with pytest.raises(oracle.OracleError) as e:
        oracle.reshard(saved, target, src)
    assert e.value.kind == "uncovered"
    got = oracle.reshard(saved, target, src, allow_uncovered=True, poison=POISON)
    assert np.array_equal(got[0][:64], src[0].numpy())
    assert np.all(got[0][64:] == POISON)


def test_shape_and_dtype_mismatch_are_errors():
    spec, full = _simple()
    saved = Layout([regular(full, 4, 0, 0)], [128])
    src = synth.materialize(saved, {0: spec}, 1)
    other_shape = Layout([regular(Part(0, (4, 8), (0, 0), (4, 8)), 4, 0, 0)], [128])
    with pytest.raises(oracle.OracleError) as e:
        oracle.reshard(saved, other_shape, src)
    assert e.value.kind == "mismatch"
    other_dtype = Layout([regular(full, 2, 0, 0)], [128])
    with pytest.raises(oracle.OracleError) as e:
        oracle.reshard(saved, other_dtype, src)
    assert e.value.kind == "mismatch"


def test_unused_saved_tensors_are_ignored_and_empty_shards_are_legal():
    spec, full = _simple()
    spec2 = TensorSpec(1, "unused", (3,), torch.float32, ("normal", 0.0, 1.0))
    empty = Part(0, (8, 4), (8, 0), (0, 4))
    saved = Layout([regular(full, 4, 0, 0), regular(Part(1, (3,), (0,), (3,)), 4, 0, 128),
                    regular(empty, 4, 0, 140)], [140])
    target = Layout([regular(full, 4, 0, 0), regular(empty, 4, 0, 128)], [128])
    src = synth.materialize(saved, {0: spec, 1: spec2}, 1)
    got = oracle.reshard(saved, target, src)
    assert np.array_equal(got[0], src[0].numpy()[:128])
