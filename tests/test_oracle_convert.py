"""Pins of the oracle's dtype-converting load (fp32 saved, bf16 asked for; Sec. 2.2: evaluation jobs
load the model only): the narrowing itself against hand-worked values, the library cast and the
defining property of round-to-nearest, then the whole transform against the library-slicing closed
form.  CPU only."""
import os

import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2407_20143_amd import synth
from paper_2407_20143_amd.synth import Case, Layout, Part, TensorSpec, regular

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
POISON = 0xA5


def golden_pairs():
    out = []
    with open(os.path.join(ROOT, "tests", "golden", "bf16_rounding.txt")) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                a, b = line.split("=")
                out.append((int(a, 16), int(b, 16)))
    return out


def torch_cast(bits: np.ndarray) -> np.ndarray:
    t = torch.from_numpy(bits.view(np.float32).copy()).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


def is_nan32(bits):
    return (bits & 0x7FFFFFFF) > 0x7F800000


def is_nan16(bits):
    return (bits & 0x7FFF) > 0x7F80


def bf16_value(bits16: np.ndarray) -> np.ndarray:
    """bfloat16 patterns as float64 (numpy: widen to binary32 by appending 16 zero bits)."""
    return (bits16.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def test_hand_worked_values():
    pairs = golden_pairs()
    assert len(pairs) >= 30
    got = oracle.f32_to_bf16(np.array([a for a, _ in pairs], dtype=np.uint32))
    for (a, want), g in zip(pairs, got):
        assert int(g) == want, f"{a:#010x}: got {int(g):#06x}, want {want:#06x}"


def test_against_the_library_cast_on_every_upper_half():
    hi = np.arange(1 << 16, dtype=np.uint32) << 16
    for lo in (0x0000, 0x0001, 0x7FFF, 0x8000, 0x8001, 0xFFFF):
        bits = hi | np.uint32(lo)
        got, lib = oracle.f32_to_bf16(bits), torch_cast(bits)
        nan = is_nan32(bits)
        assert np.array_equal(got[~nan], lib[~nan]), f"lower half {lo:#06x}"
        assert is_nan16(got[nan]).all() and is_nan16(lib[nan]).all()
        # the reading for NaN: sign and upper payload kept, quiet
        assert np.array_equal(got[nan], ((bits[nan] >> 16) | 0x40).astype(np.uint16))


def test_against_the_library_cast_on_random_bits():
    rng = np.random.default_rng(20143)
    bits = rng.integers(0, 1 << 32, size=2_000_000, dtype=np.uint64).astype(np.uint32)
    got, lib = oracle.f32_to_bf16(bits), torch_cast(bits)
    nan = is_nan32(bits)
    assert np.array_equal(got[~nan], lib[~nan])
    assert is_nan16(got[nan]).all()


def test_result_is_a_nearest_neighbour_and_ties_are_even():
    """The definition, checked without the oracle's arithmetic: no other bfloat16 value is closer."""
    rng = np.random.default_rng(7)
    bits = rng.integers(0, 1 << 32, size=500_000, dtype=np.uint64).astype(np.uint32)
    bits = bits[~is_nan32(bits) & ((bits & 0x7FFFFFFF) < 0x7F7F0000)]   # finite, away from the overflow edge
    got = oracle.f32_to_bf16(bits)
    x = bits.view(np.float32).astype(np.float64)
    y = bf16_value(got)
    mag = got & 0x7FFF
    up = bf16_value(((got & 0x8000) | (mag + 1)).astype(np.uint16))
    down = bf16_value(((got & 0x8000) | np.maximum(mag.astype(np.int32) - 1, 0).astype(np.uint16)).astype(np.uint16))
    err = np.abs(x - y)
    assert (err <= np.abs(x - up)).all() and (err <= np.abs(x - down)).all()
    tie = (err == np.abs(x - up)) | ((err == np.abs(x - down)) & (mag > 0))
    assert (got[tie & (err > 0)] & 1 == 0).all()          # on a tie the even pattern was taken
    assert ((got >> 15) == (bits >> 31)).all()            # the sign is carried over


def test_monotone_over_ordered_inputs():
    rng = np.random.default_rng(11)
    mags = np.sort(rng.integers(0, 0x7F800001, size=300_000, dtype=np.uint64).astype(np.uint32))
    got = oracle.f32_to_bf16(mags).astype(np.int64)
    assert (np.diff(got) >= 0).all()


def check_whole_transform(case: Case):
    assert case.convert == 1
    src = synth.materialize(case.saved, case.tensors, case.seed)
    want = [b.numpy() for b in synth.materialize(case.target, case.tensors, case.seed, poison=POISON)]
    got, written = oracle.reshard(case.saved, case.target, src, poison=POISON, convert=1, want_written=True)
    for i, (g, w) in enumerate(zip(got, want)):
        assert np.array_equal(g, w), f"{case.name}: buffer {i} differs from the library-slicing closed form"
    cover = [m.numpy() for m in synth.coverage_mask(case.target, {f: TensorSpec(f, s.name, s.shape, torch.bfloat16, s.dist)
                                                               for f, s in case.tensors.items()})]
    for i, (w, c) in enumerate(zip(written, cover)):
        assert np.array_equal(w, c), f"{case.name}: buffer {i}: bytes not written exactly once"


def test_whole_transform_model_shaped():
    check_whole_transform(synth.eval_load_case(layers=2, hidden=64, ffn=96, vocab=128))
    check_whole_transform(synth.eval_load_case(layers=2, hidden=72, ffn=104, vocab=160, zero_saved=True))


@pytest.mark.parametrize("modes", [("grid", "grid"), ("flat", "grid"), ("grid", "flat"), ("flat", "flat")])
@pytest.mark.parametrize("seed", range(4))
def test_whole_transform_random_layouts(seed, modes):
    case = synth.random_case(900 + seed, n_tensors=4, max_elems=2000, saved_mode=modes[0], target_mode=modes[1],
                             dtype=torch.float32, p_strided=0.3, narrow_target=True)
    # arbitrary bit patterns, except that NaN payloads differ between casts of the library: NaN -> infinity
    specs = {f: TensorSpec(f, s.name, s.shape, s.dtype, ("bits_no_nan",)) for f, s in case.tensors.items()}
    check_whole_transform(Case(case.name, case.seed, specs, case.saved, case.target, convert=1))


def test_nan_goes_through_the_whole_transform_as_the_golden_file_says():
    pairs = [(a, b) for a, b in golden_pairs() if (a & 0x7FFFFFFF) > 0x7F800000]
    assert len(pairs) >= 4
    n = len(pairs)
    part = Part(0, (n,), (0,), (n,))
    src = np.array([a for a, _ in pairs], dtype=np.uint32).view(np.uint8)
    saved, target = Layout([regular(part, 4, 0, 0)], [4 * n]), Layout([regular(part, 2, 0, 0)], [2 * n])
    got = oracle.reshard(saved, target, [src], convert=1)
    assert got[0].view(np.uint16).tolist() == [b for _, b in pairs]


def test_element_sizes_must_agree_without_the_flag_and_only_4_to_2_converts():
    part = Part(0, (8,), (0,), (8,))
    src = [np.zeros(64, dtype=np.uint8)]
    with pytest.raises(oracle.OracleError) as e:
        oracle.reshard(Layout([regular(part, 4, 0, 0)], [32]), Layout([regular(part, 2, 0, 0)], [16]), src)
    assert e.value.kind == "mismatch"
    with pytest.raises(oracle.OracleError) as e:
        oracle.reshard(Layout([regular(part, 8, 0, 0)], [64]), Layout([regular(part, 2, 0, 0)], [16]), src, convert=1)
    assert e.value.kind == "mismatch"
    with pytest.raises(oracle.OracleError) as e:
        oracle.reshard(Layout([regular(part, 2, 0, 0)], [16]), Layout([regular(part, 4, 0, 0)], [32]), src, convert=1)
    assert e.value.kind == "mismatch"
    # tensors whose element sizes agree are moved as they are, flag or not
    vals = np.arange(32, dtype=np.uint8)
    got = oracle.reshard(Layout([regular(part, 4, 0, 0)], [32]), Layout([regular(part, 4, 0, 0)], [32]), [vals], convert=1)
    assert np.array_equal(got[0], vals)
