"""GPU parity: the HIP path (through the C-ABI) against the CPU oracle, byte for byte, on the
same seeded inputs.  Sizes here are ones the oracle finishes in seconds while still spanning
several tiles and ragged tails; full-size configurations live in test_gpu_full_size.py."""
import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2407_20143_amd import binding, synth
from paper_2407_20143_amd.synth import Case, Layout, Part, Shard, TensorSpec, regular

pytestmark = pytest.mark.gpu

POISON = 0xA5


@pytest.fixture(autouse=True)
def _default_config():
    binding.configure(**binding.DEFAULT_CONFIG)
    yield
    binding.configure(**binding.DEFAULT_CONFIG)


def gpu_reshard(case: Case, src_cpu, flags=0, dst_init=None):
    if case.convert:
        flags |= binding.BCP_CONVERT_F32_TO_BF16
    sm, tm = binding.layout_to_meta(case.saved), binding.layout_to_meta(case.target)
    p = binding.plan(sm, tm, flags=flags)
    dsrc = [b.cuda() for b in src_cpu]
    if dst_init is None:
        ddst = [torch.full((n,), POISON, dtype=torch.uint8, device="cuda") for n in case.target.buf_bytes]
    else:
        ddst = [torch.as_tensor(b).cuda() for b in dst_init]
    binding.reshard(p, dsrc, ddst)
    torch.cuda.synchronize()
    return [t.cpu().numpy() for t in ddst], p


def assert_same(got, want, what):
    assert len(got) == len(want)
    for i, (g, w) in enumerate(zip(got, want)):
        if not np.array_equal(g, w):
            bad = np.flatnonzero(g != w)
            raise AssertionError(f"{what}: buffer {i}: {bad.size} of {g.size} bytes differ, first at {bad[0]}")


def check_case(case: Case, also_closed_form=True):
    src = synth.materialize(case.saved, case.tensors, case.seed)
    want = oracle.reshard(case.saved, case.target, src, poison=POISON, convert=case.convert)
    got, p = gpu_reshard(case, src)
    assert_same(got, want, case.name + " vs oracle")
    if also_closed_form:
        exp = [b.numpy() for b in synth.materialize(case.target, case.tensors, case.seed, poison=POISON)]
        assert_same(got, exp, case.name + " vs library slicing")
    st = p.stats()
    assert st["payload_bytes"] == case.target.payload_bytes()
    # bytes read: every target element at its SAVED element size
    assert st["src_bytes"] == sum(sh.numel * case.tensors[sh.parts[0].fqn].dtype.itemsize for sh in case.target.shards if sh.parts)
    p.destroy()
    return st


# ---- dtype-converting load: fp32 saved, bf16 asked for (Sec. 2.2, evaluation jobs) -------------------
@pytest.mark.parametrize("modes", [("grid", "grid"), ("grid", "flat"), ("flat", "grid"), ("flat", "flat")])
@pytest.mark.parametrize("seed", range(6))
def test_convert_random_layouts(seed, modes):
    """Arbitrary fp32 bit patterns (NaN payloads, infinities, subnormals, ties), every alignment class,
    strided shards on either side: bit-exact against the oracle's IEEE narrowing."""
    case = synth.random_case(300 + seed, n_tensors=6, max_elems=40000, saved_mode=modes[0], target_mode=modes[1],
                             dtype=torch.float32, p_strided=0.3 if "grid" in modes else 0.0, narrow_target=True)
    check_case(case, also_closed_form=False)   # (the library cast differs on NaN payloads; the oracle is the reference)


def test_convert_every_upper_half_and_the_rounding_edges():
    """One tensor holding every upper half with the lower halves around the rounding decision."""
    lows = np.array([0x0000, 0x0001, 0x7FFF, 0x8000, 0x8001, 0xFFFF], dtype=np.uint32)
    bits = ((np.arange(1 << 16, dtype=np.uint32) << 16)[None, :] | lows[:, None]).reshape(-1)
    n = bits.size
    part = Part(0, (n,), (0,), (n,))
    saved, target = Layout([regular(part, 4, 0, 0)], [4 * n]), Layout([regular(part, 2, 0, 6)], [2 * n + 6])
    src = [torch.from_numpy(bits.view(np.uint8).copy())]
    want = oracle.reshard(saved, target, src, poison=POISON, convert=1)
    case = Case("edges", 0, {0: TensorSpec(0, "t", (n,), torch.float32, ("bits",))}, saved, target, convert=1)
    got, p = gpu_reshard(case, src)
    assert_same(got, want, "rounding edges")
    p.destroy()


@pytest.mark.parametrize("n1", [504, 512, 520, 1032, 2752])
def test_convert_rows_around_the_64_group_units(n1):
    """Big converting tiles take whole units of 64 groups (512 elements) a wave at a time and the rest of every
    row group by group: rows just below, at and above one unit, and a row of five units and 24 groups; one
    long run with the destination 6 bytes off a 16-byte boundary besides."""
    rows, n = 72, n1 + 1024
    spec = TensorSpec(0, "w", (rows, n), torch.float32, ("bits",))
    saved = Layout([regular(Part(0, (rows, n), (0, 0), (rows, n)), 4, 0, 0)], [rows * n * 4])
    left, right = Part(0, (rows, n), (0, 0), (rows, n1)), Part(0, (rows, n), (0, n1), (rows, 1024))
    target = Layout([regular(left, 2, 0, 0), regular(right, 2, 1, 0)], [rows * n1 * 2, rows * 1024 * 2])
    check_case(Case("convert_rows", 40 + n1, {0: spec}, saved, target, convert=1), also_closed_form=False)
    flat = rows * n
    spec = TensorSpec(0, "f", (flat,), torch.float32, ("bits",))
    saved = Layout([regular(Part(0, (flat,), (0,), (flat,)), 4, 0, 0)], [flat * 4])
    cut = 8 * n1 + 3
    target = Layout([regular(Part(0, (flat,), (0,), (cut,)), 2, 0, 6), regular(Part(0, (flat,), (cut,), (flat - cut,)), 2, 1, 0)],
                    [cut * 2 + 6, (flat - cut) * 2])
    check_case(Case("convert_flat", 41 + n1, {0: spec}, saved, target, convert=1), also_closed_form=False)


def test_convert_model_shaped_scaled():
    for case in (synth.eval_load_case(layers=2, hidden=256, ffn=688, vocab=1000),
                 synth.eval_load_case(layers=2, hidden=264, ffn=696, vocab=1000, zero_saved=True)):
        st = check_case(case)
        assert st["n_transposed"] == 0
    # mixed: a plan with the flag where only some tensors differ in element size
    c = synth.eval_load_case(layers=1, hidden=128, ffn=344, vocab=500)
    keep = {f for f in c.tensors if f % 2 == 0}   # these stay fp32 on the target side
    wide = synth.megatron_layout(synth.llama_tensors(1, 128, 344, 500), [synth.STATE_FP32_MASTER], 1, 2, 4, replicate_norms=True)
    shards = [w if w.parts[0].fqn in keep else n for w, n in zip(wide.shards, c.target.shards)]
    # re-pack: the two layouts' offsets do not fit together
    target = synth.packed_layout(shards, [sh.buf for sh in shards], len(wide.buf_bytes))
    check_case(Case("eval_load_mixed", c.seed, c.tensors, c.saved, target, convert=1))


def test_convert_needs_the_flag():
    c = synth.eval_load_case(layers=1, hidden=64, ffn=96, vocab=128)
    with pytest.raises(binding.BcpError) as e:
        binding.plan(binding.layout_to_meta(c.saved), binding.layout_to_meta(c.target))
    assert e.value.name == "BCP_ERR_DTYPE_MISMATCH"


def test_device_and_host_verdicts_agree():
    """bcp_plan and bcp_validate_meta give the same status for the same metadata and flags."""
    from tests import meta_cases
    for name, sm, tm, flags, want in meta_cases.cases():
        dev, dtext = meta_cases.device_verdict(sm, tm, flags)
        host, htext = meta_cases.host_verdict(sm, tm, flags)
        assert dev == host == want, f"{name}: device {dev} ({dtext}), host {host} ({htext}), expected {want}"
        if dev != "BCP_OK" and "record" in htext:
            assert dtext.split(":")[1] == htext.split(":")[1], f"{name}: device names '{dtext}', host '{htext}'"


def test_checked_reshard_refuses_short_buffers():
    case = synth.cfg1(128, 96)
    src = synth.materialize(case.saved, case.tensors, case.seed)
    p = binding.plan(binding.layout_to_meta(case.saved), binding.layout_to_meta(case.target))
    se, de = p.buffer_extents()
    assert list(se) == case.saved.buf_bytes and list(de) == case.target.buf_bytes
    dsrc = [b.cuda() for b in src]
    ddst = [torch.full((n,), POISON, dtype=torch.uint8, device="cuda") for n in case.target.buf_bytes]
    for side, i in (("src", 1), ("dst", 2)):
        bufs = {"src": list(dsrc), "dst": list(ddst)}
        bufs[side][i] = bufs[side][i][:-1]
        with pytest.raises(binding.BcpError) as e:
            binding.reshard(p, bufs["src"], bufs["dst"])
        assert e.value.name == "BCP_ERR_OUT_OF_BOUNDS" and f"[{i}]" in str(e.value)
    torch.cuda.synchronize()
    assert all(bool((d == POISON).all()) for d in ddst)   # nothing was launched
    binding.reshard(p, dsrc, ddst)
    torch.cuda.synchronize()
    assert_same([d.cpu().numpy() for d in ddst], oracle.reshard(case.saved, case.target, src, poison=POISON), "checked")
    p.destroy()


def test_skip_overlap_check_flag():
    """BCP_SKIP_OVERLAP_CHECK: same plan and bytes on a valid layout; an overlap is then the caller's error
    and shows up, if at all, as a target covered more than once."""
    case = synth.cfg5(layers=1, hidden=128, experts=8, ffn=44, n_small=500)
    src = synth.materialize(case.saved, case.tensors, case.seed)
    want = oracle.reshard(case.saved, case.target, src, poison=POISON)
    got, p = gpu_reshard(case, src, flags=binding.BCP_SKIP_OVERLAP_CHECK)
    assert_same(got, want, "skip overlap check")
    got2, p2 = gpu_reshard(case, src)
    assert np.array_equal(p.regions(), p2.regions())
    p.destroy()
    p2.destroy()


@pytest.mark.parametrize("modes", [("grid", "grid"), ("grid", "flat"), ("flat", "grid"), ("flat", "flat")])
@pytest.mark.parametrize("seed", range(8))
def test_random_layouts(seed, modes):
    check_case(synth.random_case(100 + seed, n_tensors=8, max_elems=20000, saved_mode=modes[0], target_mode=modes[1]))


@pytest.mark.parametrize("side", ["read", "write"])
def test_column_blocks_in_one_buffer(side):
    """Row copies with short runs at a long pitch on one side only (the access pattern of the
    transposed case without the transposition), all blocks packed into one buffer."""
    check_case(synth.column_blocks_case(200, 384, 32, side))
    check_case(synth.column_blocks_case(130, 96, 3, side, dtype=torch.bfloat16))


def test_random_soak():
    """120 more random cases in one test: every mix of grid / flat sides, ranks up to 6, strided
    shards, all packing granules, under the default launch shape and a small-tile one."""
    modes = ("grid", "flat")
    for i in range(120):
        seed = 9000 + i
        if i == 60:
            binding.configure(tile_bytes=4096, persistent=1, wg_per_cu=2, threads=256)
        sm, tm = modes[i & 1], modes[(i >> 1) & 1]
        strided = 0.5 if (sm, tm) == ("grid", "grid") and i % 3 == 0 else 0.0
        check_case(synth.random_case(seed, n_tensors=4 + i % 5, max_elems=2000 + 500 * (i % 7), saved_mode=sm,
                                     target_mode=tm, max_rank=2 + i % 5, p_strided=strided))


@pytest.mark.parametrize("seed", range(8))
def test_random_strided(seed):
    check_case(synth.random_case(200 + seed, n_tensors=6, max_elems=30000, p_strided=0.6, granules=(4, 8, 16)))


@pytest.mark.parametrize("dtype", [torch.uint8, torch.bfloat16, torch.float32, torch.float64])
@pytest.mark.parametrize("seed", range(3))
def test_random_flat_single_dtype_odd_offsets(seed, dtype):
    """ZeRO-like slices at byte offsets of every alignment class (granule 1 or 2 for small types)."""
    check_case(synth.random_case(300 + seed, n_tensors=6, max_elems=50000, saved_mode="flat", target_mode="flat",
                                 granules=(1, 2), dtype=dtype))


def test_rank_8_tensors():
    """The dimension limit: rank-8 tensors under grid, flat (decomposition into up to 15 boxes) and
    strided layouts."""
    for seed, modes, ps in ((700, ("grid", "grid"), 0.0), (701, ("flat", "grid"), 0.0), (705, ("grid", "flat"), 0.0),
                            (703, ("grid", "grid"), 0.7), (705, ("flat", "flat"), 0.0)):
        case = synth.random_case(seed, n_tensors=4, max_elems=40000, saved_mode=modes[0], target_mode=modes[1],
                                 max_rank=8, p_strided=ps, granules=(16,) if ps else (1, 4, 16))
        assert max(len(s.shape) for s in case.tensors.values()) >= 6
        check_case(case)


@pytest.mark.parametrize("dtype", [torch.complex128, torch.float64, torch.uint8])
def test_strided_every_itemsize(dtype):
    """LDS-staged transposes with 16-, 8- and 1-byte elements (32x32 and 64x64 tiles)."""
    for seed in range(3):
        n = 96 + 37 * seed
        spec = TensorSpec(0, "w", (n, 2 * n + 5), dtype, ("bits",))
        e = dtype.itemsize
        saved = Layout([regular(Part(0, spec.shape, (0, 0), spec.shape), e, 0, 0)], [spec.shape[0] * spec.shape[1] * e])
        half = spec.shape[1] // 2
        t = [regular(Part(0, spec.shape, (0, 0), (n, half)), e, 0, 0, (1, n)),
             regular(Part(0, spec.shape, (0, half), (n, spec.shape[1] - half)), e, 1, 0, (1, n))]
        target = Layout(t, [n * half * e, n * (spec.shape[1] - half) * e])
        st = check_case(Case("transpose", seed, {0: spec}, saved, target))
        assert st["n_transposed"] == 2


@pytest.mark.parametrize("dtype", [torch.uint8, torch.bfloat16, torch.float32, torch.float64, torch.complex128])
@pytest.mark.parametrize("n,m", [(512, 768), (528, 784), (520, 776), (515, 771)])
def test_transposed_full_and_ragged_tiles(dtype, n, m):
    """Column-major targets with everything 16-byte aligned: whole tiles (the per-wave path of 4-byte and
    wider elements, the workgroup-wide vector path of the narrower ones), ragged tiles at the edges
    (multiples of 16 and of 8 elements), and extents that leave only the element-by-element path."""
    st = check_case(synth.transpose_case(n - n % 2, m - m % 2, dtype, shards=2))  # two shards: even extents
    assert st["n_transposed"] == 4


def test_metadata_already_on_the_device():
    case = synth.cfg4(layers=2, hidden=136, ffn=344, vocab=1000, dp_s=16, dp_t=12, n_states=1)
    sm, tm = binding.layout_to_meta(case.saved), binding.layout_to_meta(case.target)
    a = binding.plan(sm, tm)
    ds, ns = binding.meta_to_device(sm)
    dt, nt = binding.meta_to_device(tm)
    b = binding.plan_from_device_meta(ds, ns, dt, nt)
    assert a.regions().tobytes() == b.regions().tobytes()
    # the same records from pageable host memory, and from host arrays that are not 16-byte aligned: other
    # ways into the planner (copies instead of the validation kernel reading the caller's arrays), same plan
    pageable = binding.plan(np.array(sm), np.array(tm))
    raw_s, raw_t = np.zeros(sm.nbytes + 16, np.uint8), np.zeros(tm.nbytes + 16, np.uint8)
    off_s, off_t = (8 - raw_s.ctypes.data % 16) % 16, (8 - raw_t.ctypes.data % 16) % 16  # addresses 8 modulo 16
    ms = raw_s[off_s:off_s + sm.nbytes].view(sm.dtype)
    mt = raw_t[off_t:off_t + tm.nbytes].view(tm.dtype)
    ms[:], mt[:] = sm, tm
    assert ms.ctypes.data % 16 == 8 and mt.ctypes.data % 16 == 8
    shifted = binding.plan(ms, mt)
    for other in (pageable, shifted):
        assert a.regions().tobytes() == other.regions().tobytes()
        assert a.stats()["n_batches"] == other.stats()["n_batches"]
        other.destroy()
    src = synth.materialize(case.saved, case.tensors, case.seed)
    want = oracle.reshard(case.saved, case.target, src, poison=POISON)
    dsrc = [x.cuda() for x in src]
    ddst = [torch.full((n,), POISON, dtype=torch.uint8, device="cuda") for n in case.target.buf_bytes]
    binding.reshard(b, dsrc, ddst)
    torch.cuda.synchronize()
    assert_same([t.cpu().numpy() for t in ddst], want, "device metadata")
    a.destroy()
    b.destroy()


def test_plans_are_reproducible():
    case = synth.cfg5(layers=1, hidden=128, experts=8, ffn=44, n_small=2000)
    sm, tm = binding.layout_to_meta(case.saved), binding.layout_to_meta(case.target)
    a, b = binding.plan(sm, tm), binding.plan(sm, tm)
    ra, rb = a.regions(), b.regions()
    assert len(ra) > 2000 and ra.tobytes() == rb.tobytes()
    assert a.stats()["n_batches"] == b.stats()["n_batches"]
    a.destroy()
    b.destroy()


def test_cfg1_small_and_strided():
    st = check_case(synth.cfg1(256, 192))
    assert st["n_pairs"] == 8 and st["n_regions"] == 8
    st = check_case(synth.cfg1(256, 192, strided_target=True))
    assert st["n_transposed"] == 8


def test_cfg1_full_size():
    st = check_case(synth.cfg1())
    assert st["n_pairs"] == 8 and st["n_regions"] == 8 and st["payload_bytes"] == 4 << 20


def test_cfg1_full_size_strided_target():
    st = check_case(synth.cfg1(strided_target=True))
    assert st["n_transposed"] == 8


def test_cfg2_scaled():
    st = check_case(synth.cfg2(layers=4, hidden=256, ffn=688, vocab=4000))
    # per split tensor 4 saved x 2 target boxes -> 8 pairs, 4 regions; replicated: 1 x 2
    n_split, n_rep = 2 + 4 * 7, 1 + 4 * 2
    assert st["n_pairs"] == 8 * n_split + 2 * n_rep
    assert st["n_regions"] == 4 * n_split + 2 * n_rep


def test_cfg3_scaled_and_rank_share():
    check_case(synth.cfg3(layers=4, hidden=256, ffn=688, vocab=4000))
    check_case(synth.cfg3(layers=4, hidden=256, ffn=688, vocab=4000, rank_share=True))


def test_cfg4_scaled_ragged():
    # 16 -> 12 slices with a ragged tail, TP1 -> TP2; sizes chosen so slices cross tensor
    # boundaries at element offsets of every residue modulo 4 elements
    case = synth.cfg4(layers=3, hidden=136, ffn=344, vocab=1000, dp_s=16, dp_t=12)
    ns = sum(s.numel for s in case.saved.shards if s.group == 0)
    nt = sum(s.numel for s in case.target.shards if s.group == 0)
    assert ns % 16 != 0 and nt % 12 != 0
    check_case(case)


def test_cfg5_scaled():
    check_case(synth.cfg5(layers=2, hidden=256, experts=16, ffn=88, n_small=3000))


def test_table3_shapes_scaled():
    """The paper's Table 3 reshards at reduced width: FSDP ZeRO-2 32 -> 64 and 128 -> 64 ranks
    (per-block flat units), Megatron distributed optimizer DP 75 <-> 150 inside one TP/PP group."""
    check_case(synth.table3_vdit(32, 64, layers=3, hidden=104, text_dim=200))
    check_case(synth.table3_vdit(128, 64, layers=3, hidden=104, text_dim=200))
    check_case(synth.table3_tgpt_group(75, 150, layers=2, hidden=256, vocab=2048))
    check_case(synth.table3_tgpt_group(150, 75, layers=2, hidden=256, vocab=2048, first_stage=False))


def test_fused_gqa_qkv_to_separate_tensors():
    """Fused, group-interleaved QKV blobs (Megatron style) loaded as separate q / k / v under another TP."""
    st = check_case(synth.fused_qkv_case(layers=3, hidden=256, n_heads=16, n_kv=4, tp_s=4, tp_t=2))
    assert st["n_regions"] == 3 * 3 * 4  # per layer: 4 groups x (q, k, v), each inside one target shard
    check_case(synth.fused_qkv_case(layers=2, hidden=192, n_heads=12, n_kv=6, tp_s=2, tp_t=3, dtype=torch.float32))
    check_case(synth.fused_qkv_case(layers=2, hidden=128, n_heads=8, n_kv=8, tp_s=8, tp_t=1))


@pytest.mark.parametrize("n_bufs", [200, 700])
def test_many_buffers(n_bufs):
    """More buffers than fit the kernel arguments (pointer table in device memory), and more than
    the kernel stages in LDS."""
    specs, saved, target = synth.small_tensor_case(1500, 77, n_bufs=n_bufs, max_shards=6, hi=2000)
    check_case(Case(f"many{n_bufs}", 77, specs, saved, target))


# ---- chunked arrival: source-ordered plans -----------------------------------------------------------
def _arrival_cases():
    return [synth.cfg2(layers=2, hidden=512, ffn=1376, vocab=3000),
            synth.cfg4(layers=2, hidden=136, ffn=344, vocab=1000, dp_s=16, dp_t=12, n_states=1),
            synth.random_case(600, n_tensors=10, max_elems=60000, saved_mode="grid", target_mode="flat", p_strided=0.3,
                              granules=(4, 16)),
            synth.cfg5(layers=1, hidden=128, experts=8, ffn=44, n_small=800)]


@pytest.mark.parametrize("idx", range(4))
def test_source_ordered_plan_runs_as_chunks_arrive(idx):
    """Every chunk call may only touch source bytes below the chunk's end: the device blobs hold
    garbage until 'their' chunk lands, and the final result must still be the oracle's."""
    case = _arrival_cases()[idx]
    src = synth.materialize(case.saved, case.tensors, case.seed)
    want = oracle.reshard(case.saved, case.target, src, poison=POISON)
    sm, tm = binding.layout_to_meta(case.saved), binding.layout_to_meta(case.target)
    p = binding.plan(sm, tm, flags=binding.BCP_ORDER_BY_SOURCE)
    # (a) an ordered plan is still a complete plan
    dsrc = [b.cuda() for b in src]
    ddst = [torch.full((n,), POISON, dtype=torch.uint8, device="cuda") for n in case.target.buf_bytes]
    binding.reshard(p, dsrc, ddst)
    torch.cuda.synchronize()
    assert_same([t.cpu().numpy() for t in ddst], want, case.name + " ordered plan, one launch")
    # (b) chunk by chunk, blobs in a shuffled order, odd chunk sizes
    rng = np.random.default_rng(idx)
    dsrc = [torch.full((b.numel(),), 0x3C, dtype=torch.uint8, device="cuda") for b in src]
    ddst = [torch.full((n,), POISON, dtype=torch.uint8, device="cuda") for n in case.target.buf_bytes]
    for b in rng.permutation(len(src)):
        n, off = src[b].numel(), 0
        while off < n:
            step = int(rng.integers(1, max(2, n // 3)))
            end = min(n, off + step)
            dsrc[b][off:end] = src[b][off:end].cuda()
            binding.reshard_arrived(p, dsrc, ddst, int(b), off, end)
            off = end
    torch.cuda.synchronize()
    assert_same([t.cpu().numpy() for t in ddst], want, case.name + " chunked arrival")
    p.destroy()


@pytest.mark.parametrize("size,gaps,jitter", [(70_000, (4, 12), 900), (200_000, (0, 4), 0), (131_072, (1, 0), 5000)])
def test_packed_regions_at_shifting_offsets(size, gaps, jitter):
    """Byte tensors of one to three tiles packed with a few bytes between them, so that the alignment of the two
    sides changes from region to region: first tiles cut short to a 256-byte boundary of the destination, partial
    last tiles, the shifted-load path at every shift."""
    check_case(synth.regions_case(size, gaps[0], gaps[1], jitter, total=6_000_000))


@pytest.mark.parametrize("by_source", [False, True])
def test_small_tensors_between_big_ones_share_batches(by_source):
    """Tensors of 200 000 bytes alternating with tensors of 40 to 1200 bytes, on both sides in one buffer at odd
    offsets.  In plan order the small tiles are batched among themselves across the big tiles between them
    (fewer batches than one per small tensor); ordered by source every batch stays a run of consecutive tiles.
    Bytes against the oracle both ways, and chunk by chunk for the ordered plan."""
    rng = np.random.default_rng(11)
    specs, sv, tg, so, to = {}, [], [], 3, 5
    for f in range(120):
        n = 200_000 if f % 2 == 0 else int(rng.integers(40, 1200))
        specs[f] = TensorSpec(f, f"t{f}", (n,), torch.uint8, ("bits",))
        part = Part(f, (n,), (0,), (n,))
        sv.append(regular(part, 1, 0, so))
        tg.append(regular(part, 1, 0, to))
        so += n + int(rng.integers(0, 9))
        to += n + int(rng.integers(0, 9))
    case = Case("between", 12, specs, Layout(sv, [so]), Layout(tg, [to]))
    src = synth.materialize(case.saved, specs, case.seed)
    want = oracle.reshard(case.saved, case.target, src, poison=POISON)
    p = binding.plan(binding.layout_to_meta(case.saved), binding.layout_to_meta(case.target),
                     flags=binding.BCP_ORDER_BY_SOURCE if by_source else 0)
    st = p.stats()
    assert st["n_tiles"] >= 60 * 4 + 60
    if not by_source:
        assert st["n_batches"] < st["n_tiles"] - 50, st   # the 60 small tensors do not take a batch each
    dsrc = [b.cuda() for b in src]
    ddst = [torch.full((n,), POISON, dtype=torch.uint8, device="cuda") for n in case.target.buf_bytes]
    binding.reshard(p, dsrc, ddst)
    torch.cuda.synchronize()
    assert_same([t.cpu().numpy() for t in ddst], want, "small between big, one launch")
    if by_source:
        dsrc = [torch.full((b.numel(),), 0x3C, dtype=torch.uint8, device="cuda") for b in src]
        ddst = [torch.full((n,), POISON, dtype=torch.uint8, device="cuda") for n in case.target.buf_bytes]
        n, off = src[0].numel(), 0
        while off < n:
            end = min(n, off + int(rng.integers(1, 700_000)))
            dsrc[0][off:end] = src[0][off:end].cuda()
            binding.reshard_arrived(p, dsrc, ddst, 0, off, end)
            off = end
        torch.cuda.synchronize()
        assert_same([t.cpu().numpy() for t in ddst], want, "small between big, chunked arrival")
    p.destroy()


def test_source_ordered_plan_with_a_spare_segment_at_the_end_of_a_blob():
    """A long run with a misaligned destination is cut where the DESTINATION offset is a multiple of 256, which
    reserves a possibly empty last segment per row; here that empty segment sits at the very end of a blob,
    followed only by a tiny tensor.  Its key must still lie inside the blob, or the batch it shares with the
    tiny tensor would never run under chunked arrival."""
    n_a, n_b = 2 * 65536 - 100, 50
    specs = {0: TensorSpec(0, "a", (n_a,), torch.uint8, ("bits",)), 1: TensorSpec(1, "b", (n_b,), torch.uint8, ("bits",))}
    pa, pb = Part(0, (n_a,), (0,), (n_a,)), Part(1, (n_b,), (0,), (n_b,))
    saved = Layout([regular(pa, 1, 0, 0), regular(pb, 1, 0, n_a)], [n_a + n_b])
    target = Layout([regular(pa, 1, 0, 7), regular(pb, 1, 0, n_a + 300)], [n_a + 400])
    case = Case("spare", 5, specs, saved, target)
    src = synth.materialize(saved, specs, 5)
    want = oracle.reshard(saved, target, src, poison=POISON)
    p = binding.plan(binding.layout_to_meta(saved), binding.layout_to_meta(target), flags=binding.BCP_ORDER_BY_SOURCE)
    assert p.stats()["n_tiles"] == 4   # three segments of the long run (the last one empty) and the tiny tensor
    host = [b.pin_memory() for b in src]
    for chunk in (40000, 1 << 20):
        dsrc = [torch.full((b.numel(),), 0x3C, dtype=torch.uint8, device="cuda") for b in src]
        ddst = [torch.full((n,), POISON, dtype=torch.uint8, device="cuda") for n in target.buf_bytes]
        binding.reshard_from_host(p, host, dsrc, ddst, chunk, torch.cuda.Stream())
        torch.cuda.synchronize()
        assert_same([d.cpu().numpy() for d in ddst], want, f"spare segment, chunks of {chunk}")
    # a host blob shorter than what the plan reads is refused (its last regions would never run)
    with pytest.raises(binding.BcpError) as e:
        binding.reshard_from_host(p, [host[0][:-1]], dsrc, ddst, 40000, torch.cuda.Stream())
    assert e.value.name == "BCP_ERR_OUT_OF_BOUNDS"
    torch.cuda.synchronize()
    p.destroy()


def test_reshard_from_pinned_host_blobs():
    case = synth.cfg3(layers=2, hidden=256, ffn=688, vocab=2000)
    src = synth.materialize(case.saved, case.tensors, case.seed)
    want = oracle.reshard(case.saved, case.target, src, poison=POISON)
    p = binding.plan(binding.layout_to_meta(case.saved), binding.layout_to_meta(case.target),
                     flags=binding.BCP_ORDER_BY_SOURCE)
    host = [b.pin_memory() for b in src]
    copy_stream = torch.cuda.Stream()
    for chunk in (1 << 12, 100_000, 1 << 30):
        dsrc = [torch.full((b.numel(),), 0x3C, dtype=torch.uint8, device="cuda") for b in src]
        ddst = [torch.full((n,), POISON, dtype=torch.uint8, device="cuda") for n in case.target.buf_bytes]
        torch.cuda.synchronize()
        binding.reshard_from_host(p, host, dsrc, ddst, chunk, copy_stream)
        torch.cuda.synchronize()
        assert_same([t.cpu().numpy() for t in ddst], want, f"from host, chunk {chunk}")
        assert all(torch.equal(d.cpu(), s) for d, s in zip(dsrc, src))
    # a plan without the ordering flag refuses ranged execution
    q = binding.plan(binding.layout_to_meta(case.saved), binding.layout_to_meta(case.target))
    with pytest.raises(binding.BcpError):
        binding.reshard_arrived(q, dsrc, ddst, 0, 0, 16)
    q.destroy()
    p.destroy()


def test_round_trip_on_gpu():
    case = synth.random_case(400, n_tensors=8, max_elems=20000, saved_mode="flat", target_mode="grid")
    src = synth.materialize(case.saved, case.tensors, case.seed, poison=POISON)
    mid, p1 = gpu_reshard(case, src)
    back_case = Case("back", case.seed, case.tensors, case.target, case.saved)
    back, p2 = gpu_reshard(back_case, [torch.from_numpy(m) for m in mid])
    assert_same(back, [b.numpy() for b in src], "A->B->A")
    p1.destroy()
    p2.destroy()


@pytest.mark.parametrize("tile_bytes,persistent,wg,threads", [(4096, 0, 8, 256), (16384, 1, 2, 512), (65536, 1, 8, 256),
                                                              (65536, 0, 1, 1024), (1 << 20, 0, 8, 512),
                                                              (1 << 20, 1, 16, 1024)])
def test_launch_configurations(tile_bytes, persistent, wg, threads):
    binding.configure(tile_bytes=tile_bytes, persistent=persistent, wg_per_cu=wg, threads=threads)
    check_case(synth.cfg2(layers=2, hidden=512, ffn=1376, vocab=3000))
    check_case(synth.random_case(500, n_tensors=8, max_elems=40000, saved_mode="flat", target_mode="grid", p_strided=0.3,
                                 granules=(4, 16)))


@pytest.mark.parametrize("tile_bytes,threads", [(1 << 20, 256), (4 << 20, 1024), (65536, 512), (4096, 1024)])
def test_small_tile_batches_longer_than_a_workgroup(tile_bytes, threads):
    """Thousands of tiny tiles per batch: the batch is taken in slices of one tile per thread, and a
    tile's threads may fall into two rounds of the workgroup."""
    binding.configure(tile_bytes=tile_bytes, persistent=1, wg_per_cu=1, threads=threads)
    specs, saved, target = synth.small_tensor_case(3000, seed=77, n_bufs=5, max_shards=12, lo=1, hi=600)
    case = Case("small_batches", 77, specs, saved, target)
    st = check_case(case)
    assert st["n_tiles"] > 4 * st["n_batches"]
    if tile_bytes >= 1 << 20:
        assert st["n_tiles"] / st["n_batches"] > threads  # slices really happen
    # the same through byte-granular packing (1- and 2-byte aligned runs)
    specs, saved, target = synth.small_tensor_case(800, seed=78, n_bufs=3, max_shards=8, lo=1, hi=300,
                                                   dtype=torch.uint8, granule=1)
    check_case(Case("small_batches_u8", 78, specs, saved, target))


def test_small_tiles_every_row_length_and_alignment():
    """Rows of 1 .. 40 bytes (items of 1, 2, 4, 8 and 16 bytes, the last one of a row moved back to end with
    it) at every source and destination address modulo 16, as single runs and as three rows with padding
    between them on either side; the gaps between the tensors keep their poison, so an item that reached
    beyond its row on the destination side shows."""
    spec, sv, tg = {}, [], []
    so = to = 0
    f = 0
    for rows in (1, 3):
        for L in (list(range(1, 41)) if rows == 1 else [1, 2, 3, 5, 7, 8, 12, 13, 16, 17, 31, 33]):
            for a in range(16):
                for b in range(16):
                    shape = (rows, L)
                    spec[f] = TensorSpec(f, f"t{f}", shape, torch.uint8, ("bits",))
                    part = Part(f, shape, (0, 0), shape)
                    so = (so + 15) // 16 * 16 + a
                    to = (to + 15) // 16 * 16 + b
                    ps, pt = (L + 3, L + 6) if rows > 1 else (L, L)
                    sv.append(regular(part, 1, 0, so, (ps, 1) if rows > 1 else None))
                    tg.append(regular(part, 1, 0, to, (pt, 1) if rows > 1 else None))
                    so += rows * ps + 5
                    to += rows * pt + 5
                    f += 1
    case = Case("rows_x_alignments", 13, spec, Layout(sv, [so]), Layout(tg, [to]))
    st = check_case(case)
    assert st["n_regions"] == f


def test_plan_destroyed_right_after_its_launch():
    """Destroying a plan while its copy is still queued is legal: its device blocks are recycled by the
    next plan (same sizes here, so it does take them), ordered behind the copy that still reads them."""
    binding.release_workspace()
    case = synth.cfg2(layers=4, hidden=512, ffn=1376, vocab=3000)
    src = synth.materialize(case.saved, case.tensors, case.seed)
    want = oracle.reshard(case.saved, case.target, src, poison=POISON)
    sm, tm = binding.layout_to_meta(case.saved), binding.layout_to_meta(case.target)
    dsrc = [b.cuda() for b in src]
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    outs = []
    for rnd in range(6):
        st = s1 if rnd % 2 == 0 else s2
        ddst = [torch.full((n,), POISON, dtype=torch.uint8, device="cuda") for n in case.target.buf_bytes]
        torch.cuda.synchronize()
        p = binding.plan(sm, tm, stream=st)
        for _ in range(3):  # keep the stream busy past the destroy
            binding.reshard(p, dsrc, ddst, stream=st)
        p.destroy()
        outs.append(ddst)
    torch.cuda.synchronize()
    for rnd, ddst in enumerate(outs):
        assert_same([t.cpu().numpy() for t in ddst], want, f"round {rnd}")
    assert binding.release_workspace() > 0


def test_threads_plan_and_reshard_side_by_side():
    """The library's process-wide state is behind locks: four host threads, each with its own stream,
    case and plans, build, run and destroy plans at the same time (ctypes drops the GIL in the calls)."""
    import threading
    cases = [synth.cfg2(layers=2, hidden=128 * (i + 1), ffn=344 * (i + 1), vocab=1000) for i in range(2)]
    cases += [synth.random_case(7100 + i, n_tensors=8, max_elems=30000, saved_mode="flat", target_mode="grid") for i in range(2)]
    prepared = []
    for c in cases:
        src = synth.materialize(c.saved, c.tensors, c.seed)
        prepared.append((c, [b.cuda() for b in src], oracle.reshard(c.saved, c.target, src, poison=POISON),
                         binding.layout_to_meta(c.saved), binding.layout_to_meta(c.target)))
    torch.cuda.synchronize()
    errors = []

    def worker(k):
        try:
            c, dsrc, want, sm, tm = prepared[k]
            st = torch.cuda.Stream()
            for rnd in range(5):
                ddst = [torch.full((n,), POISON, dtype=torch.uint8, device="cuda") for n in c.target.buf_bytes]
                st.wait_stream(torch.cuda.current_stream())
                p = binding.plan(sm, tm, stream=st)
                binding.reshard(p, dsrc, ddst, stream=st)
                p.destroy()
                st.synchronize()
                for got, w in zip(ddst, want):
                    if not np.array_equal(got.cpu().numpy(), w):
                        errors.append(f"thread {k} round {rnd}: mismatch")
        except Exception as e:  # noqa: BLE001 - reported below
            errors.append(f"thread {k}: {e!r}")

    threads = [threading.Thread(target=worker, args=(k,)) for k in range(len(prepared))]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors


def test_workspace_can_be_released_and_comes_back():
    case = synth.cfg2(layers=2, hidden=128, ffn=344, vocab=1000)
    check_case(case)
    freed = binding.release_workspace()
    assert freed > 0
    assert binding.release_workspace() == 0
    check_case(case)  # allocated again on demand
    assert binding.release_workspace() > 0


def test_reshard_captured_in_a_hip_graph():
    """One launch, no memset: a captured bcp_reshard replays correctly, with eager work and other
    launches on the same plan in between (the kernel's queue rearms itself)."""
    case = synth.cfg2(layers=2, hidden=256, ffn=688, vocab=2000)
    src = synth.materialize(case.saved, case.tensors, case.seed)
    want = oracle.reshard(case.saved, case.target, src, poison=POISON)
    sm, tm = binding.layout_to_meta(case.saved), binding.layout_to_meta(case.target)
    p = binding.plan(sm, tm)
    dsrc = [b.cuda() for b in src]
    ddst = [torch.full((n,), POISON, dtype=torch.uint8, device="cuda") for n in case.target.buf_bytes]
    binding.reshard(p, dsrc, ddst)  # eager first: sets the kernel up outside the capture
    torch.cuda.synchronize()
    assert_same([t.cpu().numpy() for t in ddst], want, "eager")
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        binding.reshard(p, dsrc, ddst, stream=torch.cuda.current_stream(), check_sizes=False)
    for i in range(4):
        for t in ddst:
            t.fill_(POISON)
        if i == 2:  # an eager launch on the same plan between two replays
            binding.reshard(p, dsrc, ddst)
            torch.cuda.synchronize()
            for t in ddst:
                t.fill_(POISON)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert_same([t.cpu().numpy() for t in ddst], want, f"replay {i}")
    del g
    p.destroy()


def test_plan_replay_on_other_buffers():
    case = synth.cfg2(layers=2, hidden=128, ffn=344, vocab=1000)
    sm, tm = binding.layout_to_meta(case.saved), binding.layout_to_meta(case.target)
    p = binding.plan(sm, tm)
    for seed in (1, 2, 3):
        src = synth.materialize(case.saved, case.tensors, seed)
        want = oracle.reshard(case.saved, case.target, src, poison=POISON)
        dsrc = [b.cuda() for b in src]
        ddst = [torch.full((n,), POISON, dtype=torch.uint8, device="cuda") for n in case.target.buf_bytes]
        binding.reshard(p, dsrc, ddst)
        torch.cuda.synchronize()
        assert_same([t.cpu().numpy() for t in ddst], want, f"replay {seed}")
    p.destroy()


def test_reshard_on_side_stream():
    case = synth.cfg1(512, 256)
    src = synth.materialize(case.saved, case.tensors, case.seed)
    want = oracle.reshard(case.saved, case.target, src, poison=POISON)
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        got, p = gpu_reshard(case, src)
    assert_same(got, want, "side stream")
    p.destroy()


# ---- edge cases ------------------------------------------------------------------------------------
def test_empty_inputs():
    p = binding.plan(np.zeros(0, dtype=binding.SHARD_META), np.zeros(0, dtype=binding.SHARD_META))
    assert p.stats()["n_regions"] == 0
    binding.reshard(p, [], [])
    p.destroy()
    # zero-volume shards on both sides and a scalar tensor
    spec = {0: TensorSpec(0, "w", (6, 4), torch.float32, ("bits",)), 1: TensorSpec(1, "s", (), torch.float64, ("bits",))}
    full = Part(0, (6, 4), (0, 0), (6, 4))
    saved = Layout([regular(full, 4, 0, 0), regular(Part(0, (6, 4), (6, 0), (0, 4)), 4, 0, 96),
                    regular(Part(1, (), (), ()), 8, 0, 96)], [104])
    target = Layout([regular(Part(0, (6, 4), (0, 0), (6, 2)), 4, 0, 0), regular(Part(0, (6, 4), (0, 2), (6, 2)), 4, 0, 48),
                     regular(Part(0, (6, 4), (3, 4), (2, 0)), 4, 0, 96), regular(Part(1, (), (), ()), 8, 0, 96)], [104])
    check_case(Case("edge", 3, spec, saved, target))


def test_unused_saved_tensor_is_ignored_and_uncovered_flag():
    spec = {0: TensorSpec(0, "w", (8, 4), torch.float32, ("bits",)), 1: TensorSpec(1, "u", (5,), torch.float32, ("bits",))}
    full = Part(0, (8, 4), (0, 0), (8, 4))
    saved = Layout([regular(Part(0, (8, 4), (0, 0), (4, 4)), 4, 0, 0), regular(Part(1, (5,), (0,), (5,)), 4, 0, 64)], [84])
    target = Layout([regular(full, 4, 0, 0)], [128])
    case = Case("uncov", 4, spec, saved, target)
    src = synth.materialize(saved, spec, 4)
    with pytest.raises(binding.BcpError) as e:
        gpu_reshard(case, src)
    assert e.value.name == "BCP_ERR_UNCOVERED"
    got, p = gpu_reshard(case, src, flags=binding.BCP_ALLOW_UNCOVERED)
    want = oracle.reshard(saved, target, src, poison=POISON, allow_uncovered=True)
    assert_same(got, want, "allow_uncovered")
    p.destroy()


def test_long_stretch_of_targets_without_saved_data():
    """Hundreds of target tensors in a row that no saved shard covers (allowed by flag): the candidate pairs of
    one workgroup then span far more target boxes than it has threads, on both sides of the stretch."""
    n_gap = 700
    spec, sv, tg = {}, [], []
    so = to = 0
    for f in range(n_gap + 40):
        spec[f] = TensorSpec(f, f"t{f}", (6, 4), torch.float32, ("bits",))
        covered = f < 20 or f >= 20 + n_gap
        if covered:  # saved as two row halves, asked for whole
            sv.append(regular(Part(f, (6, 4), (0, 0), (3, 4)), 4, 0, so))
            sv.append(regular(Part(f, (6, 4), (3, 0), (3, 4)), 4, 0, so + 48))
            so += 96
        tg.append(regular(Part(f, (6, 4), (0, 0), (6, 4)), 4, 0, to))
        to += 96
    case = Case("gap", 11, spec, Layout(sv, [so]), Layout(tg, [to]))
    src = synth.materialize(case.saved, spec, 11)
    got, p = gpu_reshard(case, src, flags=binding.BCP_ALLOW_UNCOVERED)
    want = oracle.reshard(case.saved, case.target, src, poison=POISON, allow_uncovered=True)
    assert_same(got, want, "gap")
    assert p.stats()["n_regions"] == 80
    p.destroy()


@pytest.mark.parametrize("n", [4095, 4096, 4097])
def test_saved_box_count_around_the_one_workgroup_sort_limit(n):
    """Up to 4096 saved boxes are grouped by FQN inside one workgroup, more by the device-wide sort: the
    same plan on either side of the limit.  FQN ids are sparse (several digits) and arrive in descending order,
    two saved boxes per tensor, so that the grouping has work to do and its stability shows."""
    half = n // 2
    fqns = [(i * 40503) % 1000003 for i in range(half + 1)]
    assert len(set(fqns)) == len(fqns)
    spec, sv, tg = {}, [], []
    so = to = 0
    for k, f in enumerate(sorted(fqns, reverse=True)):
        spec[f] = TensorSpec(f, f"t{f}", (4, 3), torch.float32, ("bits",))
        parts = [((0, 0), (2, 3)), ((2, 0), (2, 3))] if 2 * k + 1 < n else [((0, 0), (4, 3))]
        for off, ln in parts:
            sv.append(regular(Part(f, (4, 3), off, ln), 4, 0, so))
            so += ln[0] * ln[1] * 4
        if len(sv) >= n:
            break
    for f in sorted(spec):  # asked for whole, in ascending order
        tg.append(regular(Part(f, (4, 3), (0, 0), (4, 3)), 4, 0, to))
        to += 48
    assert len(sv) == n
    case = Case("sortlimit", 12, spec, Layout(sv, [so]), Layout(tg, [to]))
    src = synth.materialize(case.saved, spec, 12)
    got, p = gpu_reshard(case, src)
    want = oracle.reshard(case.saved, case.target, src, poison=POISON)
    assert_same(got, want, f"sortlimit{n}")
    assert p.stats()["n_saved_boxes"] == n
    p.destroy()


def _plan_error(saved: Layout, target: Layout, mutate=None):
    sm, tm = binding.layout_to_meta(saved), binding.layout_to_meta(target)
    if mutate:
        mutate(sm, tm)
    with pytest.raises(binding.BcpError) as e:
        binding.plan(sm, tm)
    return e.value.name


def test_error_statuses():
    full = Part(0, (8, 4), (0, 0), (8, 4))
    ok_s = Layout([regular(full, 4, 0, 0)], [128])
    ok_t = Layout([regular(full, 4, 0, 0)], [128])
    over = Layout([regular(Part(0, (8, 4), (0, 0), (5, 4)), 4, 0, 0), regular(Part(0, (8, 4), (4, 0), (4, 4)), 4, 1, 0)], [80, 64])
    assert _plan_error(over, ok_t) == "BCP_ERR_SAVED_OVERLAP"
    assert _plan_error(ok_s, Layout([regular(Part(0, (4, 8), (0, 0), (4, 8)), 4, 0, 0)], [128])) == "BCP_ERR_SHAPE_MISMATCH"
    assert _plan_error(ok_s, Layout([regular(full, 2, 0, 0)], [64])) == "BCP_ERR_DTYPE_MISMATCH"

    def oob(sm, tm):
        tm["offsets"][0, 0] = 4
    assert _plan_error(ok_s, ok_t, oob) == "BCP_ERR_OUT_OF_BOUNDS"

    def dims(sm, tm):
        tm["ndim"][0] = 9
    assert _plan_error(ok_s, ok_t, dims) == "BCP_ERR_TOO_MANY_DIMS"

    def item(sm, tm):
        sm["itemsize"][0] = 3
    assert _plan_error(ok_s, ok_t, item) == "BCP_ERR_INVALID_ARG"

    def flat(sm, tm):
        tm["flat_end"][0] = 33
    assert _plan_error(ok_s, ok_t, flat) == "BCP_ERR_OUT_OF_BOUNDS"
    # byte addresses that would leave the 64-bit range are refused, not wrapped
    def huge_stride(sm, tm):
        tm["strides"][0, 0] = 1 << 58
        tm["strides"][0, 1] = 1
    assert _plan_error(ok_s, ok_t, huge_stride) == "BCP_ERR_INVALID_ARG"

    def huge_offset(sm, tm):
        sm["byte_offset"][0] = 1 << 61
    assert _plan_error(ok_s, ok_t, huge_offset) == "BCP_ERR_INVALID_ARG"

    def huge_volume(sm, tm):
        for m in (sm, tm):
            m["global_shape"][0, :2] = (1 << 30, 1 << 30)
            m["lengths"][0, :2] = (1 << 30, 1 << 30)
            m["flat_end"][0] = 1 << 60
    assert _plan_error(ok_s, ok_t, huge_volume) == "BCP_ERR_INVALID_ARG"
    # too few buffers at reshard time
    p = binding.plan(binding.layout_to_meta(over.__class__([over.shards[0]], [80])),
                     binding.layout_to_meta(Layout([regular(Part(0, (8, 4), (0, 0), (5, 4)), 4, 2, 0)], [0, 0, 80])))
    with pytest.raises(binding.BcpError) as e:
        binding.reshard(p, [torch.zeros(80, dtype=torch.uint8, device="cuda")],
                        [torch.zeros(80, dtype=torch.uint8, device="cuda")])
    assert e.value.name == "BCP_ERR_INVALID_ARG"
    p.destroy()


# ---- the region list: unpinned by design (many lists are valid), only its invariants ----------------
def test_region_invariants():
    case = synth.cfg4(layers=2, hidden=64, ffn=96, vocab=200, dp_s=16, dp_t=12, n_states=1)
    sm, tm = binding.layout_to_meta(case.saved), binding.layout_to_meta(case.target)
    p = binding.plan(sm, tm)
    regs = p.regions()
    st = p.stats()
    assert len(regs) == st["n_regions"]
    vol = np.array([int(r["run_bytes"]) * int(np.prod(r["len"][:r["ndim"]])) for r in regs])
    assert vol.sum() == st["payload_bytes"] == case.target.payload_bytes()
    # per target record the region bytes add up to the record's bytes
    per = np.zeros(len(tm), dtype=np.int64)
    np.add.at(per, regs["target_index"], vol)
    assert np.array_equal(per, (tm["flat_end"] - tm["flat_begin"]) * tm["itemsize"])
    # destination byte intervals of contiguous regions never overlap inside one buffer
    for b in range(len(case.target.buf_bytes)):
        iv = sorted((int(r["dst_base"]), int(r["dst_base"]) + int(r["run_bytes"])) for r in regs
                    if r["dst_buf"] == b and r["ndim"] == 0)
        for (a0, a1), (b0, _) in zip(iv[:-1], iv[1:]):
            assert a1 <= b0
    p.destroy()
