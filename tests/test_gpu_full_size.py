"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.

Per configuration:
  * the whole result is compared on the device with the library-slicing closed form
    (synth.materialize of the target layout, one group of target buffers at a time) -- a check the
    oracle itself is pinned to on small sizes;
  * the CPU oracle recomputes a sample of tensors (one of each kind, including the ones ZeRO slice
    boundaries cut) from the bytes the GPU path read, and those bytes are compared one by one.
Inputs are generated on the GPU; nothing is read from disk.
"""
import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2407_20143_amd import binding, synth

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(600)]
POISON = 0xA5


@pytest.fixture(autouse=True)
def _bench_config():
    binding.configure(**binding.DEFAULT_CONFIG)
    yield


def reshard_on_gpu(case):
    src = synth.materialize(case.saved, case.tensors, case.seed, device="cuda")
    dst = [torch.full((n,), POISON, dtype=torch.uint8, device="cuda") for n in case.target.buf_bytes]
    sm, tm = binding.layout_to_meta(case.saved), binding.layout_to_meta(case.target)
    p = binding.plan(sm, tm, flags=binding.BCP_CONVERT_F32_TO_BF16 if case.convert else 0)
    binding.reshard(p, src, dst)
    torch.cuda.synchronize()
    st = p.stats()
    assert st["payload_bytes"] == case.target.payload_bytes()
    p.destroy()
    return src, dst, sm, tm, st


def check_closed_form(case, dst, buf_groups):
    """dst == materialize(target) on the device, a group of buffers at a time."""
    for bufs in buf_groups:
        want = synth.materialize(case.target, case.tensors, case.seed, device="cuda", poison=POISON,
                                 only_bufs=set(bufs))
        for b in bufs:
            assert torch.equal(dst[b], want[b]), f"{case.name}: target buffer {b} differs from the closed form"
        del want


def check_oracle_sample(case, src, dst, sm, tm, fqns):
    """The oracle recomputes tensors `fqns` from the very bytes the GPU read; compare its output
    with the GPU's for every target record of those tensors."""
    fq = np.array(sorted(fqns), dtype=np.int64)
    src_host = [np.empty(n, dtype=np.uint8) for n in case.saved.buf_bytes]   # pages untouched unless used
    dst_host = [np.empty(n, dtype=np.uint8) for n in case.target.buf_bytes]
    for r in sm[np.isin(sm["fqn_id"], fq)]:
        n = int(r["flat_end"] - r["flat_begin"]) * int(r["itemsize"])
        o, b = int(r["byte_offset"]), int(r["buf"])
        src_host[b][o:o + n] = src[b][o:o + n].cpu().numpy()
    oracle.reshard(case.saved, case.target, src_host, dst_inplace=dst_host, only_fqns=list(fq), convert=case.convert)
    checked = 0
    for r in tm[np.isin(tm["fqn_id"], fq)]:
        n = int(r["flat_end"] - r["flat_begin"]) * int(r["itemsize"])
        o, b = int(r["byte_offset"]), int(r["buf"])
        got = dst[b][o:o + n].cpu().numpy()
        assert np.array_equal(got, dst_host[b][o:o + n]), f"{case.name}: fqn {int(r['fqn_id'])} differs from the oracle"
        checked += n
    assert checked > 0
    return checked


def fqns_by_name(case, names):
    return [f for f, s in case.tensors.items() if s.name in names]


def test_cfg2_full_against_the_whole_oracle():
    case = synth.cfg2()
    src, dst, sm, tm, st = reshard_on_gpu(case)
    assert st["n_regions"] == 4 * (2 + 24 * 7) + 2 * (1 + 24 * 2)
    want = oracle.reshard(case.saved, case.target, [b.cpu() for b in src], poison=POISON)
    for b, w in enumerate(want):
        assert np.array_equal(dst[b].cpu().numpy(), w), f"cfg2: buffer {b} differs from the oracle"
    check_closed_form(case, dst, [[b] for b in range(len(dst))])


def test_cfg3_full_model():
    case = synth.cfg3()
    src, dst, sm, tm, st = reshard_on_gpu(case)
    assert st["n_pairs"] == 4 * (226 * 8 + 65 * 2) and st["n_regions"] == 4 * (226 * 4 + 65 * 2)
    check_closed_form(case, dst, [[b] for b in range(len(dst))])
    names = {"embed.weight", "layers.0.ln1.weight", "layers.0.attn.q.weight", "layers.0.attn.o.weight",
             "layers.17.mlp.down.weight", "layers.31.mlp.up.weight", "final_norm.weight"}
    sample = [f for f, s in case.tensors.items()
              if any(s.name == n or (s.name.startswith(n) and s.name[len(n):] in (".master", ".exp_avg", ".exp_avg_sq"))
                     for n in names)]
    # all four states of a few tensors would be ~4.7 GB of oracle work; keep bf16 + one fp32 state of each
    sample = [f for f in sample if case.tensors[f].name.endswith((".weight", ".exp_avg"))]
    assert len(sample) == 14
    check_oracle_sample(case, src, dst, sm, tm, sample)


def test_cfg3_rank_share():
    case = synth.cfg3(rank_share=True)
    src, dst, sm, tm, st = reshard_on_gpu(case)
    assert len(dst) == 1 and st["payload_bytes"] == 875_102_208 * 14
    check_closed_form(case, dst, [[0]])
    check_oracle_sample(case, src, dst, sm, tm, fqns_by_name(case, {"layers.3.attn.o.weight", "layers.5.mlp.gate.weight.master",
                                                                   "layers.7.ln2.weight.exp_avg_sq"}))


def test_cfg4_full_zero_flat_shards():
    case = synth.cfg4()
    src, dst, sm, tm, st = reshard_on_gpu(case)
    # the ragged tail: 12 slices of 280778411 elements overshoot the TP-local buffer by 4
    assert case.target.shards[11].numel == 280_778_411 - 4
    groups = {}
    for sh in case.target.shards:
        groups.setdefault(sh.group, []).append(sh.buf)
    check_closed_form(case, dst, list(groups.values()))
    # tensors the DP cuts go through (row-split and column-split ones), one small one, first and last
    sample = fqns_by_name(case, {"embed.weight.master", "layers.2.attn.o.weight.master", "layers.2.ln1.weight.master",
                                 "layers.29.mlp.down.weight.exp_avg_sq"})
    assert len(sample) == 4
    check_oracle_sample(case, src, dst, sm, tm, sample)
    cut = [int(r["fqn_id"]) for r in sm if r["flat_begin"] != 0][:3]   # tensors a saved slice starts inside of
    check_oracle_sample(case, src, dst, sm, tm, [f for f in cut if case.tensors[f].shape[0] <= 4096] or cut[:1])


def _flat_target_groups(case):
    groups = {}
    for sh in case.target.shards:
        groups.setdefault(sh.group, set()).add(sh.buf)
    return groups


@pytest.mark.parametrize("dp", [(32, 64), (128, 64)])
def test_table3_vdit_full(dp):
    """vDiT-shaped FSDP ZeRO-2 reshard at full width and depth (48.6 GB one way)."""
    case = synth.table3_vdit(*dp)
    src, dst, sm, tm, st = reshard_on_gpu(case)
    # every target buffer holds a slice of every unit, so the closed form is built unit by unit
    for gid in sorted(_flat_target_groups(case))[::7]:
        shards = [sh for sh in case.target.shards if sh.group == gid]
        sub = synth.Layout(shards, case.target.buf_bytes)
        want = synth.materialize(sub, case.tensors, case.seed, device="cuda", poison=POISON)
        for sh in shards:
            n = sh.numel * sh.itemsize
            assert torch.equal(dst[sh.buf][sh.byte_offset:sh.byte_offset + n], want[sh.buf][sh.byte_offset:sh.byte_offset + n])
        del want
    sample = fqns_by_name(case, {"blocks.0.adaLN_modulation.weight", "blocks.17.attn_temp.qkv.weight.master",
                                 "blocks.47.mlp.fc2.weight.exp_avg_sq", "blocks.30.mlp.fc1.bias.exp_avg",
                                 "y_embedder.proj.weight.master"})
    assert len(sample) == 5
    check_oracle_sample(case, src, dst, sm, tm, sample)


@pytest.mark.parametrize("dp", [(75, 150), (150, 75)])
def test_table3_tgpt_group_full(dp):
    """tGPT-70B-shaped: one TP/PP group's fp32 Adam states, DP 75 <-> 150 (25.4 GB one way)."""
    case = synth.table3_tgpt_group(*dp)
    src, dst, sm, tm, st = reshard_on_gpu(case)
    for gid in _flat_target_groups(case):
        shards = [sh for sh in case.target.shards if sh.group == gid]
        sub = synth.Layout(shards, case.target.buf_bytes)
        want = synth.materialize(sub, case.tensors, case.seed, device="cuda", poison=POISON)
        for sh in shards:
            n = sh.numel * sh.itemsize
            assert torch.equal(dst[sh.buf][sh.byte_offset:sh.byte_offset + n], want[sh.buf][sh.byte_offset:sh.byte_offset + n])
        del want
    sample = fqns_by_name(case, {"layers.0.attention.qkv.weight.master", "layers.9.mlp.fc2.weight.exp_avg",
                                 "layers.4.input_layernorm.bias.exp_avg_sq", "layers.6.mlp.fc1.bias.master"})
    assert len(sample) == 4
    check_oracle_sample(case, src, dst, sm, tm, sample)


def test_one_region_beyond_4_gib():
    """A single 5 GiB region: byte offsets and tile counts past 2^32."""
    case = synth.copy_case(5 << 30, 0, 4)
    src, dst, sm, tm, st = reshard_on_gpu(case)
    assert st["n_regions"] == 1 and st["payload_bytes"] == 5 << 30
    assert torch.equal(dst[0][4:], src[0])
    assert bool((dst[0][:4] == POISON).all())


def test_transposed_target_1_gib():
    """All-LDS-path workload at 1 GiB: row blocks -> column blocks stored column-major."""
    case = synth.transpose_case()
    src, dst, sm, tm, st = reshard_on_gpu(case)
    assert st["n_transposed"] == st["n_regions"] == 16
    G = torch.cat([b.view(torch.int32).view(4096, 16384) for b in src])     # the whole tensor, row-major (as bits)
    for c in range(4):
        want = G[:, 4096 * c:4096 * (c + 1)].t().contiguous()              # column-major storage of the block
        assert torch.equal(dst[c].view(torch.int32).view(4096, 16384), want)
    case = synth.transpose_case(2048, 1536, torch.bfloat16, shards=2)
    src, dst, sm, tm, st = reshard_on_gpu(case)
    want = oracle.reshard(case.saved, case.target, [b.cpu() for b in src], poison=POISON)
    for b, w in enumerate(want):
        assert np.array_equal(dst[b].cpu().numpy(), w)


def test_fused_gqa_qkv_full():
    """32 layers, h 4096, 32 query / 8 KV heads: fused TP4 blobs -> separate q, k, v at TP2 (1.6 GB)."""
    case = synth.fused_qkv_case()
    src, dst, sm, tm, st = reshard_on_gpu(case)
    check_closed_form(case, dst, [[0], [1]])
    check_oracle_sample(case, src, dst, sm, tm, [0, 1, 2, 3 * 17, 3 * 31 + 2])


def test_cfg5_experts_full():
    case = synth.cfg5(n_small=0)
    src, dst, sm, tm, st = reshard_on_gpu(case)
    assert st["n_pairs"] == 48 * 256 and st["n_regions"] == 48 * 32
    check_closed_form(case, dst, [[b] for b in range(len(dst))])
    check_oracle_sample(case, src, dst, sm, tm, fqns_by_name(case, {"layers.0.experts.gate", "layers.9.experts.down"}))


def test_cfg5_small_tensors_full_against_the_whole_oracle():
    case = synth.cfg5(include_experts=False)
    src_cpu = synth.materialize(case.saved, case.tensors, case.seed)
    want = oracle.reshard(case.saved, case.target, src_cpu, poison=POISON)
    sm, tm = binding.layout_to_meta(case.saved), binding.layout_to_meta(case.target)
    p = binding.plan(sm, tm)
    src = [b.cuda() for b in src_cpu]
    dst = [torch.full((n,), POISON, dtype=torch.uint8, device="cuda") for n in case.target.buf_bytes]
    binding.reshard(p, src, dst)
    torch.cuda.synchronize()
    st = p.stats()
    assert st["n_saved_boxes"] + st["n_target_boxes"] > 1_000_000 and st["n_batches"] < st["n_tiles"] // 50
    for b, w in enumerate(want):
        assert np.array_equal(dst[b].cpu().numpy(), w), f"cfg5 small tensors: buffer {b} differs from the oracle"
    p.destroy()


def test_cfg5_whole_as_one_plan():
    """Configuration 5 as the ONE plan it is: the stacked expert tensors and the 100 000 small tensors together.
    Experts against the closed form on the device, small tensors against the whole oracle, counts asserted."""
    case = synth.cfg5()
    experts = {f for f, s in case.tensors.items() if "experts" in s.name}
    assert len(experts) == 48 and len(case.tensors) == 100_048
    e_saved = synth.Layout([sh for sh in case.saved.shards if sh.parts[0].fqn in experts], case.saved.buf_bytes)
    s_saved = synth.Layout([sh for sh in case.saved.shards if sh.parts[0].fqn not in experts], case.saved.buf_bytes)
    e_target = synth.Layout([sh for sh in case.target.shards if sh.parts[0].fqn in experts], case.target.buf_bytes)
    s_target = synth.Layout([sh for sh in case.target.shards if sh.parts[0].fqn not in experts], case.target.buf_bytes)
    e_bufs = sorted({sh.buf for sh in e_saved.shards})
    # small tensors are generated on the host (100k tiny tensors one by one on the GPU take minutes), experts on the GPU
    small_src = synth.materialize(s_saved, case.tensors, case.seed)
    src = synth.materialize(e_saved, case.tensors, case.seed, device="cuda", only_bufs=set(e_bufs))
    for b in range(len(src)):
        if src[b] is None:
            src[b] = small_src[b].cuda()
    assert not (set(e_bufs) & {sh.buf for sh in s_saved.shards})   # experts and small tensors live in separate blobs
    dst = [torch.full((n,), POISON, dtype=torch.uint8, device="cuda") for n in case.target.buf_bytes]
    sm, tm = binding.layout_to_meta(case.saved), binding.layout_to_meta(case.target)
    p = binding.plan(sm, tm)
    binding.reshard(p, src, dst)
    torch.cuda.synchronize()
    st = p.stats()
    assert st["payload_bytes"] == case.target.payload_bytes()
    assert st["n_saved_boxes"] + st["n_target_boxes"] > 1_000_000 and st["n_regions"] > 48 * 32
    p.destroy()
    et_bufs = sorted({sh.buf for sh in e_target.shards})
    for b in et_bufs:
        want = synth.materialize(e_target, case.tensors, case.seed, device="cuda", poison=POISON, only_bufs={b})
        assert torch.equal(dst[b], want[b]), f"cfg5: expert buffer {b} differs from the closed form"
        del want
    want = oracle.reshard(s_saved, s_target, small_src, poison=POISON)
    for b in sorted({sh.buf for sh in s_target.shards}):
        assert np.array_equal(dst[b].cpu().numpy(), want[b]), f"cfg5: small-tensor buffer {b} differs from the oracle"
    check_oracle_sample(case, src, dst, sm, tm, fqns_by_name(case, {"layers.3.experts.up"}))


@pytest.mark.parametrize("zero_saved", [False, True])
def test_eval_load_full_fp32_master_as_bf16(zero_saved):
    """The dtype-converting load at full size: the 7B fp32 master weights (27 GB), saved TP4 PP2 or as ZeRO flat
    slices, loaded as bf16 under TP2 PP4."""
    case = synth.eval_load_case(zero_saved=zero_saved)
    src, dst, sm, tm, st = reshard_on_gpu(case)
    assert st["src_bytes"] == 2 * st["payload_bytes"] == 4 * 6_738_415_616 + 4 * 65 * 4096   # (norms go to both TP ranks)
    check_closed_form(case, dst, [[b] for b in range(len(dst))])
    sample = fqns_by_name(case, {"embed.weight.master", "layers.0.ln1.weight.master", "layers.11.attn.o.weight.master",
                                 "layers.31.mlp.down.weight.master"})
    assert len(sample) == 4
    check_oracle_sample(case, src, dst, sm, tm, sample)
