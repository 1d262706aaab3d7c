"""bcp_reshard_noalloc (queue words and pointer table in the library's static device array) against
bcp_reshard, byte for byte, through the C-ABI: two calls in a row on one GPU, the second on a smaller
input, so that whatever the first call left in the shared array has to be harmless.  Collected last:
a failure here must not hide the other GPU tests."""
import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2407_20143_amd import binding, synth
from paper_2407_20143_amd.synth import Case

pytestmark = pytest.mark.gpu

POISON = 0xA5


def _run_both(case: Case):
    src_cpu = synth.materialize(case.saved, case.tensors, case.seed)
    sm, tm = binding.layout_to_meta(case.saved), binding.layout_to_meta(case.target)
    p = binding.plan(sm, tm)
    dsrc = [b.cuda() for b in src_cpu]
    ref = [torch.full((n,), POISON, dtype=torch.uint8, device="cuda") for n in case.target.buf_bytes]
    got = [torch.full((n,), POISON, dtype=torch.uint8, device="cuda") for n in case.target.buf_bytes]
    binding.reshard(p, dsrc, ref)
    torch.cuda.synchronize()
    print(f"noalloc {case.name}: {len(dsrc)} + {len(got)} buffers, {p.stats()['n_batches']} batches", flush=True)
    binding.reshard_noalloc(p, dsrc, got)
    torch.cuda.synchronize()
    for i, (g, r) in enumerate(zip(got, ref)):
        assert torch.equal(g, r), f"{case.name}: buffer {i} differs between bcp_reshard_noalloc and bcp_reshard"
    want = oracle.reshard(case.saved, case.target, src_cpu, poison=POISON)
    for i, (g, w) in enumerate(zip(got, want)):
        assert np.array_equal(g.cpu().numpy(), w), f"{case.name}: buffer {i} differs from the oracle"
    # the same plan again: the array's queue words were left rearmed or are cleared, either way correct
    for g in got:
        g.fill_(POISON)
    binding.reshard_noalloc(p, dsrc, got)
    torch.cuda.synchronize()
    for i, (g, r) in enumerate(zip(got, ref)):
        assert torch.equal(g, r), f"{case.name}: second run, buffer {i}"
    p.destroy()


def test_noalloc_matches_reshard_on_two_calls_in_a_row():
    binding.configure(**binding.DEFAULT_CONFIG)
    # 700 + 700 buffers: five chunks of the pointer table, big and small tiles
    specs, saved, target = synth.small_tensor_case(1500, 78, n_bufs=700, max_shards=6, hi=2000)
    _run_both(Case("many700", 78, specs, saved, target))
    # then a smaller input: fewer buffers (most of the table keeps the first call's pointers), one tensor
    _run_both(synth.cfg1(384, 320))
    # long rows, several tiles per batch queue, ragged flat shards
    _run_both(synth.cfg4(layers=2, hidden=136, ffn=344, vocab=1000, dp_s=16, dp_t=12, n_states=1))


def test_noalloc_rejects_more_buffers_than_the_static_table_holds():
    specs, saved, target = synth.small_tensor_case(6000, 79, n_bufs=4200, max_shards=4, hi=64)
    case = Case("toomany", 79, specs, saved, target)
    p = binding.plan(binding.layout_to_meta(case.saved), binding.layout_to_meta(case.target))
    st = p.stats()
    assert st["max_src_buf"] + st["max_dst_buf"] + 2 > 8192
    # real buffers of the right sizes, so that even a call that wrongly went through would stay in bounds
    dsrc = [torch.zeros(max(n, 1), dtype=torch.uint8, device="cuda") for n in case.saved.buf_bytes]
    ddst = [torch.zeros(max(n, 1), dtype=torch.uint8, device="cuda") for n in case.target.buf_bytes]
    with pytest.raises(binding.BcpError) as e:
        binding.reshard_noalloc(p, dsrc, ddst)
    assert e.value.name == "BCP_ERR_INVALID_ARG" and "8192" in str(e.value)
    binding.reshard(p, dsrc, ddst)   # the allocating entry point still takes it
    torch.cuda.synchronize()
    p.destroy()
