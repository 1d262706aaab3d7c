"""Save-side Worst-Fit deduplication (Sec. 4.1 "Balancing saving workload") and the save -> load
round through real save plans.  CPU tests pin the oracle (oracle/dedup_oracle.py) and compare the
library's host routine with it; the GPU test packs the kept live shards into save blobs with the
copy engine and reshards those to a new layout."""
import numpy as np
import pytest
import torch

from oracle import dedup_oracle, oracle
from paper_2407_20143_amd import binding, synth
from tests.conftest import read_golden


def _ints(s):
    return [int(v) for v in s.split()]


def _keys(meta):
    return [(int(r["fqn_id"]), int(r["ndim"]), int(r["itemsize"]), tuple(r["offsets"][:r["ndim"]].tolist()),
             tuple(r["lengths"][:r["ndim"]].tolist()), int(r["flat_begin"]), int(r["flat_end"])) for r in meta]


def _sizes(meta):
    return [int(r["flat_end"] - r["flat_begin"]) * int(r["itemsize"]) for r in meta]


def test_hand_worked_example():
    g = read_golden("worst_fit_example.txt")
    sizes, n_ranks = _ints(g["sizes"]), int(g["ranks"])
    keys, sz, ranks = [], [], []
    for s_i, s in enumerate(sizes):
        for r in range(n_ranks):
            keys.append(("shard", s_i))
            sz.append(s)
            ranks.append(r)
    keep, load = dedup_oracle.worst_fit(keys, sz, ranks, n_ranks)
    savers = [ranks[i] for i in range(len(keys)) if keep[i]]
    assert savers == _ints(g["savers"]) and load == _ints(g["loads"])
    # the library's host routine on the same example
    meta = np.zeros(len(keys), dtype=binding.SHARD_META)
    for i, (k, s) in enumerate(zip(keys, sz)):
        meta[i]["fqn_id"], meta[i]["ndim"], meta[i]["itemsize"] = k[1], 1, 1
        meta[i]["global_shape"][0] = meta[i]["lengths"][0] = meta[i]["flat_end"] = s
    keep2, load2 = binding.dedup_worst_fit(meta, ranks, n_ranks)
    assert list(keep2) == keep and list(load2) == load


def _random_instance(seed):
    rng = np.random.default_rng(seed)
    n_ranks = int(rng.integers(1, 9))
    keys, sizes, ranks = [], [], []
    for s in range(int(rng.integers(1, 60))):
        size = int(rng.integers(1, 1000))
        holders = rng.permutation(n_ranks)[:int(rng.integers(1, n_ranks + 1))]
        for r in holders:
            keys.append(("s", s))
            sizes.append(size)
            ranks.append(int(r))
    order = rng.permutation(len(keys))  # replicas of one shard need not be adjacent
    return [keys[i] for i in order], [sizes[i] for i in order], [ranks[i] for i in order], n_ranks


@pytest.mark.parametrize("seed", range(20))
def test_oracle_invariants(seed):
    keys, sizes, ranks, n_ranks = _random_instance(seed)
    keep, load = dedup_oracle.worst_fit(keys, sizes, ranks, n_ranks)
    # every shard is saved exactly once, by a rank that holds it
    kept = {}
    for i, k in enumerate(keys):
        if keep[i]:
            assert k not in kept
            kept[k] = i
    assert set(kept) == set(keys)
    assert sum(load) == sum(sizes[i] for i in kept.values())
    # replay: when its turn came, the saver was a least-loaded holder (lowest rank among ties)
    first = {}
    for i, k in enumerate(keys):
        first.setdefault(k, i)
    running = [0] * n_ranks
    for k in sorted(first, key=first.get):
        holders = sorted({ranks[i] for i, kk in enumerate(keys) if kk == k})
        chosen = ranks[kept[k]]
        assert (running[chosen], chosen) == min((running[r], r) for r in holders)
        running[chosen] += sizes[kept[k]]
    assert running == load


@pytest.mark.parametrize("seed", range(5))
def test_full_replication_is_balanced(seed):
    """When every rank holds every shard, greedy least-loaded assignment keeps the spread of the
    loads within the largest shard."""
    rng = np.random.default_rng(100 + seed)
    n_ranks = int(rng.integers(2, 9))
    sizes = [int(v) for v in rng.integers(1, 5000, size=200)]
    keys = [("s", s) for s in range(len(sizes)) for _ in range(n_ranks)]
    sz = [sizes[s] for s in range(len(sizes)) for _ in range(n_ranks)]
    ranks = [r for _ in sizes for r in range(n_ranks)]
    _, load = dedup_oracle.worst_fit(keys, sz, ranks, n_ranks)
    assert max(load) - min(load) <= max(sizes)


def _live_case(dp=3):
    model = synth.llama_tensors(2, 64, 176, 256)
    states = [synth.STATE_BF16_WEIGHT, synth.STATE_FP32_EXP_AVG]
    live, rank_of = synth.replicated_live_layout(model, states, 2, tp=2, pp=2, dp=dp)
    return model, states, synth._specs(model, states), live, rank_of, 2 * 2 * dp


def test_library_matches_oracle_on_model_layout():
    _, _, _, live, rank_of, n_ranks = _live_case()
    meta = binding.layout_to_meta(live)
    keep, load = binding.dedup_worst_fit(meta, rank_of, n_ranks)
    okeep, oload = dedup_oracle.worst_fit(_keys(meta), _sizes(meta), rank_of, n_ranks)
    assert list(keep) == okeep and list(load) == oload
    # one saver per distinct shard (split shards have dp replicas, norms tp * dp)
    assert keep.sum() == len(set(_keys(meta))) < len(meta) // 3 + 1
    for seed in range(10):
        keys, sizes, ranks, n = _random_instance(500 + seed)
        m = np.zeros(len(keys), dtype=binding.SHARD_META)
        for i, (k, s) in enumerate(zip(keys, sizes)):
            m[i]["fqn_id"], m[i]["ndim"], m[i]["itemsize"] = k[1], 1, 1
            m[i]["global_shape"][0] = m[i]["lengths"][0] = m[i]["flat_end"] = s
        k2, l2 = binding.dedup_worst_fit(m, ranks, n)
        ok, ol = dedup_oracle.worst_fit(keys, sizes, ranks, n)
        assert list(k2) == ok and list(l2) == ol


def test_bad_arguments():
    m = np.zeros(2, dtype=binding.SHARD_META)
    m["itemsize"] = 4
    with pytest.raises(binding.BcpError):
        binding.dedup_worst_fit(m, [0, 5], 2)


@pytest.mark.gpu
def test_save_plan_then_load_plan_on_gpu():
    """live shards (DP-replicated) -> Worst-Fit savers -> pack into save blobs (copy engine, live ->
    saved) -> load into another parallelism; every stage against the oracle, the end against the
    library-slicing closed form."""
    model, states, specs, live, rank_of, n_ranks = _live_case(dp=3)
    seed = 11
    meta = binding.layout_to_meta(live)
    keep, load = binding.dedup_worst_fit(meta, rank_of, n_ranks)
    assert load.max() - load.min() <= max(_sizes(meta)) * 2
    kept = [sh for sh, k in zip(live.shards, keep) if k]
    kept_live = synth.Layout(kept, live.buf_bytes)                       # where the savers' bytes are now
    blobs = synth.packed_layout(kept, [sh.buf for sh in kept], n_ranks)  # the checkpoint: one blob per rank
    target = synth.megatron_layout(model, states, 2, tp=1, pp=1, replicate_norms=True)
    live_bufs = synth.materialize(live, specs, seed)
    # save
    p = binding.plan(binding.layout_to_meta(kept_live), binding.layout_to_meta(blobs))
    d_live = [b.cuda() for b in live_bufs]
    d_blobs = [torch.full((n,), 0xA5, dtype=torch.uint8, device="cuda") for n in blobs.buf_bytes]
    binding.reshard(p, d_live, d_blobs)
    torch.cuda.synchronize()
    want_blobs = oracle.reshard(kept_live, blobs, live_bufs, poison=0xA5)
    for g, w in zip(d_blobs, want_blobs):
        assert np.array_equal(g.cpu().numpy(), w)
    p.destroy()
    # load with a new layout
    p = binding.plan(binding.layout_to_meta(blobs), binding.layout_to_meta(target))
    d_t = [torch.full((n,), 0xA5, dtype=torch.uint8, device="cuda") for n in target.buf_bytes]
    binding.reshard(p, d_blobs, d_t)
    torch.cuda.synchronize()
    want = [b.numpy() for b in synth.materialize(target, specs, seed, poison=0xA5)]
    for g, w in zip(d_t, want):
        assert np.array_equal(g.cpu().numpy(), w)
    p.destroy()
