"""CPU oracle of the save-side Worst-Fit deduplication.  TEST INFRASTRUCTURE ONLY.

Sec. 4.1 "Balancing saving workload" of the paper: model states are replicated across data-parallel
groups; the coordinator gives every tensor shard to one saver, namely the rank whose cumulative
assigned size is smallest when the shard's turn comes.  This is an algorithm (a greedy heuristic),
so the oracle takes its steps as stated, with the readings the library documents: shards are taken
in order of first appearance, only ranks that hold a replica are candidates, sizes are bytes, ties
go to the lowest rank.

Parity status: pinned by tests/test_dedup.py (every shard saved exactly once by a holder; replay
check that each choice was a least-loaded holder; the load spread bound of greedy assignment when
every rank holds every shard; a hand-worked example in tests/golden/worst_fit_example.txt).
"""
from typing import Dict, List, Sequence, Tuple


def worst_fit(shard_keys: Sequence[Tuple], sizes: Sequence[int], rank_of: Sequence[int], n_ranks: int):
    """shard_keys[i]: hashable identity of record i's shard; sizes[i]: its bytes; rank_of[i]: holder.
    Returns (keep flags, bytes per rank)."""
    order: List[Tuple] = []
    holders: Dict[Tuple, List[int]] = {}
    for i, k in enumerate(shard_keys):
        if k not in holders:
            holders[k] = []
            order.append(k)
        holders[k].append(i)
    load = [0] * n_ranks
    keep = [False] * len(shard_keys)
    for k in order:
        best = None
        for i in holders[k]:
            if best is None or (load[rank_of[i]], rank_of[i]) < (load[rank_of[best]], rank_of[best]):
                best = i
        keep[best] = True
        load[rank_of[best]] += sizes[best]
    return keep, load
