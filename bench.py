#!/usr/bin/env python3
"""Benchmark of the load-time reshard hot path on one MI355X.

A step is one pass of the whole path over one synthetic checkpoint already resident in HBM:
bcp_plan (decompose flat shards, intersect saved and target boxes, compact, tile) followed by
bcp_reshard (the batched strided copy).  The default workload is the 7B-shaped decoder with bf16
weights and three fp32 Adam states, saved TP4 PP2 and loaded TP2 PP4, all eight target ranks
(94.3 GB read + 94.3 GB written per step).

Prints ONE JSON line: whole-step throughput in GB/s (bytes read + bytes written), the copy
kernel's HBM roofline figures measured with HIP events on the launch stream, and the CPU oracle
timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X HBM3E peak

# HBM bytes per k_reshard launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled by what the same
# counters read for a plain elementwise copy kernel of known size in the same run), per workload, with
# the hash of the kernel sources they were taken on.  Reported as null as soon as the sources differ.
MEASURED_TRAFFIC = {
    "cfg3": {"bytes_per_launch": 188971693554,
             "csrc_sha256": "9f86919682707823fae184debd7d4760935052a13a139c6e28df1a2f412a555f"},
    "eval_load": {"bytes_per_launch": 40469915879,
             "csrc_sha256": "9f86919682707823fae184debd7d4760935052a13a139c6e28df1a2f412a555f"},
    "cfg5_small": {"bytes_per_launch": 1931143684,
             "csrc_sha256": "9f86919682707823fae184debd7d4760935052a13a139c6e28df1a2f412a555f"},
}


def csrc_sha256() -> str:
    import glob
    import hashlib
    h = hashlib.sha256()
    for f in sorted(glob.glob(os.path.join(ROOT, "paper_2407_20143_amd", "csrc", "*"))):
        with open(f, "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()


def measured_traffic(workload: str):
    m = MEASURED_TRAFFIC.get(workload)
    if m is None or m["csrc_sha256"] != csrc_sha256():
        return None
    return m["bytes_per_launch"]


def build_case(name: str):
    from paper_2407_20143_amd import synth
    if name == "cfg1":
        return synth.cfg1(), "fp32 [1024,1024], 2 row shards -> 4 column shards (cache resident)"
    if name == "cfg2":
        return synth.cfg2(), "24-layer h2048 bf16 decoder, TP4PP2 -> TP2PP4, all target shards"
    if name == "cfg3":
        return synth.cfg3(), "7B decoder bf16 + 3 fp32 Adam states, TP4PP2 -> TP2PP4, all 8 target ranks"
    if name == "cfg3_rank0":
        return synth.cfg3(rank_share=True), "7B decoder bf16 + 3 fp32 Adam states, TP4PP2 -> TP2PP4, target rank (pp0,tp0)"
    if name == "cfg4":
        return synth.cfg4(), "7B fp32 optimizer states, ZeRO flat DP16 -> TP2 x DP12"
    if name == "cfg4_1state":
        return synth.cfg4(n_states=1), "7B fp32 optimizer state (one of three), ZeRO flat DP16 -> TP2 x DP12"
    if name == "cfg5":
        return synth.cfg5(), "MoE expert weights bf16 EP8TP2 -> EP4TP4 plus 100k small fp32 tensors, one plan"
    if name == "eval_load":
        return synth.eval_load_case(), "7B fp32 master weights saved TP4PP2, loaded as bf16 TP2PP4 (dtype-converting load)"
    if name == "eval_load_zero":
        return (synth.eval_load_case(zero_saved=True),
                "7B fp32 master weights saved as ZeRO flat slices DP16, loaded as bf16 TP2PP4 (dtype-converting load)")
    if name == "cfg5_experts":
        return synth.cfg5(n_small=0), "MoE expert weights bf16, EP8TP2 -> EP4TP4"
    if name == "cfg5_small":
        return synth.cfg5(include_experts=False), "100k small fp32 tensors under random 1-D shardings"
    if name == "vdit_32to64":
        return synth.table3_vdit(32, 64), "vDiT-shaped (h1664, 48 blocks) FSDP ZeRO-2 bf16 + 3 fp32 states, 32 -> 64 ranks"
    if name == "vdit_128to64":
        return synth.table3_vdit(128, 64), "vDiT-shaped (h1664, 48 blocks) FSDP ZeRO-2 bf16 + 3 fp32 states, 128 -> 64 ranks"
    if name == "tgpt_75to150":
        return synth.table3_tgpt_group(75, 150), "tGPT-70B-shaped, one TP4/PP8 group, fp32 Adam states, DP 75 -> 150"
    if name == "tgpt_150to75":
        return synth.table3_tgpt_group(150, 75), "tGPT-70B-shaped, one TP4/PP8 group, fp32 Adam states, DP 150 -> 75"
    if name == "cfg1_strided":
        return synth.cfg1(strided_target=True), "cfg1 with column-major target buffers (LDS-staged transpose, cache resident)"
    if name == "transpose":
        return synth.transpose_case(), "fp32 [16384,16384], 4 row blocks -> 4 column blocks stored column-major (LDS-staged transpose)"
    if name == "transpose_bf16":
        return synth.transpose_case(dtype=__import__("torch").bfloat16), "bf16 [16384,16384] row blocks -> column-major column blocks"
    if name in ("strided_read", "strided_write", "rows_1gib"):
        # fp32 [16384,16384] without a transposition: column blocks of 128 columns (512-byte runs at a
        # 64 KiB pitch) on the read or the write side; rows_1gib: no split at all (contiguous, same size)
        if name == "rows_1gib":
            return synth.column_blocks_case(cols=16384), "fp32 [16384,16384] copied whole (1 GiB, contiguous)"
        side = name.split("_")[1]
        return (synth.column_blocks_case(strided_side=side),
                f"fp32 [16384,16384] <-> 128 column blocks, 512-byte runs at a 64 KiB pitch on the {side} side, no transposition")
    if name == "fused_qkv":
        return synth.fused_qkv_case(), "fused GQA QKV blobs (32 layers, h4096, 32q/8kv heads) TP4 -> separate q,k,v TP2"
    if name.startswith("copy"):  # copy, copy_s4 (source shifted 4 bytes), copy_d4, copy_d2, copy_b4 (both sides) ...
        shift = int(name.split("_")[1][1:]) if "_" in name else 0
        side = name.split("_")[1][0] if "_" in name else "s"
        return (synth.copy_case(8 << 30, shift if side in "sb" else 0, shift if side in "db" else 0),
                "plain copy of one 8 GiB byte tensor through the reshard kernel (bandwidth ceiling)")
    if name.startswith("regions_"):  # regions_<bytes>_<gap before each, source>_<the same, destination>_<jitter>
        size, gs, gd, jit = (int(v) for v in name.split("_")[1:5])
        return (synth.regions_case(size, gs, gd, jit),
                f"6 GiB of byte tensors of {size} (+ up to {jit}) bytes packed with {gs} / {gd} bytes between them (source / destination)")
    raise SystemExit(f"unknown workload {name}")


def host_description():
    model, mem_kib = "unknown", 0
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
        with open("/proc/meminfo") as f:
            for line in f:
                if line.startswith("MemTotal"):
                    mem_kib = int(line.split()[1])
                    break
    except OSError:
        pass
    return {"cpu": model, "logical_cpus": os.cpu_count(), "ram_GiB": round(mem_kib / (1 << 20), 1)}


def oracle_samples(workload: str):
    """(case, description) for the all-cores run and for the single-thread run of the oracle: bounded parts of
    the workload, sized for roughly 10 s each."""
    from paper_2407_20143_amd import synth

    def llama_layers(n_layers, states, tp_s, tp_t, seed):
        model = synth.llama_tensors(n_layers, 4096, 11008, 32000)[1:1 + 9 * n_layers]
        return synth.Case("sample", seed, synth._specs(model, states),
                          synth.megatron_layout(model, states, n_layers, tp_s, 1, replicate_norms=False),
                          synth.megatron_layout(model, states, n_layers, tp_t, 1, replicate_norms=True))

    if workload.startswith("cfg3"):
        return ((llama_layers(8, synth.CFG3_STATES, 4, 2, synth.BASE_SEED + 3),
                 "eight of the 32 decoder layers (72 tensors x 4 states, 22.7 GB one way) of the 7B workload, TP4 -> TP2"),
                (llama_layers(1, synth.CFG3_STATES, 4, 2, synth.BASE_SEED + 3),
                 "one of the 32 decoder layers (9 tensors x 4 states, 2.8 GB one way) of the 7B workload, TP4 -> TP2"))
    if workload.startswith("eval_load"):
        def conv(n_layers):
            c = llama_layers(n_layers, [synth.STATE_FP32_MASTER], 4, 2, synth.BASE_SEED + 6)
            return synth.Case("sample", c.seed, c.tensors, c.saved, synth.narrowed(c.target), convert=1)
        return ((conv(8), "eight of the 32 decoder layers of the fp32 master weights, TP4 -> TP2 as bf16"),
                (conv(1), "one of the 32 decoder layers of the fp32 master weights, TP4 -> TP2 as bf16"))
    if workload.startswith("cfg4"):
        return ((synth.cfg4(layers=1, n_states=1), "embedding + one decoder layer + lm_head of one fp32 state, ZeRO flat DP16 -> TP2 x DP12"),
                (synth.cfg4(layers=1, vocab=4000, n_states=1), "one decoder layer + a 4000-row embedding and lm_head of one fp32 state"))
    if workload == "cfg2":
        return ((synth.cfg2(layers=4), "4 of 24 layers plus embedding and lm_head of the cfg2 workload"),
                (synth.cfg2(layers=1), "1 of 24 layers plus embedding and lm_head of the cfg2 workload"))
    if workload == "cfg5_experts":
        return ((synth.cfg5(layers=1, n_small=0), "one of 16 MoE layers of expert weights"),) * 2
    if workload in ("cfg5_small", "cfg5"):
        return ((synth.cfg5(include_experts=False, n_small=20000), "20000 of the 100000 small tensors"),
                (synth.cfg5(include_experts=False, n_small=5000), "5000 of the 100000 small tensors"))
    if workload.startswith("copy"):
        return ((synth.copy_case(1 << 30), "1 GiB of the 8 GiB byte tensor"),) * 2
    if workload.startswith("vdit"):
        a, b = (int(v) for v in workload.split("_")[1].split("to"))
        return ((synth.table3_vdit(a, b, layers=3), "3 of the 48 blocks (all four states) of the vDiT-shaped workload"),
                (synth.table3_vdit(a, b, layers=1), "1 of the 48 blocks (all four states) of the vDiT-shaped workload"))
    if workload.startswith("tgpt"):
        a, b = (int(v) for v in workload.split("_")[1].split("to"))
        c = synth.table3_tgpt_group(a, b, layers=1, first_stage=False)
        return ((c, "one of the 10 layers of the tGPT-shaped group (three fp32 states)"),) * 2
    return ((synth.cfg1(), "the whole cfg1 workload"),) * 2


def cpu_baseline(workload: str):
    """The oracle, as it stands, on bounded samples of the workload, on the host cores of the machine it runs on:
    with every core (at most 16 threads) and with one thread."""
    import torch
    from oracle import oracle
    from paper_2407_20143_amd import synth
    dev = "cuda" if torch.cuda.is_available() else "cpu"
    (case_n, what_n), (case_1, what_1) = oracle_samples(workload)
    threads = min(os.cpu_count() or 1, 16)

    def run(case, n_threads):
        src = [b.cpu() for b in synth.materialize(case.saved, case.tensors, case.seed, device=dev)]
        t0 = time.perf_counter()
        oracle.reshard(case.saved, case.target, src, threads=n_threads, convert=case.convert)
        dt = time.perf_counter() - t0
        moved = case.target.payload_bytes() * (3 if case.convert else 2)   # bytes read + bytes written
        return round(moved / dt / 1e9, 4), round(dt, 2)

    v_n, s_n = run(case_n, threads)
    v_1, s_1 = run(case_1, 1)
    return {"value": v_n, "unit": "GB/s", "cores": threads, "kind": "oracle", "sample": what_n, "seconds": s_n,
            "single_thread": {"value": v_1, "unit": "GB/s", "cores": 1, "sample": what_1, "seconds": s_1},
            "host": host_description()}


def count_mismatches(a, b) -> int:
    """Differing bytes of two equally long byte tensors on one device (in pieces: a whole-buffer mask would
    take as much memory again as the buffers)."""
    import torch
    if torch.equal(a, b):
        return 0
    step, bad = 256 << 20, 0
    for i in range(0, a.numel(), step):
        bad += int(torch.count_nonzero(a[i:i + step] != b[i:i + step]))
    return bad


def host_generated_fqns(workload: str, case):
    """Tensors whose values are generated on the host (torch's CPU and GPU generators give different streams, so
    the check below has to build every tensor where its input was built): the 100k small tensors of configuration
    5 -- one by one on the GPU they would take minutes; everything else is generated on the GPU."""
    import math
    if workload not in ("cfg5", "cfg5_small"):
        return set()
    return {f for f, spec in case.tensors.items() if math.prod(spec.shape) <= (1 << 20)}


def verify_result(case, src, dst, stream, reshard_once, generated: bool, on_host=frozenset()):
    """After the timed loop, outside it: the destination buffers are poisoned, one more reshard runs, and its
    result is compared on the device with the library-slicing closed form (synth.materialize of the TARGET
    layout), unit by unit: a flat buffer's slices together, otherwise one destination buffer at a time.
    Returns the number of differing bytes (must be 0) and how many were compared."""
    import torch
    from paper_2407_20143_amd import synth
    if not generated:
        return {"mismatched_bytes": None, "compared_bytes": 0, "method": "inputs are raw random bytes: not verified"}
    POISON = 0xA5
    for d in dst:
        d.fill_(POISON)
    reshard_once()
    torch.cuda.synchronize()
    bad = compared = 0
    groups, plain = {}, {}
    for sh in case.target.shards:
        (groups.setdefault(sh.group, []) if sh.group >= 0 else plain.setdefault(sh.buf, [])).append(sh)
    for b, shards in plain.items():
        where = {sh.parts[0].fqn in on_host for sh in shards}
        assert len(where) == 1, "a destination buffer mixes host-generated and GPU-generated tensors"
        dev = "cpu" if where.pop() else "cuda"
        want = synth.materialize(synth.Layout(shards, case.target.buf_bytes), case.tensors, case.seed, device=dev,
                                 poison=POISON, only_bufs={b})[b]
        bad += count_mismatches(dst[b], want.to(dst[b].device))
        compared += dst[b].numel()
        del want
    for gid, shards in groups.items():
        bufs = {sh.buf for sh in shards}
        want = synth.materialize(synth.Layout(shards, case.target.buf_bytes), case.tensors, case.seed, device="cuda",
                                 poison=POISON, only_bufs=bufs)
        for sh in shards:
            n = sh.numel * sh.itemsize
            bad += count_mismatches(dst[sh.buf][sh.byte_offset:sh.byte_offset + n], want[sh.buf][sh.byte_offset:sh.byte_offset + n])
            compared += n
        del want
    return {"mismatched_bytes": bad, "compared_bytes": compared,
            "method": "device compare with the library-slicing closed form of the target layout, after the timed loop"}


def from_host_leg(binding, saved_meta, target_meta, src, dst, chunk_bytes, payload):
    """Saved blobs start in pinned host memory.  (1) copy them all, then reshard; (2) copy chunk by
    chunk on a copy stream while a source-ordered plan reshards what has arrived."""
    import torch
    note("pinning host copies of the saved blobs")
    host = [b.cpu().pin_memory() for b in src]
    stage = [torch.empty_like(b) for b in src]
    copy_stream = torch.cuda.Stream()
    main = torch.cuda.current_stream()
    p_seq = binding.plan(saved_meta, target_meta, stream=main)
    p_ord = binding.plan(saved_meta, target_meta, flags=binding.BCP_ORDER_BY_SOURCE, stream=main)
    total_src = sum(b.numel() for b in src)

    def h2d_only():
        for h, d in zip(host, stage):
            d.copy_(h, non_blocking=True)

    def sequential():
        h2d_only()
        binding.reshard(p_seq, stage, dst, stream=main)

    def pipelined():
        binding.reshard_from_host(p_ord, host, stage, dst, chunk_bytes, copy_stream, stream=main)

    out = {"chunk_MiB": chunk_bytes >> 20, "host_bytes": total_src,
           "ordered_plan_ms": round(p_ord.stats()["plan_wall_ms"], 3), "plain_plan_ms": round(p_seq.stats()["plan_wall_ms"], 3)}
    for name, fn in (("h2d_only", h2d_only), ("copy_then_reshard", sequential), ("pipelined", pipelined)):
        fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(3):
            t0 = time.perf_counter()
            fn()
            torch.cuda.synchronize()
            ts.append((time.perf_counter() - t0) * 1e3)
        out[name + "_ms"] = round(min(ts), 3)
    out["h2d_GBps"] = round(total_src / out["h2d_only_ms"] / 1e6, 2)
    out["pipelined_payload_GBps"] = round(payload / out["pipelined_ms"] / 1e6, 2)
    out["tail_after_last_byte_ms"] = {"copy_then_reshard": round(out["copy_then_reshard_ms"] - out["h2d_only_ms"], 3),
                                      "pipelined": round(out["pipelined_ms"] - out["h2d_only_ms"], 3)}
    p_seq.destroy()
    p_ord.destroy()
    return out


def dedup_timing():
    """Save side (Sec. 4.1 'Balancing saving workload'): bcp_dedup_worst_fit on the live layout of the 7B model with
    four states under TP4 PP2 and 16 data-parallel replicas -- a host routine, no GPU involved."""
    import numpy as np
    from paper_2407_20143_amd import binding, synth
    model = synth.llama_tensors(32, 4096, 11008, 32000)
    live, rank_of = synth.replicated_live_layout(model, synth.CFG3_STATES, 32, 4, 2, 16)
    meta = binding.layout_to_meta(live, pinned=False)
    ts = []
    for _ in range(5):
        t0 = time.perf_counter()
        keep, load = binding.dedup_worst_fit(meta, rank_of, 4 * 2 * 16)
        ts.append((time.perf_counter() - t0) * 1e3)
    return {"metric": "bcp_dedup_worst_fit wall time", "value": round(min(ts), 3), "unit": "ms", "records": len(meta),
            "distinct_shards": int(keep.sum()), "ranks": 128, "max_over_mean_load": round(float(load.max() / load.mean()), 4),
            "host": host_description()}


def memfloor():
    """Run the stand-alone memory-floor measurement (bench_memfloor.hip, built by __graft_entry__.build)."""
    import subprocess
    exe = os.path.join(ROOT, "bench_memfloor")
    if not os.path.exists(exe):
        raise SystemExit("bench_memfloor is not built: run python -c 'import __graft_entry__ as g; g.build()' first")
    return subprocess.call([exe])


def note(msg: str):
    """Progress line on stderr (stdout carries only the JSON result)."""
    print(f"[bench {time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg3")
    ap.add_argument("--tile-bytes", type=int, default=0)
    ap.add_argument("--persistent", type=int, default=-1)
    ap.add_argument("--wg-per-cu", type=int, default=0)
    ap.add_argument("--threads", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--order-by-source", action="store_true",
                    help="build the plan with BCP_ORDER_BY_SOURCE (work ordered by source blob and source byte)")
    ap.add_argument("--meta-on-device", action="store_true",
                    help="upload the shard records once and plan from device memory (BCP_META_ON_DEVICE)")
    ap.add_argument("--raw-inputs", action="store_true",
                    help="fill the saved blobs with one random fill each instead of per-tensor values (byte traffic "
                         "is the same; keeps the dispatch count low under rocprofv3 --pmc)")
    ap.add_argument("--from-host", type=int, default=0, metavar="CHUNK_MIB",
                    help="also time the chunked host-to-HBM arrival overlapped with the reshard (pinned host copies "
                         "of the saved blobs, chunks of this many MiB) against copy-then-reshard")
    ap.add_argument("--pmc-reference", action="store_true",
                    help="for counter runs under rocprofv3 --pmc: instead of the ceiling copies (which would add other "
                         "k_reshard launches to the per-kernel averages) run one plain elementwise copy kernel of known "
                         "size, whose FETCH_SIZE / WRITE_SIZE readings give the scale of those counters")
    ap.add_argument("--reshard-only", action="store_true",
                    help="extra timing loop of bcp_reshard alone on a prebuilt plan (reported beside the step numbers)")
    ap.add_argument("--dedup-only", action="store_true",
                    help="time the save-side Worst-Fit deduplication (host routine) on the 7B live layout and exit")
    ap.add_argument("--memfloor", action="store_true",
                    help="run the stand-alone small-tile memory-floor measurement (bench_memfloor.hip) and exit")
    args = ap.parse_args()
    if args.dedup_only:
        print(json.dumps(dedup_timing()), flush=True)
        return
    if args.memfloor:
        raise SystemExit(memfloor())
    if args.gpus != 1:
        raise SystemExit("bench.py measures one GPU: the reshard path has no multi-GPU part (run with --gpus 1)")

    import torch
    from paper_2407_20143_amd import binding, synth
    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU")
    torch.cuda.set_device(0)
    binding.lib()
    binding.configure(tile_bytes=args.tile_bytes, persistent=args.persistent, wg_per_cu=args.wg_per_cu,
                      threads=args.threads)

    case, desc = build_case(args.workload)
    note(f"workload {args.workload}: generating inputs on the GPU")
    t0 = time.perf_counter()
    on_host = host_generated_fqns(args.workload, case)
    if args.raw_inputs:
        src = [torch.randint(0, 256, (n,), dtype=torch.uint8, device="cuda") for n in case.saved.buf_bytes]
    elif on_host:
        small_layout = synth.Layout([sh for sh in case.saved.shards if sh.parts[0].fqn in on_host], case.saved.buf_bytes)
        big_layout = synth.Layout([sh for sh in case.saved.shards if sh.parts[0].fqn not in on_host], case.saved.buf_bytes)
        small_bufs = {sh.buf for sh in small_layout.shards}
        assert not small_bufs & {sh.buf for sh in big_layout.shards}, "a blob mixes host-generated and GPU-generated tensors"
        src = synth.materialize(big_layout, case.tensors, case.seed, device="cuda", only_bufs=set(range(len(case.saved.buf_bytes))) - small_bufs)
        host = synth.materialize(small_layout, case.tensors, case.seed, only_bufs=small_bufs)
        src = [s if s is not None else h.cuda() for s, h in zip(src, host)]
        del host
    else:
        src = synth.materialize(case.saved, case.tensors, case.seed, device="cuda")
    dst = [torch.empty(n, dtype=torch.uint8, device="cuda") for n in case.target.buf_bytes]
    torch.cuda.synchronize()
    torch.cuda.empty_cache()  # hand the generator's temporaries back: the library allocates with hipMalloc
    t_gen = time.perf_counter() - t0
    saved_meta, target_meta = binding.layout_to_meta(case.saved), binding.layout_to_meta(case.target)
    payload = case.target.payload_bytes()
    stream = torch.cuda.current_stream()

    plan_flags = (binding.BCP_ORDER_BY_SOURCE if args.order_by_source else 0) | \
                 (binding.BCP_CONVERT_F32_TO_BF16 if case.convert else 0)
    if args.meta_on_device:
        (dev_s, n_s), (dev_t, n_t) = binding.meta_to_device(saved_meta), binding.meta_to_device(target_meta)

        def make_plan():
            return binding.plan_from_device_meta(dev_s, n_s, dev_t, n_t, flags=plan_flags, stream=stream)
    else:
        def make_plan():
            return binding.plan(saved_meta, target_meta, flags=plan_flags, stream=stream)

    def step():
        p = make_plan()
        binding.reshard(p, src, dst, stream=stream)
        return p

    note(f"inputs ready in {t_gen:.1f} s; first plan + checked reshard")
    # one checked pass first: buffer sizes against the plan's extents
    p = make_plan()
    binding.reshard(p, src, dst, stream=stream)
    stats = p.stats()
    assert stats["payload_bytes"] == payload
    moved = stats["src_bytes"] + stats["payload_bytes"]   # bytes read + bytes written per step (2 x payload unless converting)
    torch.cuda.synchronize()
    for _ in range(args.warmup):
        step().destroy()
    torch.cuda.synchronize()
    # plan build on its own: inside the timed loop a plan first waits for the previous step's copy
    iso_ms = []
    for _ in range(max(3, min(args.steps, 10))):
        torch.cuda.synchronize()
        tp = time.perf_counter()
        q = make_plan()
        iso_ms.append((time.perf_counter() - tp) * 1e3)
        q.destroy()
    note(f"warm-up done; timing {args.steps} steps")

    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    plan_ms = []
    prev = None
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        tp = time.perf_counter()
        pl = make_plan()
        plan_ms.append((time.perf_counter() - tp) * 1e3)
        ev[i][0].record(stream)
        binding.reshard(pl, src, dst, stream=stream)
        ev[i][1].record(stream)
        if prev is not None:
            prev.destroy()  # its copy has finished: building this step's plan waited for the stream
        prev = pl
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    prev.destroy()
    kern_ms = [a.elapsed_time(b) for a, b in ev]
    ms_per_step = dt * 1e3 / args.steps
    kern_avg = sum(kern_ms) / len(kern_ms)
    value = moved / (ms_per_step * 1e-3) / 1e9
    achieved = moved / (kern_avg * 1e-3) / 1e9

    note(f"timed: {ms_per_step:.3f} ms per step; verification and ceiling copies")
    verified = verify_result(case, src, dst, stream,
                             lambda: binding.reshard(p, src, dst, stream=stream), not args.raw_inputs, on_host)
    extra = {}
    if args.reshard_only:
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(args.steps):
            binding.reshard(p, src, dst, stream=stream)
        e1.record(stream)
        torch.cuda.synchronize()
        extra["reshard_only_ms"] = round(e0.elapsed_time(e1) / args.steps, 4)

    if args.from_host:
        extra["from_host"] = from_host_leg(binding, saved_meta, target_meta, src, dst, args.from_host << 20, payload)

    # Beside the result: (1) the practical ceiling -- one plain contiguous copy, as large as the buffers at hand
    # allow (at most 8 GiB), through the same plan and copy-kernel body: what the kernel reaches when there is
    # nothing to reshard.  It is launched through bcp_reshard_noalloc, whose kernel instance takes the buffer
    # pointers from a table (k_reshard_table): same body, another name, so that a kernel trace of this run keeps
    # the workload's launches (k_reshard) apart from these; (2) the runtime's own device-to-device copy of the
    # same bytes, for scale.
    n_copy = min(max(b.numel() for b in src), max(b.numel() for b in dst), 8 << 30) // 256 * 256
    big_s = max(src, key=lambda b: b.numel())
    big_d = max(dst, key=lambda b: b.numel())
    ceil, naive = {}, {}
    if args.pmc_reference:
        # torch's elementwise kernel for bitwise_xor on int32: reads n_ref bytes, writes n_ref bytes, nothing else
        n_ref = min(n_copy, 1 << 30) // 4 * 4
        a, b = big_s[:n_ref].view(torch.int32), big_d[:n_ref].view(torch.int32)
        for _ in range(3):
            torch.bitwise_xor(a, 0, out=b)
        torch.cuda.synchronize()
        ceil = {"reference_kernel": "elementwise bitwise_xor(int32, 0)", "reference_bytes_each_way": n_ref}
    elif n_copy >= 1 << 20:
        cc = synth.copy_case(n_copy)
        cp = binding.plan(binding.layout_to_meta(cc.saved), binding.layout_to_meta(cc.target), stream=stream)
        for name, fn, out in (("copy_through_k_reshard", lambda: binding.reshard_noalloc(cp, [big_s], [big_d], stream=stream), ceil),
                              ("runtime_memcpy_DtoD", lambda: big_d[:n_copy].copy_(big_s[:n_copy]), naive)):
            fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(5):
                fn()
            e1.record(stream)
            torch.cuda.synchronize()
            out[name + "_GBps"] = round(2 * n_copy * 5 / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1)
        cp.destroy()
        ceil["copy_bytes"] = naive["copy_bytes"] = n_copy
        ceil["achieved_over_ceiling"] = round(achieved / ceil["copy_through_k_reshard_GBps"], 4)
    p.destroy()

    # the instance of the copy kernel this plan runs on, as the profiler names it
    kernel_name = ("k_reshard_table" if stats["max_src_buf"] + stats["max_dst_buf"] + 2 > 256 else "k_reshard") + \
                  ("<true, " if stats["n_transposed"] else "<false, ") + ("true>" if case.convert else "false>")
    out = {
        "metric": "reshard GB/s (read+written)" + ("; 7B TP4PP2->TP2PP4" if args.workload == "cfg3" else "") +
                  "; plan + copy per step (% of HBM peak and plan-build ms alongside)",
        "value": round(value, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u8",
        "data": "synthetic",
        "config": {"workload": f"{args.workload}: {desc}", "payload_GB_one_way": round(payload / 1e9, 3),
                   "bytes_read_plus_written_GB": round(moved / 1e9, 3),
                   "tile_bytes": args.tile_bytes or "default", "persistent": args.persistent,
                   "wg_per_cu": args.wg_per_cu or "default", "threads": args.threads or "default",
                   "metadata": "device" if args.meta_on_device else "host",
                   "order": "by source" if args.order_by_source else "by target"},
        "pct_of_hbm_peak": round(100 * value / HBM_PEAK_GBPS, 2),
        "plan_build_ms": {"wall_median": round(sorted(iso_ms)[len(iso_ms) // 2], 4), "wall_min": round(min(iso_ms), 4),
                          "in_loop_avg_incl_wait_for_previous_copy": round(sum(plan_ms) / len(plan_ms), 4)},
        "reshard_kernel_ms": {"avg": round(kern_avg, 4), "min": round(min(kern_ms), 4), "max": round(max(kern_ms), 4)},
        "plan": {k: stats[k] for k in ("n_saved_boxes", "n_target_boxes", "n_pairs", "n_regions", "n_tiles",
                                       "n_batches", "n_transposed")},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": measured_traffic(args.workload),
                     "kernel": kernel_name, "bytes_per_launch": moved},
        "verified": verified,
        "ceiling": ceil,
        "naive_copy": naive,
        "input_generation_s": round(t_gen, 1),
    }
    out.update(extra)
    if not args.no_cpu_baseline:
        note("CPU oracle baseline on a sample of the workload")
        out["cpu_baseline"] = cpu_baseline(args.workload)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
