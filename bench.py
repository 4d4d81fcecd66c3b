#!/usr/bin/env python3
"""Benchmark of the train->generation weight reshard (HybridFlow Section 5.2 step 1) on
one MI355X.  One "step" = one hf_reshard_execute over all materialised generation
ranks of the workload, inputs resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2] [--direction fwd|back]
                    [--flags skip_own|copy_own] [--from-gen] [--variant V] [--tile-bytes B] [--grid G]
                    [--no-cpu-baseline] [--no-ceilings] [--no-full-refresh]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, vendor figure

CONFIGS = {
    1: dict(name="tiny", model=dict(n_layers=2, hidden=256, n_q_heads=4, n_kv_heads=4, head_dim=64, ffn=688, vocab=1024),
            train=(1, 4, 1), gen=(1, 2), mat=None),
    2: dict(name="llama7b_tp8_to_tp2", model=dict(n_layers=32, hidden=4096, n_q_heads=32, n_kv_heads=32, head_dim=128, ffn=11008, vocab=32000),
            train=(1, 8, 1), gen=(1, 2), mat=None),
    3: dict(name="llama13b_tp4pp2_to_tp2", model=dict(n_layers=40, hidden=5120, n_q_heads=40, n_kv_heads=40, head_dim=128, ffn=13824, vocab=32000),
            train=(2, 4, 1), gen=(1, 2), mat=None),
    4: dict(name="llama34b_gqa_tp8pp2_to_tp4", model=dict(n_layers=48, hidden=8192, n_q_heads=64, n_kv_heads=8, head_dim=128, ffn=22016, vocab=32000),
            train=(2, 8, 1), gen=(1, 4), mat=[0, 2, 4, 6]),
    5: dict(name="llama70b_gqa_tp8pp4_to_tp4", model=dict(n_layers=80, hidden=8192, n_q_heads=64, n_kv_heads=8, head_dim=128, ffn=28672, vocab=128256),
            train=(4, 8, 1), gen=(1, 4), mat=[0, 31]),
}


def measured_traffic(workload, direction, default_config):
    """(HBM bytes per launch, source) from the committed rocprofv3 counter summary of this
    workload and direction (a separate profiling run of the same launch configuration: it is
    NOT measured in this process); (None, None) if there is none or if this run does not use
    the default configuration the counters were taken with."""
    name = "hbm_traffic_default_launches.txt"
    path = os.path.join(ROOT, "profiles", name)
    if not default_config or not os.path.exists(path):
        return None, None
    for line in open(path):
        f = line.split()
        if len(f) == 5 and f[0] == workload and f[1] == direction:
            return int(f[2]) + int(f[3]), f"profiles/{name} (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of a separate run, replayed here)"
    return None, None


def cpu_baseline(cfg, seconds_target=9.0):
    """The CPU oracle, as it stands, on a bounded sample of the same workload: whole layers
    of all materialised generation ranks, first on one thread, then (further layers) with a
    plain thread pool over (rank, tensor) on all cores the process may use.  Bytes are
    counted as for the GPU figure of a full refresh: every generation byte the oracle writes
    plus every distinct training byte it reads."""
    from concurrent.futures import ThreadPoolExecutor

    import numpy as np

    from oracle.reshard_oracle import GenLayout, Model, ReshardOracle, TrainLayout
    from seeded_inputs import bits16_torch, config_seed, stream_key, tensor_uid

    m = cfg["model"]
    orc = ReshardOracle(Model(m["n_layers"], m["hidden"], m["n_q_heads"], m["n_kv_heads"], m["head_dim"], m["ffn"], m["vocab"]),
                        TrainLayout(*cfg["train"]), GenLayout(*cfg["gen"]))
    ranks = cfg["mat"] if cfg["mat"] is not None else list(range(orc.n_ranks))
    seed = config_seed(cfg["index"] - 1)
    offs = orc.train_region_offsets()
    cores = len(os.sched_getaffinity(0))
    for r in range(orc.n_ranks):                      # table caches, so that threads only read them
        e0 = orc.train_table(r)[0][0]
        orc.train_entry(r, e0.kind, e0.layer)

    def layer_inputs(layer):                          # not timed
        store, n = {}, 0
        for r in range(orc.n_ranks):
            _, pp, tp = orc.train_coords(r)
            if layer // orc.lps != pp:
                continue
            for e in orc.train_table(r)[0]:
                if e.layer == layer:
                    uid = tensor_uid(e.kind, layer, 0 if e.kind in ("ln1", "ln2") else tp)
                    store[offs[r] + e.offset] = bits16_torch(stream_key(seed, uid), 0, e.n).numpy().view(np.uint16)
                    n += e.n
        return store, 2 * n

    def one(fetch, r, e):
        out = np.ascontiguousarray(orc.gen_tensor(fetch, r, e.kind, e.layer))     # the write into the generation buffer
        return 2 * out.size

    # one layer's inputs are generated once (seeded, not timed) and that layer is resharded again
    # and again: every layer of the model has the same shapes, and the oracle never looks at values
    layer = orc.m.n_layers // 2
    store, in_bytes = layer_inputs(layer)
    fetch = lambda o, n: store[o]
    work = [(r, e) for r in ranks for e in orc.gen_table(r)[0] if e.layer == layer]
    legs = []
    for threads in sorted({1, cores}):
        spent, written, read, reps = 0.0, 0, 0, 0
        pool = ThreadPoolExecutor(threads) if threads > 1 else None
        while spent < seconds_target:
            t0 = time.perf_counter()
            if pool:
                written += sum(pool.map(lambda re: one(fetch, *re), work))
            else:
                written += sum(one(fetch, r, e) for r, e in work)
            spent += time.perf_counter() - t0
            read += in_bytes
            reps += 1
        if pool:
            pool.shutdown()
        legs.append({"value": round((written + read) / spent / 1e9, 3), "cores": threads, "reps": reps,
                     "seconds": round(spent, 1), "GB": round((written + read) / 1e9, 2)})
    best = legs[-1]
    return {"value": best["value"], "unit": "GB/s", "cores": best["cores"], "kind": "oracle",
            "single_thread": {"value": legs[0]["value"], "unit": "GB/s", "cores": 1},
            "sample": f"numpy oracle (rebuild every full tensor from all training shards, slice): layer {layer} of {orc.m.n_layers} (all layers "
                      f"have the same shapes) for all {len(ranks)} generation ranks of {cfg['name']}, repeated: {legs[0]['reps']} times on 1 thread "
                      f"({legs[0]['GB']} GB in {legs[0]['seconds']} s)"
                      + (f", {best['reps']} times on a pool of {best['cores']} threads over (rank, tensor) ({best['GB']} GB in {best['seconds']} s)"
                         if len(legs) > 1 else "")
                      + "; bytes = generation bytes written + distinct training bytes read (the accounting of the GPU's full refresh)"}


def measured_ceilings(ar, n_dst, stream):
    """What this machine sustains for plain streams of known traffic, from the library's
    calibration kernels, in this process after the timed region: one-shot workgroups like the
    default kernel, a read-only, a write-only and a 1:1 stream, and the workload's own mix of
    one read per n_dst writes (loaded once and stored n_dst times, copied block-wise so that
    L2 serves the re-reads, or stored n_dst times after a load-only pass over the block).  The
    copies scribble over gen_buf."""
    import torch

    from paper_2409_19256_amd import binding as B

    src_bytes = min(4 << 30, ar.train.numel() * 2, ar.gen.numel() * 2 // max(n_dst, 1)) // 65536 * 65536
    region = ar.gen.numel() * 2 // max(len(ar.plan.mat_ranks), 1) // 256 * 256
    stride = region if region >= src_bytes and (n_dst - 1) * region + src_bytes <= ar.gen.numel() * 2 else src_bytes

    def timed(fn, traffic, reps=5):
        fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return round(traffic / (a.elapsed_time(b) / reps * 1e-3) / 1e9, 1)

    def fan(src, dst, n, blk, wg, method=None):
        method = (B.HF_FANOUT_CACHE_BLOCKED if blk else B.HF_FANOUT_REGISTERS) if method is None else method
        return lambda: B.check(B.hf_calib_fanout(src, dst, src_bytes, n, stride if n > 1 else src_bytes, method, blk, wg, stream),
                               "hf_calib_fanout")

    t, g = ar.train_ptr, ar.gen_ptr
    out = {"unit": "GB/s", "source_bytes": src_bytes,
           "read_only": timed(fan(t, None, 1, 0, 4096), src_bytes),
           "write_only": timed(fan(None, g, 1, 0, 4096), src_bytes),
           "copy_1_to_1": max(timed(fan(t, g, 1, 0, wg), 2 * src_bytes) for wg in (1024, 4096))}
    if n_dst > 1:
        mix = {f"registers_{wg}B": timed(fan(t, g, n_dst, 0, wg), (1 + n_dst) * src_bytes) for wg in (1024, 4096)}
        mix.update({f"cache_blocked_{blk >> 20}MiB_{wg}B": timed(fan(t, g, n_dst, blk, wg), (1 + n_dst) * src_bytes)
                    for blk in (2 << 20, 4 << 20) for wg in (4096, 8192)})
        mix.update({f"prefetched_{blk >> 20}MiB_1024B": timed(fan(t, g, n_dst, blk, 1024, B.HF_FANOUT_PREFETCHED), (1 + n_dst) * src_bytes)
                    for blk in (8 << 20, 16 << 20)})
        out["mix"] = f"1 read : {n_dst} writes, destinations {stride} bytes apart"
        out["mix_variants"] = mix
        out["mix_best"] = max(mix.values())
    else:
        out["mix"] = "1 read : 1 write"
        out["mix_best"] = out["copy_1_to_1"]
    return out


def placement_ab(cfg, flags, placements, steps):
    """The time of one launch depends on the physical pages behind the buffers by several per cent, and a process
    gets them by lot; comparing two launch configurations in two processes compares two lots.  Here every
    alternative runs on the same `placements` allocations of the buffers: between two of them the buffers are
    freed, a little more memory is held back, and they are allocated again."""
    import torch

    from paper_2409_19256_amd import Plan, binding as B
    from paper_2409_19256_amd.arena import Arena
    variants = [("library defaults", []),
                ("prefetched, one load-only tile per copy tile", [(B.HF_PARAM_MULTICAST, 3), (B.HF_PARAM_PREFETCH_MERGE, 1)]),
                ("prefetched, 2 copy tiles per load-only tile", [(B.HF_PARAM_MULTICAST, 3), (B.HF_PARAM_PREFETCH_MERGE, 2)]),
                ("prefetched, 4 copy tiles per load-only tile", [(B.HF_PARAM_MULTICAST, 3), (B.HF_PARAM_PREFETCH_MERGE, 4)]),
                ("prefetched, blocks of 4 MiB", [(B.HF_PARAM_MULTICAST, 3), (B.HF_PARAM_PREFETCH_BLOCK_BYTES, 4 << 20)]),
                ("prefetched, blocks of 8 MiB", [(B.HF_PARAM_MULTICAST, 3), (B.HF_PARAM_PREFETCH_BLOCK_BYTES, 8 << 20)]),
                ("prefetched, blocks of 16 MiB", [(B.HF_PARAM_MULTICAST, 3), (B.HF_PARAM_PREFETCH_BLOCK_BYTES, 16 << 20)]),
                ("tiles of 64 KiB", [(B.HF_PARAM_TILE_BYTES, 65536)]),
                ("tiles of 256 KiB", [(B.HF_PARAM_TILE_BYTES, 262144)]),
                ("row interleave off", [(B.HF_PARAM_ROW_INTERLEAVE, 0)]),
                ("cache-blocked list", [(B.HF_PARAM_MULTICAST, 2)]),
                ("cache-blocked list, blocks of 4 MiB", [(B.HF_PARAM_MULTICAST, 2), (B.HF_PARAM_MC_BLOCK_BYTES, 4 << 20)]),
                ("multicast in registers", [(B.HF_PARAM_MULTICAST, 1)]),
                ("multicast off", [(B.HF_PARAM_MULTICAST, 0)])]
    defaults = [(B.HF_PARAM_MULTICAST, B.HF_MULTICAST_AUTO), (B.HF_PARAM_PREFETCH_MERGE, 0), (B.HF_PARAM_PREFETCH_BLOCK_BYTES, 6 << 20),
                (B.HF_PARAM_TILE_BYTES, 131072), (B.HF_PARAM_ROW_INTERLEAVE, 1), (B.HF_PARAM_MC_BLOCK_BYTES, 2 << 20)]

    def timed(ar):
        for _ in range(2):
            ar.execute()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()                                  # Arena launches on torch's current stream
        for _ in range(steps):
            ar.execute()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / steps

    with Plan(cfg["model"], cfg["train"], cfg["gen"], flags=flags, mat_ranks=cfg["mat"]) as plan:
        res = {name: [] for name, _ in variants}
        held, ar = [], None
        for j in range(placements):
            del ar
            torch.cuda.empty_cache()
            held.append(torch.empty((j + 1) * 37 << 20, dtype=torch.uint8, device="cuda"))   # the next allocation gets other pages
            ar = Arena(plan)
            ar.train.fill_(1)
            ar.gen.fill_(2)
            for name, params in variants:
                for k, v in defaults + params:
                    plan.set_param(k, v)
                res[name].append(timed(ar))
        print(f"# {cfg['name']}, {'HF_COPY_OWN' if flags & B.HF_COPY_OWN else 'HF_SKIP_OWN'}: ms per launch (mean of {steps}) on {placements} "
              f"placements of the buffers, the same for every row")
        for name, _ in variants:
            v = res[name]
            print(f"{name:48s} mean {sum(v) / len(v):7.3f} | " + " ".join(f"{x:7.3f}" for x in v))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=2)
    ap.add_argument("--direction", default="fwd", choices=["fwd", "back"])
    ap.add_argument("--flags", default="skip_own", choices=["skip_own", "copy_own"])
    ap.add_argument("--grouping", default="hybridflow", choices=["hybridflow", "vanilla"],
                    help="vanilla = the paper's HybridFlow-V generation grouping (Section 5.3)")
    ap.add_argument("--from-gen", action="store_true",
                    help="HF_GATHER_FROM_GEN: the peers' pieces are read from the owners' generation buffers (Section 5.3: the "
                         "training weights are a sub-part of the generation weights), train_buf is not touched")
    ap.add_argument("--variant", type=int, default=None)
    ap.add_argument("--tile-bytes", type=int, default=None)
    ap.add_argument("--grid", type=int, default=None)
    ap.add_argument("--multicast", type=int, default=None, choices=[0, 1, 2, 3])
    ap.add_argument("--part-bytes", type=int, default=None)
    ap.add_argument("--mc-block-bytes", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the calibration streams after the timed region")
    ap.add_argument("--no-full-refresh", action="store_true", help="skip the HF_COPY_OWN leg after the timed region")
    ap.add_argument("--calib-copy-bytes", type=int, default=0,
                    help="after the timed region, launch the library's plain copy kernel once over this many bytes "
                         "(a dispatch of known traffic, to scale rocprofv3's FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--placement-ab", type=int, default=0, metavar="N",
                    help="instead of the benchmark line: time the transition under alternative launch parameters over the SAME N "
                         "physical placements of the buffers (the buffers are re-allocated N times inside this process), prints a table")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU: all simulated ranks live in one HBM allocation and there is no "
              "multi-GPU path; run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2409_19256_amd import Plan, binding as B
    from paper_2409_19256_amd.arena import Arena
    from seeded_inputs import config_seed

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the reshard library has no CPU path", file=sys.stderr)
        sys.exit(3)
    cfg = dict(CONFIGS[args.config], index=args.config)
    if args.placement_ab:
        placement_ab(cfg, B.HF_COPY_OWN if args.flags == "copy_own" else B.HF_SKIP_OWN, args.placement_ab, args.steps)
        return
    default_config = (args.flags == "skip_own" and not args.from_gen and args.grouping == "hybridflow" and args.variant is None and args.tile_bytes is None
                      and args.grid is None and args.multicast is None and not args.part_bytes and not args.mc_block_bytes)
    flags = B.HF_COPY_OWN if args.flags == "copy_own" else B.HF_SKIP_OWN
    if args.grouping == "vanilla":
        flags |= B.HF_GROUPING_VANILLA
    if args.from_gen:
        flags |= B.HF_GATHER_FROM_GEN
    t0 = time.perf_counter()
    plan = Plan(cfg["model"], cfg["train"], cfg["gen"], flags=flags, mat_ranks=cfg["mat"])
    plan_ms = (time.perf_counter() - t0) * 1e3
    if args.tile_bytes:
        plan.set_param(B.HF_PARAM_TILE_BYTES, args.tile_bytes)
    if args.grid:
        plan.set_param(B.HF_PARAM_GRID_WGS, args.grid)
    if args.variant is not None:
        plan.set_param(B.HF_PARAM_VARIANT, args.variant)
    if args.multicast is not None:
        plan.set_param(B.HF_PARAM_MULTICAST, args.multicast)
    if args.part_bytes:
        plan.set_param(B.HF_PARAM_PART_BYTES, args.part_bytes)
    if args.mc_block_bytes:
        plan.set_param(B.HF_PARAM_MC_BLOCK_BYTES, args.mc_block_bytes)
    ar = Arena(plan)
    ar.gen.zero_()
    ar.fill_train_seeded(config_seed(args.config - 1))
    ar.install_own()                       # own pieces resident before the timed region
    torch.cuda.synchronize()

    direction = B.HF_DIR_TRAIN_TO_GEN if args.direction == "fwd" else B.HF_DIR_GEN_TO_TRAIN
    step = ar.execute if args.direction == "fwd" else ar.back
    W = plan.bytes_moved(direction)                     # bytes written
    R = plan.unique_src_bytes(direction)                # distinct bytes read
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    t0 = time.perf_counter()
    for a, b in ev:                                      # events on the stream the kernel is launched on
        a.record()
        step()
        b.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    kern_ms = sorted(a.elapsed_time(b) for a, b in ev)
    ms_per_step = wall_ms / args.steps
    avg_kernel_ms = sum(kern_ms) / len(kern_ms)

    # algorithmic bytes of one launch: every destination byte is written once; source bytes
    # are read once per destination, or once in all when the kernel multicasts a training
    # piece to every rank that wants it (then the smaller, distinct-bytes figure counts)
    multicast = plan.get_param(B.HF_PARAM_MULTICAST) if args.direction == "fwd" else 0
    alg_bytes = W + (R if multicast else W)
    value = alg_bytes / (ms_per_step * 1e-3) / 1e9
    achieved = alg_bytes / (avg_kernel_ms * 1e-3) / 1e9

    # The transition a caller pays per RLHF iteration when the trainer updates train_buf (and
    # not the own view inside gen_buf): the own pieces must be refreshed too.  One launch of a
    # HF_COPY_OWN plan rewrites every byte of every generation buffer.
    full_refresh = None
    if args.direction == "fwd" and args.flags == "skip_own" and not args.no_full_refresh and not args.from_gen:
        with Plan(cfg["model"], cfg["train"], cfg["gen"], flags=flags | B.HF_COPY_OWN, mat_ranks=cfg["mat"]) as pc:
            for k, v in ((B.HF_PARAM_MULTICAST, args.multicast), (B.HF_PARAM_PART_BYTES, args.part_bytes),
                         (B.HF_PARAM_MC_BLOCK_BYTES, args.mc_block_bytes), (B.HF_PARAM_TILE_BYTES, args.tile_bytes)):
                if v:
                    pc.set_param(k, v)
            st = ar.stream_handle()
            for _ in range(3):
                pc.execute(ar.train_ptr, ar.gen_ptr, st)
            torch.cuda.synchronize()
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(10)]
            for a, b in evs:
                a.record()
                pc.execute(ar.train_ptr, ar.gen_ptr, st)
                b.record()
            torch.cuda.synchronize()
            ms = sum(a.elapsed_time(b) for a, b in evs) / len(evs)
            Wc, Rc = pc.bytes_moved(0), pc.unique_src_bytes(0)
            algc = Wc + (Rc if pc.get_param(B.HF_PARAM_MULTICAST) else Wc)
            full_refresh = {"what": "one hf_reshard_execute of a HF_COPY_OWN plan: own pieces rewritten too (needed when the trainer "
                                    "updates train_buf rather than the own view inside gen_buf)",
                            "ms": round(ms, 4), "bytes_written": Wc, "unique_bytes_read": Rc,
                            "GBps": round(algc / (ms * 1e-3) / 1e9, 1), "frac_of_peak": round(algc / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
    ceilings = None
    if not args.no_ceilings and cfg["name"] != "tiny":
        ceilings = measured_ceilings(ar, max(1, round(W / R)) if multicast else 1, ar.stream_handle())
    if args.calib_copy_bytes:
        n = min(args.calib_copy_bytes, ar.gen.numel()) // 16 * 16
        B.check(B.hf_calib_copy(ar.train_ptr, ar.gen_ptr, min(n, ar.train.numel() * 2 // 16 * 16), ar.stream_handle()), "hf_calib_copy")
        torch.cuda.synchronize()
    traffic, traffic_source = measured_traffic(cfg["name"], args.direction, default_config)
    out = {
        "metric": "reshard GB/s (read+write), train->gen transition" if args.direction == "fwd" else "reshard GB/s (read+write), gen->train",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u16", "data": "synthetic",
        "config": {"workload": cfg["name"], "direction": args.direction, "flags": args.flags, "grouping": args.grouping,
                   "source_of_peer_pieces": "gen_buf (own views)" if args.from_gen else "train_buf",
                   "ranks": plan.n_ranks, "materialised_gen_ranks": len(plan.mat_ranks), "micro_dp": plan.micro_dp_size,
                   "bytes_written": W, "unique_bytes_read": R, "arena_bytes": ar.buf.numel() * 2,
                   "tile_bytes": plan.get_param(B.HF_PARAM_TILE_BYTES), "grid_wgs": plan.get_param(B.HF_PARAM_GRID_WGS),
                   "part_bytes": plan.get_param(B.HF_PARAM_PART_BYTES), "mc_block_bytes": plan.get_param(B.HF_PARAM_MC_BLOCK_BYTES),
                   "prefetch_block_bytes": plan.get_param(B.HF_PARAM_PREFETCH_BLOCK_BYTES),
                   "prefetch_merge": plan.get_param(B.HF_PARAM_PREFETCH_MERGE),
                   "variant": plan.get_param(B.HF_PARAM_VARIANT), "multicast": int(multicast),
                   "unicast_equivalent_GBps": round(2 * W / (avg_kernel_ms * 1e-3) / 1e9, 1),
                   "tiles": plan.num_tiles(direction),
                   "descriptors": plan.num_desc(direction)},
        "transition_ms": {"mean": round(avg_kernel_ms, 4), "median": round(kern_ms[len(kern_ms) // 2], 4), "min": round(kern_ms[0], 4)},
        "pct_hbm_peak": round(100 * achieved / HBM_PEAK_GBS, 2),
        "plan_build_upload_ms": round(plan_ms, 2),
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": traffic, "traffic_source": traffic_source,
                     "kernel": ["reshard_persistent", "reshard_one_tile", "reshard_persistent_lds", "reshard_wave_persistent",
                                "reshard_parts"][plan.get_param(B.HF_PARAM_VARIANT)],
                     "algorithmic_bytes_per_launch": alg_bytes,
                     "avg_kernel_ms": round(avg_kernel_ms, 4),
                     "measured_ceiling": ceilings,
                     "frac_of_measured_mix_ceiling": round(achieved / ceilings["mix_best"], 4) if ceilings else None,
                     "run_to_run": ("the same launch takes 8.3-9.0 ms (0.76-0.81 of peak) from process to process on one box: the "
                                    "physical pages behind the buffers decide it (measured; not address translation)")
                     if default_config and args.config == 2 and args.direction == "fwd" else None},
        "transition_full_refresh": full_refresh,
    }
    if not args.no_cpu_baseline:
        del ar
        torch.cuda.empty_cache()
        out["cpu_baseline"] = cpu_baseline(cfg)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
