#!/usr/bin/env python3
"""Benchmark of the train->generation weight reshard (HybridFlow Section 5.2 step 1) on
one MI355X.  One "step" = one hf_reshard_execute over all materialised generation
ranks of the workload, inputs resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2] [--direction fwd|back]
                    [--flags skip_own|copy_own] [--variant V] [--tile-bytes B] [--grid G]
                    [--no-cpu-baseline]
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


def measured_traffic(workload, default_config):
    """HBM bytes per launch from the committed rocprofv3 counter summary of this workload (a
    separate profiling run of the same launch configuration); None if there is none or if
    this run does not use the default configuration the counters were taken with."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}.txt")
    if not default_config or not os.path.exists(path):
        return None
    vals = {}
    for line in open(path):
        if "=" in line and not line.startswith("#"):
            k, v = line.split("=")
            vals[k.strip()] = int(v)
    return vals.get("fetch_bytes_per_launch", 0) + vals.get("write_bytes_per_launch", 0) or None


def cpu_baseline(cfg, alg_per_written_byte, seconds_target=15.0):
    """The CPU oracle, as it stands, on a bounded sample of the same workload: whole
    layers of all materialised generation ranks until about `seconds_target` s are spent."""
    import numpy as np

    from oracle.reshard_oracle import GenLayout, Model, ReshardOracle, TrainLayout
    from seeded_inputs import bits16_torch, config_seed, stream_key, tensor_uid

    m = cfg["model"]
    orc = ReshardOracle(Model(m["n_layers"], m["hidden"], m["n_q_heads"], m["n_kv_heads"], m["head_dim"], m["ffn"], m["vocab"]),
                        TrainLayout(*cfg["train"]), GenLayout(*cfg["gen"]))
    ranks = cfg["mat"] if cfg["mat"] is not None else list(range(orc.n_ranks))
    seed = config_seed(cfg["index"] - 1)
    offs = orc.train_region_offsets()
    spent, moved, layers_done = 0.0, 0, 0
    for layer in range(orc.m.n_layers):
        # inputs of this layer for every training rank (not timed)
        store = {}
        for r in range(orc.n_ranks):
            _, pp, tp = orc.train_coords(r)
            if layer // orc.lps != pp:
                continue
            for e in orc.train_table(r)[0]:
                if e.layer == layer:
                    uid = tensor_uid(e.kind, layer, 0 if e.kind in ("ln1", "ln2") else tp)
                    store[offs[r] + e.offset] = bits16_torch(stream_key(seed, uid), 0, e.n).numpy().view(np.uint16)
        fetch = lambda o, n: store[o]
        t0 = time.perf_counter()
        for r in ranks:
            own = {(e.kind, e.layer) for e in orc.train_table(r)[0]}
            for e in orc.gen_table(r)[0]:
                if e.layer != layer:
                    continue
                out = orc.gen_tensor(fetch, r, e.kind, e.layer)
                out = np.ascontiguousarray(out)      # the write into the generation buffer
                # bytes the GPU path moves for this tensor: everything but the own training piece
                own_n = 0
                if layer // orc.lps == orc.train_coords(r)[1]:
                    own_n = e.n // orc.a if e.kind not in ("ln1", "ln2") else e.n
                moved += 2 * (e.n - own_n)
        spent += time.perf_counter() - t0
        layers_done += 1
        if spent >= seconds_target:
            break
    alg = alg_per_written_byte * moved       # same byte accounting as the GPU figure
    return {"value": round(alg / spent / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": f"oracle (rebuild full tensors from all shards, slice) on layers 0..{layers_done - 1} of {orc.m.n_layers} for all "
                      f"{len(ranks)} generation ranks of {cfg['name']}: {moved / 1e9:.2f} GB of remote pieces produced, "
                      f"{alg / 1e9:.2f} GB by the GPU figure's read+write accounting, in {spent:.1f} s; numpy, 1 thread"}


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
    ap.add_argument("--variant", type=int, default=None)
    ap.add_argument("--tile-bytes", type=int, default=None)
    ap.add_argument("--grid", type=int, default=None)
    ap.add_argument("--multicast", type=int, default=None, choices=[0, 1, 2])
    ap.add_argument("--part-bytes", type=int, default=None)
    ap.add_argument("--mc-block-bytes", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calib-copy-bytes", type=int, default=0,
                    help="after the timed region, launch the library's plain copy kernel once over this many bytes "
                         "(a dispatch of known traffic, to scale rocprofv3's FETCH_SIZE / WRITE_SIZE)")
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
    default_config = (args.direction == "fwd" and args.flags == "skip_own" and args.grouping == "hybridflow" and args.variant is None and args.tile_bytes is None
                      and args.grid is None and args.multicast is None and not args.part_bytes and not args.mc_block_bytes)
    flags = B.HF_COPY_OWN if args.flags == "copy_own" else B.HF_SKIP_OWN
    if args.grouping == "vanilla":
        flags |= B.HF_GROUPING_VANILLA
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
    if args.calib_copy_bytes:
        n = min(args.calib_copy_bytes, ar.gen.numel()) // 16 * 16
        B.check(B.hf_calib_copy(ar.train_ptr, ar.gen_ptr, min(n, ar.train.numel() * 2 // 16 * 16), ar.stream_handle()), "hf_calib_copy")
        torch.cuda.synchronize()
        ar.install_own()   # the calibration copy scribbled over gen_buf; nothing after this reads it
        torch.cuda.synchronize()
    value = alg_bytes / (ms_per_step * 1e-3) / 1e9
    achieved = alg_bytes / (avg_kernel_ms * 1e-3) / 1e9
    out = {
        "metric": "reshard GB/s (read+write), train->gen transition" if args.direction == "fwd" else "reshard GB/s (read+write), gen->train",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u16", "data": "synthetic",
        "config": {"workload": cfg["name"], "direction": args.direction, "flags": args.flags, "grouping": args.grouping,
                   "ranks": plan.n_ranks, "materialised_gen_ranks": len(plan.mat_ranks), "micro_dp": plan.micro_dp_size,
                   "bytes_written": W, "unique_bytes_read": R, "arena_bytes": ar.buf.numel() * 2,
                   "tile_bytes": plan.get_param(B.HF_PARAM_TILE_BYTES), "grid_wgs": plan.get_param(B.HF_PARAM_GRID_WGS),
                   "part_bytes": plan.get_param(B.HF_PARAM_PART_BYTES), "mc_block_bytes": plan.get_param(B.HF_PARAM_MC_BLOCK_BYTES),
                   "variant": plan.get_param(B.HF_PARAM_VARIANT), "multicast": int(multicast),
                   "unicast_equivalent_GBps": round(2 * W / (avg_kernel_ms * 1e-3) / 1e9, 1),
                   "tiles": plan.num_tiles(direction),
                   "descriptors": plan.num_desc(direction)},
        "transition_ms": {"mean": round(avg_kernel_ms, 4), "median": round(kern_ms[len(kern_ms) // 2], 4), "min": round(kern_ms[0], 4)},
        "pct_hbm_peak": round(100 * achieved / HBM_PEAK_GBS, 2),
        "plan_build_upload_ms": round(plan_ms, 2),
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": measured_traffic(cfg["name"], default_config),
                     "kernel": ["reshard_persistent", "reshard_one_tile", "reshard_persistent_lds", "reshard_wave_persistent",
                                "reshard_parts"][plan.get_param(B.HF_PARAM_VARIANT)],
                     "algorithmic_bytes_per_launch": alg_bytes,
                     "avg_kernel_ms": round(avg_kernel_ms, 4)},
    }
    if not args.no_cpu_baseline:
        del ar
        torch.cuda.empty_cache()
        out["cpu_baseline"] = cpu_baseline(cfg, alg_bytes / W)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
