"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle,
bit for bit (the data are opaque 16-bit words: tolerance zero).

Small and medium shapes: whole buffers, element by element, padding included.
BASELINE shapes 2-5 at full size, in the launch configuration bench.py times: EVERY tensor
of EVERY materialised generation rank against the oracle's concat/slice code (streamed
layer by layer from device memory), every byte between the tensors against a canary, the
count of words the kernel leaves alone (own pieces + padding) by a two-canary argument,
and every materialised rank's whole training shard after the reverse path."""
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

from paper_2409_19256_amd import binding as B
from paper_2409_19256_amd.arena import Arena
from seeded_inputs import config_seed, fill_regions_torch, tensor_uid
from oracle.reshard_oracle import GenLayout
from tests.cases import BASELINE, MEDIUM, SMALL
from tests.libcases import make_plan
from tests.oracle_util import POISON, make_oracle, mat_ranks, seeded_train_buf, source_index_map

pytestmark = pytest.mark.gpu

CANARY = 0xC0DE


def _i16(x):  # uint16 pattern -> python int as int16
    return x - 0x10000 if x >= 0x8000 else x


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _payload_mask(orc, ranks, which):
    if which == "gen":
        offs = orc.gen_region_offsets(ranks)
        pay = np.zeros(offs[-1], bool)
        for i, r in enumerate(ranks):
            for e in orc.gen_table(r)[0]:
                pay[offs[i] + e.offset: offs[i] + e.offset + e.n] = True
        return pay
    offs = orc.train_region_offsets()
    pay = np.zeros(offs[-1], bool)
    for r in range(orc.n_ranks):
        for e in orc.train_table(r)[0]:
            pay[offs[r] + e.offset: offs[r] + e.offset + e.n] = True
    return pay


def _own_mask(orc, ranks):
    src = source_index_map(orc, ranks)
    offs, gb = orc.train_region_offsets(), orc.gen_region_offsets(ranks)
    own = np.zeros(src.shape, bool)
    for i, r in enumerate(ranks):
        reg = src[gb[i]:gb[i + 1]]
        own[gb[i]:gb[i + 1]] = (reg >= offs[r]) & (reg < offs[r + 1])
    return own


def _d2h(t):
    return t.cpu().numpy().view(np.uint16)


# (kernel variant, tile bytes, persistent grid or bytes per workgroup, multicast)
VARIANTS = [(B.HF_VARIANT_PERSISTENT, 128 * 1024, 2048, 1), (B.HF_VARIANT_PERSISTENT, 4096, 7, 0),
            (B.HF_VARIANT_ONE_WG_PER_TILE, 64 * 1024, 1, 1), (B.HF_VARIANT_LDS_STAGED, 128 * 1024, 512, 1),
            (B.HF_VARIANT_WAVE_PERSISTENT, 16 * 1024, 1024, 1), (B.HF_VARIANT_WAVE_PERSISTENT, 8192, 3, 0),
            (B.HF_VARIANT_PARTS, 32 * 1024, 4096, 1), (B.HF_VARIANT_PARTS, 128 * 1024, 16384, 0),
            (B.HF_VARIANT_PARTS, 12288, 8192, 1), (B.HF_VARIANT_PARTS, 128 * 1024, 4096, 2),
            (B.HF_VARIANT_PERSISTENT, 64 * 1024, 1024, 2), (B.HF_VARIANT_PARTS, 64 * 1024, -2048, 2),
            (B.HF_VARIANT_PARTS, 16 * 1024, -1024, 1), (B.HF_VARIANT_PARTS, 128 * 1024, -1024, 3),
            (B.HF_VARIANT_PERSISTENT, 32 * 1024, 64, 3), (B.HF_VARIANT_PARTS, 8192, 4096, 3),
            (B.HF_VARIANT_PARTS, 128 * 1024, None, B.HF_MULTICAST_AUTO)]   # last: everything left to the library


def _configure(pl, variant, tile_bytes, grid, multicast):
    pl.set_param(B.HF_PARAM_TILE_BYTES, tile_bytes)
    if grid is None:
        pass                                                      # launch shape chosen by the library
    elif variant == B.HF_VARIANT_PARTS:
        pl.set_param(B.HF_PARAM_PART_BYTES, abs(grid))            # third field = bytes per workgroup,
        pl.set_param(B.HF_PARAM_WG_THREADS, 64 if grid < 0 else 256)   # negative: 64-lane workgroups
    else:
        pl.set_param(B.HF_PARAM_GRID_WGS, grid)
    pl.set_param(B.HF_PARAM_VARIANT, variant)
    pl.set_param(B.HF_PARAM_MULTICAST, B.HF_MULTICAST_REGISTERS)   # leave the automatic choice, then return to it or not
    pl.set_param(B.HF_PARAM_MULTICAST, multicast)
    if multicast in (B.HF_MULTICAST_CACHE_BLOCKED, B.HF_MULTICAST_AUTO):
        pl.set_param(B.HF_PARAM_MC_BLOCK_BYTES, 1 << 20)           # several blocks even at these sizes
    if multicast in (B.HF_MULTICAST_PREFETCHED, B.HF_MULTICAST_AUTO):
        pl.set_param(B.HF_PARAM_PREFETCH_BLOCK_BYTES, 1 << 20)


@pytest.mark.parametrize("case", SMALL + [BASELINE[0]] + MEDIUM, ids=lambda c: c["name"])
def test_whole_buffers_match_oracle(case):
    orc = make_oracle(case)
    ranks = mat_ranks(case, orc)
    seed = config_seed(0) if case["name"] == "tiny" else 1000 + len(case["name"])
    train = seeded_train_buf(orc, seed)
    want = orc.reshard(train, np.full(orc.gen_region_offsets(ranks)[-1], POISON, np.uint16), ranks)
    pay, own = _payload_mask(orc, ranks, "gen"), _own_mask(orc, ranks)
    remote = pay & ~own
    tpay = _payload_mask(orc, ranks, "train")
    for variant, tile_bytes, grid, multicast in VARIANTS:
        _say(f"[case {case['name']} variant {variant} tile {tile_bytes} grid {grid} multicast {multicast}]")
        # --- COPY_OWN: complete generation buffers, padding untouched
        with make_plan(case, B.HF_COPY_OWN) as pl:
            _configure(pl, variant, tile_bytes, grid, multicast)
            ar = Arena(pl)
            ar.train.copy_(torch.from_numpy(train.view(np.int16)))
            ar.gen.fill_(_i16(POISON))
            ar.execute()
            torch.cuda.synchronize()
            assert np.array_equal(_d2h(ar.gen), want)
            assert np.array_equal(_d2h(ar.train), train)          # the source is never written
        # --- SKIP_OWN: only remote pieces written; install_own + execute = complete; reverse
        with make_plan(case, 0) as pl:
            _configure(pl, variant, tile_bytes, grid, multicast)
            assert pl.bytes_moved(0) == 2 * int(remote.sum())
            ar = Arena(pl)
            ar.train.copy_(torch.from_numpy(train.view(np.int16)))
            ar.gen.fill_(_i16(CANARY))
            ar.execute()
            torch.cuda.synchronize()
            got = _d2h(ar.gen)
            assert np.array_equal(got[remote], want[remote])
            assert (got[~remote] == CANARY).all()                  # own pieces and padding never touched
            ar.install_own()
            torch.cuda.synchronize()
            got = _d2h(ar.gen)
            assert np.array_equal(got[pay], want[pay]) and (got[~pay] == CANARY).all()
            ar.train.fill_(_i16(0xBEEF))
            ar.back()
            torch.cuda.synchronize()
            back = _d2h(ar.train)
            assert np.array_equal(back[tpay], train[tpay]) and (back[~tpay] == 0xBEEF).all()


@pytest.mark.parametrize("case", SMALL + [BASELINE[0]] + MEDIUM, ids=lambda c: c["name"])
def test_gather_out_of_the_generation_buffers(case):
    """HF_GATHER_FROM_GEN: every peer's piece is read from that peer's generation buffer.  The
    buffers start with the own pieces only; train_buf is poisoned (and not even passed) to show
    that it is not a source; the result must be the oracle's gather_in_place, which is the
    oracle's reshard of the training shards."""
    orc = make_oracle(case)
    ranks = list(range(orc.n_ranks))
    train = seeded_train_buf(orc, 77)
    complete = orc.reshard(train, np.full(orc.gen_region_offsets(ranks)[-1], CANARY, np.uint16), ranks)
    own = _own_mask(orc, ranks)
    start = np.full(complete.shape, CANARY, np.uint16)
    start[own] = complete[own]
    want = orc.gather_in_place(start.copy(), ranks)
    assert np.array_equal(want, complete)
    for variant, tile_bytes, grid, multicast in [VARIANTS[0], VARIANTS[1], VARIANTS[4], VARIANTS[6], VARIANTS[7], VARIANTS[9], VARIANTS[11], VARIANTS[13], VARIANTS[16]]:
        _say(f"[from-gen {case['name']} variant {variant} tile {tile_bytes} grid {grid} multicast {multicast}]")
        with make_plan(case, B.HF_GATHER_FROM_GEN) as pl:
            _configure(pl, variant, tile_bytes, grid, multicast)
            ar = Arena(pl)
            ar.train.copy_(torch.from_numpy(train.view(np.int16)))
            ar.gen.fill_(_i16(CANARY))
            ar.install_own()                                      # the own pieces, from the training shards, once
            ar.train.fill_(_i16(0xBEEF))                          # from here on train_buf holds nothing
            torch.cuda.synchronize()
            assert np.array_equal(_d2h(ar.gen), start)
            pl.execute(None, ar.gen_ptr, Arena.stream_handle())   # no train_buf at all
            torch.cuda.synchronize()
            assert np.array_equal(_d2h(ar.gen), want)
            ar.gen.copy_(torch.from_numpy(start.view(np.int16)))
            pl.execute_static(None, ar.gen_ptr, Arena.stream_handle())
            torch.cuda.synchronize()
            assert np.array_equal(_d2h(ar.gen), want)
            assert bool((ar.train == _i16(0xBEEF)).all())


def test_subset_of_materialised_ranks_and_stream():
    case = MEDIUM[0]
    orc = make_oracle(case)
    ranks = [9, 0, 14]                                     # arbitrary order, both stages
    train = seeded_train_buf(orc, 5)
    want = orc.reshard(train, np.full(orc.gen_region_offsets(ranks)[-1], POISON, np.uint16), ranks)
    with make_plan(case, B.HF_COPY_OWN, mat=ranks) as pl:
        ar = Arena(pl)
        ar.train.copy_(torch.from_numpy(train.view(np.int16)))
        ar.gen.fill_(_i16(POISON))
        st = torch.cuda.Stream()                           # default priority
        torch.cuda.synchronize()
        with torch.cuda.stream(st):
            ar.execute()                                   # Arena passes torch's current stream
        st.synchronize()
        assert np.array_equal(_d2h(ar.gen), want)
        # reverse only rewrites the materialised ranks' shards
        ar.train.fill_(_i16(0xBEEF))
        ar.back()
        torch.cuda.synchronize()
        back = _d2h(ar.train)
        offs = orc.train_region_offsets()
        for r in range(orc.n_ranks):
            for e in orc.train_table(r)[0]:
                s = slice(offs[r] + e.offset, offs[r] + e.offset + e.n)
                if r in ranks:
                    assert np.array_equal(back[s], train[s])
                else:
                    assert (back[s] == 0xBEEF).all()


def test_one_plan_two_host_threads_two_streams():
    """The execution entry points take a const plan: two host threads run the same plan at the
    same time, each on a stream and on buffers of its own (streams of default priority), and
    both sets of generation buffers equal the oracle after every round."""
    import threading
    case = MEDIUM[0]
    orc = make_oracle(case)
    ranks = list(range(orc.n_ranks))
    trains = [seeded_train_buf(orc, 31), seeded_train_buf(orc, 32)]
    wants = [orc.reshard(t, np.full(orc.gen_region_offsets(ranks)[-1], CANARY, np.uint16), ranks) for t in trains]
    with make_plan(case, B.HF_COPY_OWN) as pl:
        arenas = [Arena(pl), Arena(pl)]
        streams = [torch.cuda.Stream(), torch.cuda.Stream()]
        for ar, t in zip(arenas, trains):
            ar.train.copy_(torch.from_numpy(t.view(np.int16)))
        torch.cuda.synchronize()
        errors = []

        def work(k):
            try:
                for _ in range(20):
                    with torch.cuda.stream(streams[k]):
                        arenas[k].gen.fill_(_i16(CANARY))
                        pl.execute(arenas[k].train_ptr, arenas[k].gen_ptr, streams[k].cuda_stream)
                        pl.back(arenas[k].train_ptr, arenas[k].gen_ptr, streams[k].cuda_stream)
                    streams[k].synchronize()
                    if not np.array_equal(_d2h(arenas[k].gen), wants[k]) or not np.array_equal(_d2h(arenas[k].train), trains[k]):
                        errors.append(k)
                        return
            except Exception as e:                                  # noqa: BLE001 - reported by the main thread
                errors.append(repr(e))

        threads = [threading.Thread(target=work, args=(k,)) for k in range(2)]
        for t in threads:
            t.start()
        for t in threads:
            t.join(timeout=100)
        assert not any(t.is_alive() for t in threads)
        assert errors == []


def test_vanilla_grouping_on_gpu():
    from oracle.reshard_oracle import GenLayout
    case = dict(MEDIUM[1], gen=GenLayout(1, 2, "vanilla"), name="mid_vanilla")
    orc = make_oracle(case)
    ranks = list(range(orc.n_ranks))
    train = seeded_train_buf(orc, 6)
    want = orc.reshard(train, np.full(orc.gen_region_offsets(ranks)[-1], POISON, np.uint16), ranks)
    with make_plan(case, B.HF_COPY_OWN) as pl:
        ar = Arena(pl)
        ar.train.copy_(torch.from_numpy(train.view(np.int16)))
        ar.gen.fill_(_i16(POISON))
        ar.execute()
        torch.cuda.synchronize()
        assert np.array_equal(_d2h(ar.gen), want)
        with pytest.raises(B.HfError):
            ar.back()


def test_cache_policies_and_calibration_copies():
    case = MEDIUM[1]
    orc = make_oracle(case)
    ranks = list(range(orc.n_ranks))
    train = seeded_train_buf(orc, 8)
    want = orc.reshard(train, np.full(orc.gen_region_offsets(ranks)[-1], POISON, np.uint16), ranks)
    with make_plan(case, B.HF_COPY_OWN) as pl:
        ar = Arena(pl)
        ar.train.copy_(torch.from_numpy(train.view(np.int16)))
        for policy in (0, 1, 2, 3, 4, 5):
            pl.set_param(B.HF_PARAM_CACHE_POLICY, policy)
            ar.gen.fill_(_i16(POISON))
            ar.execute()
            torch.cuda.synchronize()
            assert np.array_equal(_d2h(ar.gen), want), policy
        # calibration kernels: copy is exact, read-only leaves the data alone, write-only fills
        n = ar.train.numel() // 8 * 8
        dst = ar.gen[:n]
        st = Arena.stream_handle()
        B.check(B.hf_calib_copy(ar.train.data_ptr(), dst.data_ptr(), 2 * n, st), "copy")
        torch.cuda.synchronize()
        assert torch.equal(dst, ar.train[:n])
        B.check(B.hf_calib_copy(ar.train.data_ptr(), None, 2 * n, st), "read")
        torch.cuda.synchronize()
        assert np.array_equal(_d2h(ar.train), train)
        B.check(B.hf_calib_copy(None, dst.data_ptr(), 2 * n, st), "write")
        torch.cuda.synchronize()
        assert bool((dst == 0x5A5A).all())


def test_work_lists_longer_than_one_grid_are_split_into_launches():
    """A HIP grid holds fewer than 2^32 threads; longer work lists must go out in several
    launches.  Forced here with a tiny per-launch limit on a medium shape."""
    case = MEDIUM[0]
    orc = make_oracle(case)
    ranks = list(range(orc.n_ranks))
    train = seeded_train_buf(orc, 12)
    want = orc.reshard(train, np.full(orc.gen_region_offsets(ranks)[-1], POISON, np.uint16), ranks)
    for variant, mc in [(B.HF_VARIANT_PARTS, 2), (B.HF_VARIANT_PARTS, 0), (B.HF_VARIANT_ONE_WG_PER_TILE, 1)]:
        with make_plan(case, B.HF_COPY_OWN) as pl:
            pl.set_param(B.HF_PARAM_VARIANT, variant)
            pl.set_param(B.HF_PARAM_MULTICAST, mc)
            pl.set_param(B.HF_PARAM_MAX_WGS_PER_LAUNCH, 1024)
            if variant == B.HF_VARIANT_ONE_WG_PER_TILE:
                pl.set_param(B.HF_PARAM_TILE_BYTES, 4096)
            assert pl.num_tiles(0) * (32 if variant == B.HF_VARIANT_PARTS else 1) > 3 * 1024
            ar = Arena(pl)
            ar.train.copy_(torch.from_numpy(train.view(np.int16)))
            ar.gen.fill_(_i16(POISON))
            ar.execute()
            torch.cuda.synchronize()
            assert np.array_equal(_d2h(ar.gen), want)


def test_execute_and_back_can_be_captured_in_a_hip_graph():
    """The entry points only enqueue kernels on the given stream (no allocation, no memset,
    no synchronisation), so a caller may capture them.  Every replay is checked, with eager
    work and synchronisation between replays."""
    case = SMALL[3]
    orc = make_oracle(case)
    ranks = list(range(orc.n_ranks))
    with make_plan(case, B.HF_COPY_OWN) as pl:
        ar = Arena(pl)
        g = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()                       # default priority
        ar.train.zero_()
        ar.gen.zero_()
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            ar.execute()                                 # warm-up outside capture
        side.synchronize()
        with torch.cuda.graph(g, stream=side):
            ar.execute()                                 # Arena passes the capturing stream
        for k in range(4):
            train = seeded_train_buf(orc, 100 + k)
            want = orc.reshard(train, np.full(orc.gen_region_offsets(ranks)[-1], POISON, np.uint16), ranks)
            ar.train.copy_(torch.from_numpy(train.view(np.int16)))
            ar.gen.fill_(_i16(POISON))
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            assert np.array_equal(_d2h(ar.gen), want), f"replay {k}"
            ar.gen.fill_(_i16(POISON))                   # eager launch of the same call in between
            ar.execute()
            torch.cuda.synchronize()
            assert np.array_equal(_d2h(ar.gen), want)


def test_runtime_argument_errors():
    with make_plan(SMALL[0], 0) as pl:
        ar = Arena(pl)
        assert B.hf_reshard_execute(pl._h, ar.train_ptr + 2, ar.gen_ptr, None) == B.HF_EINVAL      # misaligned
        assert B.hf_reshard_execute(pl._h, ar.train_ptr, ar.train_ptr + 256, None) == B.HF_EINVAL  # overlapping
        assert B.hf_reshard_back(pl._h, None, ar.gen_ptr, None) == B.HF_EINVAL


# ------------------------------------------------------------------ full-size configs
POOL_THREADS = 12                       # the GPU machine gives one GPU's share of 16 CPUs


def _oracle_gen_tensors(orc, ranks, train_i16):
    """Streams the oracle's generation partition at full size: yields (rank, entry, expected
    uint16 array [rows, cols]) for EVERY tensor of EVERY rank in `ranks`.  Input of the
    oracle = the training shards as they sit in device memory, fetched one layer at a time
    (peak host memory: the full tensors of one layer), concat/slice on a thread pool."""
    offs = orc.train_region_offsets()
    for r in range(orc.n_ranks):            # fill the oracle's table caches before threads use them
        orc.train_table(r)
        orc.train_entry(r, orc.train_table(r)[0][0].kind, orc.train_table(r)[0][0].layer)
    for r in ranks:
        orc.gen_entry(r, orc.gen_table(r)[0][0].kind, orc.gen_table(r)[0][0].layer)

    def group_of(e):
        return "embed" if e.kind == "embed" else "tail" if e.kind in ("lnf", "head") else e.layer

    with ThreadPoolExecutor(POOL_THREADS) as pool:
        for grp in ["embed"] + list(range(orc.m.n_layers)) + ["tail"]:
            store = {}
            for q in range(orc.n_ranks):
                for e in orc.train_table(q)[0]:
                    if group_of(e) == grp:
                        o = offs[q] + e.offset
                        store[o] = train_i16[o:o + e.n].cpu().numpy().view(np.uint16)

            def fetch(o, n, store=store):
                a = store[o]
                assert a.shape[0] == n
                return a

            work = [(r, e) for r in ranks for e in orc.gen_table(r)[0] if group_of(e) == grp]
            wants = pool.map(lambda re: np.ascontiguousarray(orc.gen_tensor(fetch, re[0], re[1].kind, re[1].layer)), work)
            for (r, e), want in zip(work, wants):
                assert want.shape == (e.rows, e.cols) and want.dtype == np.uint16
                yield r, e, want


def _to_dev(want):
    return torch.from_numpy(want.view(np.int16)).cuda()


def _equal_chunked(a, b, step=1 << 28):
    return all(torch.equal(a[c:c + step], b[c:c + step]) for c in range(0, a.numel(), step))


def _count_untouched(ar, pl, orc, ranks, gb, gend, label):
    """Two-canary count: a word the kernel does not write keeps both canaries.  Under
    SKIP_OWN the kernel must leave alone exactly the own pieces and the padding."""
    first, untouched = {}, {}
    for k, canary in enumerate((0x1357, 0x2468)):
        ar.gen.fill_(_i16(canary))
        ar.execute()
        torch.cuda.synchronize()
        for r in ranks:
            reg = ar.gen[gb[r]:gend[r]]
            if k == 0:
                first[r] = reg == _i16(canary)
            else:                                   # chunked: reductions over 10^10 words need big temporaries
                n, step = 0, 1 << 28
                for c in range(0, reg.numel(), step):
                    n += int(torch.count_nonzero(first[r][c:c + step] & (reg[c:c + step] == _i16(canary))).item())
                untouched[r] = n
    del first
    for r in ranks:
        region = gend[r] - gb[r]
        payload = sum(e.n for e in orc.gen_table(r)[0])
        own = sum(e.n for e in orc.train_table(r)[0])
        assert untouched[r] == region - (payload - own), f"{label} rank {r}: wrong number of untouched words"


def _check_gaps(gen_region, entries, canary, what):
    end = 0
    for e in entries:                               # table order = address order
        assert bool((gen_region[end:e.offset] == _i16(canary)).all()), (what, e.kind, e.layer)
        end = e.offset + e.n
    assert bool((gen_region[end:] == _i16(canary)).all()), what


def _check_reverse(ar, orc, ranks, label):
    """Step 4 at full size: every materialised rank's whole training shard, tensor by
    tensor, against the bytes it held before (the oracle's round-trip identity:
    re-partitioning the generation buffers gives back the training shards), and every
    byte between the tensors against the poison."""
    offs = orc.train_region_offsets()
    saved = {r: ar.train[offs[r]:offs[r + 1]].clone() for r in ranks}
    for r in ranks:
        ar.train[offs[r]:offs[r + 1]].fill_(_i16(0xBEEF))
    ar.back()
    torch.cuda.synchronize()
    for r in ranks:
        now = ar.train[offs[r]:offs[r + 1]]
        end = 0
        for e in orc.train_table(r)[0]:
            assert bool((now[end:e.offset] == _i16(0xBEEF)).all()), (label, r, e.kind, e.layer)
            assert torch.equal(now[e.offset:e.offset + e.n], saved[r][e.offset:e.offset + e.n]), (label, r, e.kind, e.layer)
            end = e.offset + e.n
        assert bool((now[end:] == _i16(0xBEEF)).all())
        now.copy_(saved[r])                         # padding back to what it was
        del saved[r]
    _say(f"[{label}] reverse: all {len(ranks)} training shards whole")


def _check_full_size_streaming(case, cfg_index):
    """Configs 3-5: default launch configuration (what bench.py times), every tensor of every
    materialised rank compared with the oracle while it streams; no cut is made."""
    t0 = time.perf_counter()
    orc = make_oracle(case)
    ranks = mat_ranks(case, orc)
    with make_plan(case, 0) as pl:                         # bench.py's configuration: SKIP_OWN, defaults
        ar = Arena(pl)
        pl.check_buffers(ar.train_ptr, ar.train.numel() * 2, ar.gen_ptr, ar.gen.numel() * 2)
        _say(f"[{case['name']}] arena {ar.buf.numel() * 2 / 1e9:.1f} GB, W = {pl.bytes_moved(0) / 1e9:.2f} GB; filling inputs")
        ar.train.fill_(_i16(POISON))
        fill_regions_torch(ar.train, orc.input_regions(tensor_uid), config_seed(cfg_index))   # regions from the ORACLE's tables
        gb = dict(zip(ranks, orc.gen_region_offsets(ranks)))
        gend = dict(zip(ranks, orc.gen_region_offsets(ranks)[1:]))
        _count_untouched(ar, pl, orc, ranks, gb, gend, case["name"])
        _say(f"[{case['name']}] untouched-word counts ok ({time.perf_counter() - t0:.0f} s); final pass")
        ar.gen.fill_(_i16(CANARY))
        ar.execute()
        ar.install_own()
        torch.cuda.synchronize()
        n = 0
        for r, e, want in _oracle_gen_tensors(orc, ranks, ar.train):
            got = ar.gen[gb[r] + e.offset: gb[r] + e.offset + e.n]
            assert torch.equal(got, _to_dev(want).reshape(-1)), (case["name"], r, e.kind, e.layer)
            n += 1
            if n % 500 == 0:
                _say(f"[{case['name']}] {n} tensors equal the oracle ({time.perf_counter() - t0:.0f} s)")
        assert n == sum(len(orc.gen_table(r)[0]) for r in ranks)
        for r in ranks:
            _check_gaps(ar.gen[gb[r]:gend[r]], orc.gen_table(r)[0], CANARY, (case["name"], r))
        _say(f"[{case['name']}] all {n} generation tensors of {len(ranks)} ranks equal the oracle, padding untouched "
             f"({time.perf_counter() - t0:.0f} s)")
        _check_reverse(ar, orc, ranks, case["name"])
        del ar
    torch.cuda.empty_cache()
    _say(f"[{case['name']}] done in {time.perf_counter() - t0:.0f} s")


def test_llama7b_full_size_every_launch_configuration():
    """Config 2 (the headline workload), whole buffers: the oracle's generation buffers are
    assembled once in device memory (every tensor from the oracle, canaries between them);
    then every launch configuration must reproduce that buffer exactly: bench.py's default
    (SKIP_OWN, prefetched list), multicast off, in registers and cache-blocked, another
    load-only tile size, the persistent-wavefront kernel, the gather out of the generation buffers (HF_GATHER_FROM_GEN) and the HF_COPY_OWN
    plan (one-launch full refresh)."""
    t0 = time.perf_counter()
    case, cfg_index = BASELINE[1], 1
    orc = make_oracle(case)
    ranks = mat_ranks(case, orc)
    gb = dict(zip(ranks, orc.gen_region_offsets(ranks)))
    gend = dict(zip(ranks, orc.gen_region_offsets(ranks)[1:]))
    with make_plan(case, 0) as pl, make_plan(case, B.HF_COPY_OWN) as pl_copy:
        ar = Arena(pl)
        pl.check_buffers(ar.train_ptr, ar.train.numel() * 2, ar.gen_ptr, ar.gen.numel() * 2)
        ar.train.fill_(_i16(POISON))
        fill_regions_torch(ar.train, orc.input_regions(tensor_uid), config_seed(cfg_index))
        ref = torch.full_like(ar.gen, _i16(CANARY))
        n = 0
        for r, e, want in _oracle_gen_tensors(orc, ranks, ar.train):
            ref[gb[r] + e.offset: gb[r] + e.offset + e.n].copy_(_to_dev(want).reshape(-1))
            n += 1
        assert n == sum(len(orc.gen_table(r)[0]) for r in ranks)
        _say(f"[llama7b] oracle buffers of {n} tensors assembled on the device ({time.perf_counter() - t0:.0f} s)")

        configs = [("default", []),
                   ("multicast off", [(B.HF_PARAM_MULTICAST, B.HF_MULTICAST_OFF)]),
                   ("multicast in registers", [(B.HF_PARAM_MULTICAST, B.HF_MULTICAST_REGISTERS)]),
                   ("cache-blocked list", [(B.HF_PARAM_MULTICAST, B.HF_MULTICAST_CACHE_BLOCKED)]),
                   ("prefetched, four copy tiles per load-only tile", [(B.HF_PARAM_MULTICAST, B.HF_MULTICAST_PREFETCHED),
                                                                       (B.HF_PARAM_PREFETCH_MERGE, 4)]),
                   ("persistent wavefronts", [(B.HF_PARAM_MULTICAST, B.HF_MULTICAST_CACHE_BLOCKED),
                                              (B.HF_PARAM_VARIANT, B.HF_VARIANT_WAVE_PERSISTENT), (B.HF_PARAM_TILE_BYTES, 16384)])]
        for label, params in configs:
            for k, v in params:
                pl.set_param(k, v)
            _count_untouched(ar, pl, orc, ranks, gb, gend, label)
            ar.gen.fill_(_i16(CANARY))
            ar.execute()
            ar.install_own()
            torch.cuda.synchronize()
            assert _equal_chunked(ar.gen, ref), label
            _say(f"[llama7b] {label}: whole generation buffers equal the oracle ({time.perf_counter() - t0:.0f} s)")
        pl.set_param(B.HF_PARAM_VARIANT, B.HF_VARIANT_PARTS)
        pl.set_param(B.HF_PARAM_TILE_BYTES, 128 * 1024)
        _check_reverse(ar, orc, ranks, "llama7b")

        # gather out of the generation buffers: own pieces in place, train_buf poisoned and not passed
        with make_plan(case, B.HF_GATHER_FROM_GEN) as pl_gen:
            saved_train = ar.train.clone()
            ar.gen.fill_(_i16(CANARY))
            ar.install_own()
            ar.train.fill_(_i16(0xBEEF))
            pl_gen.execute(None, ar.gen_ptr, Arena.stream_handle())
            torch.cuda.synchronize()
            assert _equal_chunked(ar.gen, ref), "gather from gen"
            ar.train.copy_(saved_train)
            del saved_train
            _say(f"[llama7b] HF_GATHER_FROM_GEN: whole generation buffers equal the oracle ({time.perf_counter() - t0:.0f} s)")

        # one-launch full refresh (HF_COPY_OWN plan on the same buffers)
        ar.gen.fill_(_i16(CANARY))
        pl_copy.execute(ar.train_ptr, ar.gen_ptr, Arena.stream_handle())
        torch.cuda.synchronize()
        assert _equal_chunked(ar.gen, ref), "copy_own"
        _say(f"[llama7b] HF_COPY_OWN: whole generation buffers equal the oracle ({time.perf_counter() - t0:.0f} s)")
        del ref, ar
    torch.cuda.empty_cache()


def test_llama13b_full_size_with_reverse():
    _check_full_size_streaming(BASELINE[2], 2)


def test_llama34b_gqa_full_size():
    _check_full_size_streaming(BASELINE[3], 3)


def test_llama70b_gqa_full_size():
    _check_full_size_streaming(BASELINE[4], 4)


def test_llama34b_one_whole_micro_dp_group_full_size():
    """Config 4's shape with the four ranks of ONE micro-DP group (two TP neighbours x two merged
    stages) instead of four unrelated ranks: every piece then has three destinations on the GPU
    and the multicast work list runs at the 34B GQA shape."""
    _check_full_size_streaming(dict(BASELINE[3], name="llama34b_gqa_group_0_1_8_9", mat=[0, 1, 8, 9]), 3)


def test_llama70b_two_members_of_one_micro_dp_group_full_size():
    """Config 5's shape with two members of one micro-DP group: pieces of the other six members
    have two destinations, the two members' own pieces one (mixed fan-out in one list)."""
    _check_full_size_streaming(dict(BASELINE[4], name="llama70b_gqa_ranks_0_1", mat=[0, 1]), 4)


@pytest.mark.parametrize("t_g", [1, 4])
def test_llama7b_generation_tp_sweep(t_g):
    """Section 8.4 ("Transition and generation time") varies the generation TP size of the 7B
    actor under training layout 1-8-d: t_g = 1 (micro-DP 8: every piece goes to seven peers),
    2 (the headline configuration above), 4 (micro-DP 2: one peer), 8 (nothing to move).
    Full size, default launch configuration, every tensor of every rank against the oracle."""
    case = dict(BASELINE[1], name=f"llama7b_tp8_to_tp{t_g}", gen=GenLayout(1, t_g))
    _check_full_size_streaming(case, 1)


def test_refresh_after_the_training_shards_change():
    """Freshness contract of the header: train_buf and gen_buf are separate memory.  After the
    training shards change, a HF_SKIP_OWN execute refreshes the peers' pieces only (the own
    pieces keep the OLD values until install_own runs); execute + install_own, or one execute
    of a HF_COPY_OWN plan, gives the complete new generation buffers."""
    case = MEDIUM[0]
    orc = make_oracle(case)
    ranks = list(range(orc.n_ranks))
    old, new = seeded_train_buf(orc, 21), seeded_train_buf(orc, 22)
    blank = lambda: np.full(orc.gen_region_offsets(ranks)[-1], CANARY, np.uint16)
    want_old, want_new = orc.reshard(old, blank(), ranks), orc.reshard(new, blank(), ranks)
    own = _own_mask(orc, ranks)
    with make_plan(case, 0) as pl, make_plan(case, B.HF_COPY_OWN) as pl_copy:
        ar = Arena(pl)
        ar.gen.fill_(_i16(CANARY))
        ar.train.copy_(torch.from_numpy(old.view(np.int16)))
        ar.install_own()
        ar.execute()
        torch.cuda.synchronize()
        assert np.array_equal(_d2h(ar.gen), want_old)
        ar.train.copy_(torch.from_numpy(new.view(np.int16)))      # "the actor was updated"
        ar.execute()
        torch.cuda.synchronize()
        got = _d2h(ar.gen)
        assert np.array_equal(got[~own], want_new[~own])          # peers' pieces: new
        assert np.array_equal(got[own], want_old[own])            # own pieces: still the old ones
        ar.install_own()
        torch.cuda.synchronize()
        assert np.array_equal(_d2h(ar.gen), want_new)
        ar.train.copy_(torch.from_numpy(old.view(np.int16)))      # and back, in one launch
        pl_copy.execute(ar.train_ptr, ar.gen_ptr, Arena.stream_handle())
        torch.cuda.synchronize()
        assert np.array_equal(_d2h(ar.gen), want_old)


def test_check_buffers_on_the_device():
    with make_plan(SMALL[0], 0) as pl:
        ar = Arena(pl)
        pl.check_buffers(ar.train_ptr, ar.train.numel() * 2, ar.gen_ptr, ar.gen.numel() * 2)
        host = np.zeros(1 << 16, np.uint8)
        p = (host.ctypes.data + 255) // 256 * 256
        assert B.hf_plan_check_buffers(pl._h, p, pl.train_bytes, ar.gen_ptr, pl.gen_bytes) == B.HF_ERANGE   # not device memory
        small = torch.empty(1024, dtype=torch.int16, device="cuda")
        rc = B.hf_plan_check_buffers(pl._h, ar.train_ptr, pl.train_bytes, small.data_ptr(), pl.gen_bytes)
        assert rc in (B.HF_OK, B.HF_ERANGE)      # torch may carve `small` out of a larger device segment
        assert B.hf_plan_check_buffers(pl._h, ar.train_ptr, pl.train_bytes, small.data_ptr(), 2048) == B.HF_EINVAL


def test_fanout_calibration_kernels_copy_exactly():
    n = 3 * 65536 + 8192                                   # bytes: several blocks and a ragged one
    src = torch.randint(-30000, 30000, (n // 2,), dtype=torch.int16, device="cuda")
    st = Arena.stream_handle()
    R, CB, PF = B.HF_FANOUT_REGISTERS, B.HF_FANOUT_CACHE_BLOCKED, B.HF_FANOUT_PREFETCHED
    for method, block, wg in [(R, 0, 1024), (R, 0, 4096), (R, 0, 8192), (CB, 65536, 1024), (CB, 65536, 4096), (CB, 131072, 8192),
                              (PF, 65536, 1024), (PF, 131072, 4096), (PF, 65536, 8192)]:
        for n_dst in (1, 3):
            stride = n + 256
            dst = torch.full((n_dst * stride // 2,), 77, dtype=torch.int16, device="cuda")
            B.check(B.hf_calib_fanout(src.data_ptr(), dst.data_ptr(), n, n_dst, stride, method, block, wg, st), "fanout")
            torch.cuda.synchronize()
            for j in range(n_dst):
                assert torch.equal(dst[j * stride // 2: j * stride // 2 + n // 2], src), (method, block, wg, n_dst, j)
                assert bool((dst[j * stride // 2 + n // 2: (j + 1) * stride // 2] == 77).all())
    dst = torch.full((n // 2,), 77, dtype=torch.int16, device="cuda")
    B.check(B.hf_calib_fanout(None, dst.data_ptr(), n, 1, n, R, 0, 4096, st), "write only")
    B.check(B.hf_calib_fanout(src.data_ptr(), None, n, 1, n, R, 0, 4096, st), "read only")
    torch.cuda.synchronize()
    assert bool((dst == 0x5A5A).all())
