"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle,
bit for bit (the data are opaque 16-bit words: tolerance zero).

Small and medium shapes: whole buffers, element by element, padding included.
BASELINE shapes 2-5 at full size, in the launch configuration bench.py times: whole
tensors of sampled (rank, layer) pairs through the oracle's concat/slice code, single
sampled elements through its element definition, and the count of untouched words
(own pieces + padding) by a two-canary argument."""
import sys

import numpy as np
import pytest
import torch

from paper_2409_19256_amd import binding as B
from paper_2409_19256_amd.arena import Arena
from seeded_inputs import config_seed, fill_regions_torch, tensor_uid
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
            (B.HF_VARIANT_PARTS, 16 * 1024, -1024, 1)]


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
            pl.set_param(B.HF_PARAM_TILE_BYTES, tile_bytes)
            if variant == B.HF_VARIANT_PARTS:
                pl.set_param(B.HF_PARAM_PART_BYTES, abs(grid))  # third field = bytes per workgroup,
                pl.set_param(B.HF_PARAM_WG_THREADS, 64 if grid < 0 else 256)  # negative: 64-lane workgroups
            else:
                pl.set_param(B.HF_PARAM_GRID_WGS, grid)
            pl.set_param(B.HF_PARAM_VARIANT, variant)
            pl.set_param(B.HF_PARAM_MULTICAST, multicast)
            if multicast == B.HF_MULTICAST_CACHE_BLOCKED:
                pl.set_param(B.HF_PARAM_MC_BLOCK_BYTES, 1 << 20)   # several blocks even at these sizes
            ar = Arena(pl)
            ar.train.copy_(torch.from_numpy(train.view(np.int16)))
            ar.gen.fill_(_i16(POISON))
            ar.execute()
            torch.cuda.synchronize()
            assert np.array_equal(_d2h(ar.gen), want)
            assert np.array_equal(_d2h(ar.train), train)          # the source is never written
        # --- SKIP_OWN: only remote pieces written; install_own + execute = complete; reverse
        with make_plan(case, 0) as pl:
            pl.set_param(B.HF_PARAM_TILE_BYTES, tile_bytes)
            if variant == B.HF_VARIANT_PARTS:
                pl.set_param(B.HF_PARAM_PART_BYTES, abs(grid))  # third field = bytes per workgroup,
                pl.set_param(B.HF_PARAM_WG_THREADS, 64 if grid < 0 else 256)  # negative: 64-lane workgroups
            else:
                pl.set_param(B.HF_PARAM_GRID_WGS, grid)
            pl.set_param(B.HF_PARAM_VARIANT, variant)
            pl.set_param(B.HF_PARAM_MULTICAST, multicast)
            if multicast == B.HF_MULTICAST_CACHE_BLOCKED:
                pl.set_param(B.HF_PARAM_MC_BLOCK_BYTES, 1 << 20)   # several blocks even at these sizes
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
def _device_fetch(train_i16):
    def fetch(off, n):
        return train_i16[off:off + n].cpu().numpy().view(np.uint16)
    return fetch


def _check_full_size(case, cfg_index, sampled_layers, n_elem_samples=400, check_back=False, params=()):
    orc = make_oracle(case)
    ranks = mat_ranks(case, orc)
    seed = config_seed(cfg_index)
    rng = np.random.default_rng(cfg_index)
    with make_plan(case, 0) as pl:                         # bench.py's configuration: SKIP_OWN, defaults
        for k, v in params:
            pl.set_param(k, v)
        ar = Arena(pl)
        _say(f"[{case['name']}] arena {ar.buf.numel() * 2 / 1e9:.1f} GB, W = {pl.bytes_moved(0) / 1e9:.2f} GB; filling inputs")
        ar.train.fill_(_i16(POISON))
        fill_regions_torch(ar.train, orc.input_regions(tensor_uid), seed)   # regions from the ORACLE's tables
        gb = dict(zip(ranks, orc.gen_region_offsets(ranks)))
        gend = dict(zip(ranks, orc.gen_region_offsets(ranks)[1:]))

        # two-canary count of untouched words: a word untouched in both runs kept both canaries
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
            # the kernel must write exactly the payload that comes from peers
            assert untouched[r] == region - (payload - own), f"rank {r}: wrong number of untouched words"
        _say(f"[{case['name']}] untouched-word counts ok; installing own pieces")
        ar.install_own()
        torch.cuda.synchronize()

        # whole tensors of sampled (rank, layer) pairs through the oracle's concat/slice code
        fetch = _device_fetch(ar.train)
        for r, layer in sampled_layers:
            for e in orc.gen_table(r)[0]:
                if e.layer != layer:
                    continue
                want = orc.gen_tensor(fetch, r, e.kind, e.layer)
                got = ar.gen[gb[r] + e.offset: gb[r] + e.offset + e.n].cpu().numpy().view(np.uint16).reshape(e.rows, e.cols)
                assert np.array_equal(got, want), (r, e.kind, e.layer)
            _say(f"[{case['name']}] rank {r} layer {layer}: all tensors equal the oracle")

        # single elements, one by one, through the element definition
        names = orc.full_tensor_names()
        for _ in range(n_elem_samples):
            name, layer = names[rng.integers(len(names))]
            rows, cols = orc.full_shape(name)
            row, col = int(rng.integers(rows)), int(rng.integers(cols))
            (_, toff), *_ = orc.where_train(0, name, layer, row, col)
            v = int(ar.train[toff].item())
            for r, off in orc.where_gen(0, name, layer, row, col):
                if r in gb:
                    assert int(ar.gen[gb[r] + off].item()) == v, (name, layer, row, col, r)
        _say(f"[{case['name']}] {n_elem_samples} sampled elements ok")

        if check_back:
            offs = orc.train_region_offsets()
            keep = {}
            for r in ranks[:2]:
                keep[r] = ar.train[offs[r]:offs[r + 1]].clone()
            for r in ranks:
                ar.train[offs[r]:offs[r + 1]].fill_(_i16(0xBEEF))
            ar.back()
            torch.cuda.synchronize()
            for r, saved in keep.items():
                now = ar.train[offs[r]:offs[r + 1]]
                end = 0
                for e in orc.train_table(r)[0]:          # tensor by tensor; gaps keep the poison
                    assert bool((now[end:e.offset] == _i16(0xBEEF)).all())
                    assert torch.equal(now[e.offset:e.offset + e.n], saved[e.offset:e.offset + e.n]), (r, e.kind, e.layer)
                    end = e.offset + e.n
                assert bool((now[end:] == _i16(0xBEEF)).all())
            # sampled single elements of the other ranks: shard value must equal the generation value
            for _ in range(200):
                name, layer = names[rng.integers(len(names))]
                rows, cols = orc.full_shape(name)
                row, col = int(rng.integers(rows)), int(rng.integers(cols))
                holders = {r: off for r, off in orc.where_gen(0, name, layer, row, col) if r in gb}
                for tr, toff in orc.where_train(0, name, layer, row, col):
                    if tr in holders:
                        assert int(ar.train[toff].item()) == int(ar.gen[gb[tr] + holders[tr]].item())
            _say(f"[{case['name']}] reverse ok")
        del ar
    torch.cuda.empty_cache()


def test_llama7b_full_size():
    _check_full_size(BASELINE[1], 1, [(0, 0), (5, 17), (7, 31), (3, -1)], check_back=True)


@pytest.mark.parametrize("mode", [B.HF_MULTICAST_OFF, B.HF_MULTICAST_REGISTERS])
def test_llama7b_full_size_other_multicast_modes(mode):
    _check_full_size(BASELINE[1], 1, [(2, 9)], n_elem_samples=200, params=[(B.HF_PARAM_MULTICAST, mode)])


def test_llama7b_full_size_persistent_wavefront_kernel():
    _check_full_size(BASELINE[1], 1, [(6, 30)], n_elem_samples=200,
                     params=[(B.HF_PARAM_VARIANT, B.HF_VARIANT_WAVE_PERSISTENT), (B.HF_PARAM_TILE_BYTES, 16384)])


def test_llama13b_full_size_with_reverse():
    _check_full_size(BASELINE[2], 2, [(0, 0), (6, 20), (7, 39), (1, -1)], check_back=True)


def test_llama34b_gqa_full_size():
    _check_full_size(BASELINE[3], 3, [(0, 0), (4, 24), (6, 47), (2, -1)], check_back=True)


def test_llama70b_gqa_full_size():
    _check_full_size(BASELINE[4], 4, [(0, 0), (31, 79), (0, 40), (31, -1)], n_elem_samples=300, check_back=True)
