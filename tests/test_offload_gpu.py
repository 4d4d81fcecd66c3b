"""GPU parity of hf_offload_remote / hf_reload_remote (Section 7: the generation copy of
the weights is kept in host memory while the model trains) against the oracle's image of
the remote pieces, bit for bit, through the C ABI."""
import sys

import numpy as np
import pytest
import torch

from paper_2409_19256_amd import binding as B
from paper_2409_19256_amd.arena import Arena
from seeded_inputs import config_seed, fill_regions_torch, tensor_uid
from tests.cases import BASELINE, MEDIUM, SMALL
from tests.libcases import make_plan
from tests.oracle_util import POISON, make_oracle, seeded_train_buf

pytestmark = pytest.mark.gpu

CANARY = 0xC0DE


def _i16(x):
    return x - 0x10000 if x >= 0x8000 else x


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _pinned(n_elems, fill):
    t = torch.empty(max(n_elems, 1), dtype=torch.int16, pin_memory=True)
    t.fill_(_i16(fill))
    assert t.data_ptr() % 256 == 0
    return t


@pytest.mark.parametrize("case,ranks", [(SMALL[0], None), (SMALL[3], [9, 0, 14]), (SMALL[5], None), (SMALL[6], None),
                                        (BASELINE[0], None), (MEDIUM[0], None), (MEDIUM[1], None), (MEDIUM[2], [3, 17, 30, 12])],
                         ids=lambda v: v["name"] if isinstance(v, dict) else "")
def test_offload_image_and_reload_match_oracle(case, ranks):
    orc = make_oracle(case)
    ranks = list(range(orc.n_ranks)) if ranks is None else ranks
    train = seeded_train_buf(orc, 31)
    gen = orc.reshard(train, np.full(orc.gen_region_offsets(ranks)[-1], CANARY, np.uint16), ranks)
    parts, _, total = orc.remote_layout(ranks)
    want_image = orc.pack_remote(gen, ranks, np.full(max(total, 1), 0xABCD, np.uint16))
    lost = gen.copy()                                   # remote pieces overwritten, as after a training stage
    tags = orc.owner_tags(ranks)
    for i, r in enumerate(ranks):
        lo, hi = orc.gen_region_offsets(ranks)[i:i + 2]
        lost[lo:hi][(tags[lo:hi] >= 0) & (tags[lo:hi] != r)] = POISON
    for tile_bytes, wgs in [(128 * 1024, 8), (4096, 300)]:
        _say(f"[offload {case['name']} tile {tile_bytes} workgroups {wgs}]")
        with make_plan(case, B.HF_PLAN_OFFLOAD, mat=ranks) as pl:
            pl.set_param(B.HF_PARAM_TILE_BYTES, tile_bytes)
            pl.set_param(B.HF_PARAM_OFFLOAD_WGS, wgs)
            assert pl.remote_bytes == 2 * total
            ar = Arena(pl)
            ar.train.copy_(torch.from_numpy(train.view(np.int16)))
            ar.gen.copy_(torch.from_numpy(gen.view(np.int16)))
            host = _pinned(total, 0xABCD)
            st = Arena.stream_handle()
            pl.offload_remote(ar.gen_ptr, host.data_ptr(), st)
            torch.cuda.synchronize()
            assert np.array_equal(host.numpy().view(np.uint16)[:want_image.shape[0]] if total else want_image, want_image)
            assert np.array_equal(ar.gen.cpu().numpy().view(np.uint16), gen)          # the source is left alone
            ar.gen.copy_(torch.from_numpy(lost.view(np.int16)))
            pl.reload_remote(host.data_ptr(), ar.gen_ptr, st)
            torch.cuda.synchronize()
            assert np.array_equal(ar.gen.cpu().numpy().view(np.uint16), gen)          # remote pieces back, nothing else written
            # the gather gives the same bytes as the reload (the remote pieces need not survive)
            ar.gen.copy_(torch.from_numpy(lost.view(np.int16)))
            ar.execute()
            torch.cuda.synchronize()
            assert np.array_equal(ar.gen.cpu().numpy().view(np.uint16), gen)


def test_offload_argument_errors():
    case = SMALL[0]
    with make_plan(case, B.HF_PLAN_OFFLOAD) as pl, make_plan(case, 0) as plain:
        ar = Arena(pl)
        host = _pinned(pl.remote_bytes // 2, 0)
        pageable = np.zeros(pl.remote_bytes + 512, np.uint8)
        p = (pageable.ctypes.data + 255) // 256 * 256
        assert B.hf_offload_remote(pl._h, ar.gen_ptr, p, None) == B.HF_EINVAL            # not pinned
        assert b"pinned" in B.hf_last_error()
        assert B.hf_reload_remote(pl._h, p, ar.gen_ptr, None) == B.HF_EINVAL
        assert B.hf_offload_remote(pl._h, ar.gen_ptr, host.data_ptr() + 2, None) == B.HF_EINVAL   # misaligned
        assert B.hf_offload_remote(plain._h, ar.gen_ptr, host.data_ptr(), None) == B.HF_EINVAL    # plan without the flag
        assert B.hf_offload_remote(pl._h, None, host.data_ptr(), None) == B.HF_EINVAL
        torch.cuda.synchronize()


def test_llama7b_two_ranks_full_size_round_trip_over_the_host_link():
    """Two generation buffers of the headline workload (image of 10 GB, offsets beyond 4 GiB):
    gather, offload, lose the remote pieces, reload: the whole generation buffers must be the
    gathered ones again, canaries between the tensors included."""
    case = BASELINE[1]
    orc = make_oracle(case)
    ranks = [0, 5]
    with make_plan(case, B.HF_PLAN_OFFLOAD, mat=ranks) as pl:
        ar = Arena(pl)
        ar.train.fill_(_i16(POISON))
        fill_regions_torch(ar.train, orc.input_regions(tensor_uid), config_seed(1))
        ar.gen.fill_(_i16(CANARY))
        ar.install_own()
        ar.execute()
        torch.cuda.synchronize()
        ref = ar.gen.clone()
        assert pl.remote_bytes > (1 << 32) and pl.bytes_moved(B.HF_DIR_OFFLOAD) == pl.bytes_moved(0)
        host = _pinned(pl.remote_bytes // 2, 0xABCD)
        _say(f"[offload llama7b ranks {ranks}] image {pl.remote_bytes / 1e9:.2f} GB pinned")
        st = Arena.stream_handle()
        pl.offload_remote(ar.gen_ptr, host.data_ptr(), st)
        torch.cuda.synchronize()
        ar.gen.fill_(_i16(CANARY))                       # everything lost ...
        ar.install_own()                                 # ... except the own pieces, which never left
        pl.reload_remote(host.data_ptr(), ar.gen_ptr, st)
        torch.cuda.synchronize()
        assert torch.equal(ar.gen, ref)
        # one tensor part of the image against the oracle: rank 5's q of layer 17, fed from device memory
        parts_off = pl.remote_rank_offset(5) // 2
        e = orc.gen_entry(5, "q", 17)
        want = orc.gen_tensor(lambda o, n: ar.train[o:o + n].cpu().numpy().view(np.uint16), 5, "q", 17)
        # rank 5 = TP 5 of 8: generation shard 1 = TP 4..7, own piece = second quarter of the rows
        rows = e.rows // 4
        remote = np.concatenate([want[:rows], want[2 * rows:]]).reshape(-1)
        image = host.numpy().view(np.uint16)
        # the part's position: found through the library's own descriptors
        d = next(x for x in pl.descs(B.HF_DIR_OFFLOAD) if x.src_rank == 5 and x.layer == 17 and x.tensor_id == B.HF_G_Q)
        assert d.dst_off // 2 >= parts_off
        assert np.array_equal(image[d.dst_off // 2: d.dst_off // 2 + remote.shape[0]], remote)
        del ref, ar, host
    torch.cuda.empty_cache()
