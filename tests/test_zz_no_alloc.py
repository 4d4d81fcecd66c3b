"""hf_reshard_execute_static, the entry point for callers that cannot allocate device
memory: its output, through the C ABI, against hf_reshard_execute's (and the oracle's), bit
for bit, on two calls in a row, the second with a smaller input."""
import numpy as np
import pytest
import torch

from paper_2409_19256_amd import binding as B
from paper_2409_19256_amd.arena import Arena
from tests.cases import BASELINE, MEDIUM, SMALL
from tests.libcases import make_plan
from tests.oracle_util import make_oracle, seeded_train_buf

CANARY = 0xC0DE


def _i16(x):
    return x - 0x10000 if x >= 0x8000 else x


def test_work_list_beyond_the_static_scratch_is_refused():
    """Size check on the host, before anything touches a device: Llama-13B's cache-blocked
    work list (604 k tiles, 29 MB) does not fit 16 MiB; with 512 KiB tiles it does."""
    with make_plan(BASELINE[2], B.HF_PLAN_HOST_ONLY) as pl:
        pl.set_param(B.HF_PARAM_MULTICAST, B.HF_MULTICAST_CACHE_BLOCKED)
        assert pl.num_tiles(0) * 48 > B.HF_STATIC_SCRATCH_BYTES
        assert B.hf_reshard_execute_static(pl._h, 1 << 20, 1 << 40, None) == B.HF_ERANGE
        assert b"static scratch" in B.hf_last_error()
        assert B.hf_reshard_execute_static(pl._h, None, 1 << 40, None) == B.HF_EINVAL
        assert B.hf_reshard_execute_static(pl._h, (1 << 20) + 2, 1 << 40, None) == B.HF_EINVAL
        pl.set_param(B.HF_PARAM_TILE_BYTES, 512 * 1024)
        assert pl.num_tiles(0) * 48 <= B.HF_STATIC_SCRATCH_BYTES


@pytest.mark.gpu
def test_static_entry_point_matches_execute_on_two_calls_in_a_row():
    st = Arena.stream_handle()
    # first a medium shape in every multicast mode and both flag settings, then smaller shapes:
    # every call after the first finds another plan's work list in the array
    runs = [(MEDIUM[0], B.HF_COPY_OWN, m) for m in (2, 1, 0, 3)] + [(MEDIUM[0], 0, 2), (SMALL[3], B.HF_COPY_OWN, 2),
                                                                 (SMALL[3], 0, 1), (BASELINE[0], 0, 2), (SMALL[6], 0, 2)]
    for case, flags, mode in runs:
        print(f"[static {case['name']} flags {flags} multicast {mode}]", flush=True)
        orc = make_oracle(case)
        ranks = list(range(orc.n_ranks))
        train = seeded_train_buf(orc, 41)
        with make_plan(case, flags) as pl, make_plan(case, flags | B.HF_PLAN_HOST_ONLY) as host_plan:
            pl.set_param(B.HF_PARAM_MULTICAST, mode)
            host_plan.set_param(B.HF_PARAM_MULTICAST, mode)
            ar = Arena(pl)
            ar.train.copy_(torch.from_numpy(train.view(np.int16)))
            ar.gen.fill_(_i16(CANARY))
            ar.execute()                                                 # the existing entry point
            torch.cuda.synchronize()
            want = ar.gen.clone()
            if flags & B.HF_COPY_OWN:
                oracle = orc.reshard(train, np.full(orc.gen_region_offsets(ranks)[-1], CANARY, np.uint16), ranks)
                assert np.array_equal(want.cpu().numpy().view(np.uint16), oracle)
            for plan in (host_plan, pl, pl):                             # a plan without any device memory; twice the same plan
                ar.gen.fill_(_i16(CANARY))
                plan.execute_static(ar.train_ptr, ar.gen_ptr, st)
                torch.cuda.synchronize()
                assert torch.equal(ar.gen, want), (case["name"], flags, mode)
            assert torch.equal(ar.train.cpu(), torch.from_numpy(train.view(np.int16)))
