"""Step 3 of the 3D-HybridEngine workflow (Section 5.2): all-gather of the generation
results inside each micro-DP group.  Oracle pinned to the paper's worked groups; library
group table against the oracle on the host; kernel against the oracle on the GPU."""
import numpy as np
import pytest

from oracle.reshard_oracle import GenLayout, Model, ReshardOracle, TrainLayout
from paper_2409_19256_amd import binding as B
from tests.cases import BASELINE, MEDIUM, SMALL
from tests.libcases import make_plan
from tests.oracle_util import make_oracle

M = Model(2, 32, 4, 4, 8, 24, 64)


def test_oracle_gather_on_the_papers_figure8_groups():
    """Figure 8(b): micro-DP groups [G1,G2] [G3,G4] [G5,G6] [G7,G8] (typed from Section 5.3).
    After the all-gather both members of a group hold [results of the first, results of the second]."""
    o = ReshardOracle(M, TrainLayout(1, 4, 2), GenLayout(1, 2))
    resp = np.arange(8 * 3).reshape(8, 3) + 100           # rank r produced [100+3r, 101+3r, 102+3r]
    out = o.gather_responses(resp)
    assert out.shape == (8, 2, 3)
    for a, b in [(0, 1), (2, 3), (4, 5), (6, 7)]:
        want = np.stack([resp[a], resp[b]])
        assert np.array_equal(out[a], want) and np.array_equal(out[b], want)


def test_oracle_gather_invariants():
    # Figure 7's example (4 GPUs, 1-2-2 -> 1-1-2-2) and a merged-stage layout
    for tl, gl in [(TrainLayout(1, 2, 2), GenLayout(1, 1)), (TrainLayout(2, 4, 1), GenLayout(1, 2)),
                   (TrainLayout(4, 4, 2), GenLayout(2, 2))]:
        o = ReshardOracle(Model(8, 32, 8, 8, 4, 32, 64), tl, gl)
        resp = np.random.default_rng(1).integers(0, 1 << 30, size=(o.n_ranks, 5))
        out = o.gather_responses(resp)
        for g in o.micro_dp_groups():
            assert len(g) == o.dg
            for r in g:                                   # every member ends with the same thing
                assert np.array_equal(out[r], out[g[0]])
            # ... which is exactly the group's results, each once
            assert sorted(map(tuple, out[g[0]])) == sorted(tuple(resp[r]) for r in g)
        # members are ordered by micro-DP index
        for r in range(o.n_ranks):
            assert [o.gen_coords(q)[2] for q in o.micro_dp_members(r)] == list(range(o.dg))


@pytest.mark.parametrize("case", SMALL + MEDIUM + BASELINE, ids=lambda c: c["name"])
def test_library_group_table_matches_oracle(case):
    orc = make_oracle(case)
    with make_plan(case, B.HF_PLAN_HOST_ONLY) as pl:
        for r in range(orc.n_ranks):
            assert pl.micro_dp_peers(r) == orc.micro_dp_members(r)
        assert B.hf_plan_micro_dp_peer(pl._h, 0, orc.dg) == -1 and B.hf_plan_micro_dp_peer(pl._h, -1, 0) == -1
        assert B.hf_gather_responses(pl._h, 256, 1 << 20, 16, None) == B.HF_EINVAL       # host-only plan


@pytest.mark.gpu
@pytest.mark.parametrize("case", [SMALL[0], SMALL[3], SMALL[4], MEDIUM[0], BASELINE[1], BASELINE[4],
                                  dict(SMALL[0], gen=GenLayout(1, 2, "vanilla"), name="vanilla")], ids=lambda c: c["name"])
def test_gather_on_gpu_matches_oracle(case):
    import torch
    orc = make_oracle(case)
    n, dg = orc.n_ranks, orc.dg
    rng = np.random.default_rng(7)
    with make_plan(case, 0, mat=[0]) as pl:               # the response path needs no generation buffers
        for slot_elems in (4, 1, 3, 1000, 64 * 1024 + 4, 7):   # int32 items: 16-byte and 4-byte-only slot sizes
            resp = rng.integers(-2**31, 2**31 - 1, size=(n, slot_elems), dtype=np.int64).astype(np.int32)
            want = orc.gather_responses(resp)
            d_in = torch.from_numpy(resp).cuda()
            d_out = torch.full((n * dg * slot_elems + 64,), 0x5EED, dtype=torch.int32, device="cuda")
            pl.gather_responses(d_in.data_ptr(), d_out.data_ptr(), slot_elems * 4, torch.cuda.current_stream().cuda_stream)
            torch.cuda.synchronize()
            got = d_out.cpu().numpy()
            assert np.array_equal(got[: n * dg * slot_elems].reshape(n, dg, slot_elems), want)
            assert (got[n * dg * slot_elems:] == 0x5EED).all()
            assert np.array_equal(d_in.cpu().numpy(), resp)
        # argument errors
        assert B.hf_gather_responses(pl._h, d_in.data_ptr(), d_out.data_ptr(), 6, None) == B.HF_EINVAL
        assert B.hf_gather_responses(pl._h, d_in.data_ptr(), d_in.data_ptr(), 4, None) == B.HF_EINVAL
        assert B.hf_gather_responses(pl._h, d_in.data_ptr() + 4, d_out.data_ptr(), 4, None) == B.HF_EINVAL
