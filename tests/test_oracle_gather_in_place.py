"""Pins of the oracle's gather out of the generation buffers (Section 5.3 / 5.4: the training
weights are a sub-part of the generation weights and are used in place, so step 1 collects
every peer's piece from that peer's generation partition)."""
import numpy as np
import pytest

from tests.cases import BASELINE, MEDIUM, SMALL
from tests.oracle_util import POISON, make_oracle, seeded_train_buf

CANARY = 0xC0DE
CASES = [c for c in SMALL + [BASELINE[0], MEDIUM[0], MEDIUM[2]]]


def _only_own_pieces(orc, ranks, complete):
    """Generation buffers in which only the own pieces (and nothing else) are valid."""
    tags = orc.owner_tags(ranks)
    gb = orc.gen_region_offsets(ranks)
    start = np.full(complete.shape, CANARY, np.uint16)
    for i, r in enumerate(ranks):
        own = tags[gb[i]:gb[i + 1]] == r
        start[gb[i]:gb[i + 1]][own] = complete[gb[i]:gb[i + 1]][own]
    return start


@pytest.mark.parametrize("case", CASES, ids=lambda c: c["name"])
def test_gather_from_own_views_equals_gather_from_training_shards(case):
    """Two routes to the same buffers: (a) rebuild from the training shards, (b) place only
    the own pieces, then gather out of the generation buffers.  Padding is left alone."""
    orc = make_oracle(case)
    ranks = list(range(orc.n_ranks))
    train = seeded_train_buf(orc, 55)
    want = orc.reshard(train, np.full(orc.gen_region_offsets(ranks)[-1], CANARY, np.uint16), ranks)
    start = _only_own_pieces(orc, ranks, want)
    if orc.dg > 1:
        assert not np.array_equal(start, want)
    assert np.array_equal(orc.gather_in_place(start, ranks), want)


@pytest.mark.parametrize("case", SMALL[:5], ids=lambda c: c["name"])
def test_gather_in_place_against_the_element_definition(case):
    """Brute force: an element of rank r's buffer takes the value stored at the place where
    the rank that trains it (where_train) keeps it in its own generation buffer (where_gen)."""
    orc = make_oracle(case)
    ranks = list(range(orc.n_ranks))
    gb = orc.gen_region_offsets(ranks)
    start = np.arange(gb[-1], dtype=np.int64)                 # every slot holds its own address
    got = orc.gather_in_place(start.copy(), ranks)
    for dp in range(orc.d):
        for name, layer in orc.full_tensor_names():
            rows, cols = orc.full_shape(name)
            for row in range(rows):
                for col in (0, cols // 2, cols - 1):
                    holders = dict(orc.where_gen(dp, name, layer, row, col))
                    trainers = [q for q, _ in orc.where_train(dp, name, layer, row, col)]
                    for r, off in holders.items():
                        # norms: every TP rank of the stage trains a copy; r takes the one with its own TP index
                        q = trainers[0] if len(trainers) == 1 else next(x for x in trainers if orc.train_coords(x)[2] == orc.train_coords(r)[2])
                        assert got[gb[r] + off] == gb[q] + holders[q], (name, layer, row, col, r)


def test_gather_in_place_needs_the_owners_and_the_hybridflow_grouping():
    from oracle.reshard_oracle import GenLayout, ReshardOracle
    orc = make_oracle(SMALL[0])
    gen = np.zeros(orc.gen_region_offsets([0])[-1], np.uint16)
    with pytest.raises(KeyError):
        orc.gather_in_place(gen, [0])                        # rank 1's buffer is missing
    v = ReshardOracle(SMALL[0]["model"], SMALL[0]["train"], GenLayout(1, 2, "vanilla"))
    with pytest.raises(ValueError):
        v.gather_in_place(np.zeros(v.gen_region_offsets([0, 1, 2, 3])[-1], np.uint16), [0, 1, 2, 3])
