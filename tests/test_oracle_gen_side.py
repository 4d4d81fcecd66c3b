"""Pins of the oracle's generation-side arithmetic: the slice rule of the generation
partition (hand-derived fixture, and `full_coords_of_gen` against `where_gen` on every
element of the small shapes) and the vanilla grouping with p_g > 1 (hand-worked groups)."""
import os
import re

import numpy as np
import pytest

from oracle.reshard_oracle import GenLayout, Model, ReshardOracle, TrainLayout
from tests.cases import SMALL
from tests.oracle_util import index_train_buf, make_oracle, owner_of_train_offset, source_index_map

G = os.path.join(os.path.dirname(__file__), "golden")


def _lines(name):
    for line in open(os.path.join(G, name)):
        line = line.strip()
        if line and not line.startswith("#"):
            yield line


def test_hand_derived_generation_layout_spots():
    n = 0
    cache = {}
    for line in _lines("gen_layout_spots.txt"):
        model, train, gen, spot = [s.strip() for s in line.split("|")]
        key = (model, train, gen)
        if key not in cache:
            p, t = map(int, train.split())
            pg, tg = map(int, gen.split())
            orc = ReshardOracle(Model(*map(int, model.split())), TrainLayout(p, t), GenLayout(pg, tg))
            cache[key] = (orc, index_train_buf(orc))
        orc, idx = cache[key]
        f = spot.split()
        rank, kind, layer, lrow, lcol, name, frow, fcol = int(f[0]), f[1], int(f[2]), int(f[3]), int(f[4]), f[6], int(f[7]), int(f[8])
        e = orc.gen_entry(rank, kind, layer)
        assert 0 <= lrow < e.rows and 0 <= lcol < e.cols, line
        # (1) array formulation: the training element that lands at the spot
        orc.check_replicas = False                      # transporting indices: norm copies differ
        got = orc.gen_tensor(lambda o, k: idx[o:o + k], rank, kind, layer)[lrow, lcol]
        orc.check_replicas = True
        assert got in [off for _, off in orc.where_train(0, name, layer, frow, fcol)], line
        # (2) element formulation, both directions
        assert (rank, e.offset + lrow * e.cols + lcol) in orc.where_gen(0, name, layer, frow, fcol), line
        assert orc.full_coords_of_gen(rank, kind, lrow, lcol) == (name, frow, fcol), line
        n += 1
    assert n == 18


@pytest.mark.parametrize("case", SMALL, ids=lambda c: c["name"])
def test_full_coords_of_gen_inverts_where_gen_on_every_element(case):
    """full_coords_of_gen is the generation slice rule read backwards: for every element of
    every generation tensor of every rank, where_gen of the coordinates it returns must name
    that very (rank, offset); and the training location of those coordinates must be the
    element the array formulation delivers there."""
    orc = make_oracle(case)
    ranks = list(range(orc.n_ranks))
    src = source_index_map(orc, ranks)
    gb = orc.gen_region_offsets(ranks)
    for i, r in enumerate(ranks):
        dp = orc.train_coords(r)[0]
        for e in orc.gen_table(r)[0]:
            for lrow in range(e.rows):
                for lcol in (range(e.cols) if lrow in (0, e.rows // 2, e.rows - 1) else (0, e.cols // 3, e.cols - 1)):
                    name, frow, fcol = orc.full_coords_of_gen(r, e.kind, lrow, lcol)
                    off = e.offset + lrow * e.cols + lcol
                    assert (r, off) in orc.where_gen(dp, name, e.layer, frow, fcol)
                    assert src[gb[i] + off] in [o for _, o in orc.where_train(dp, name, e.layer, frow, fcol)]


def _groups(s):
    return sorted(sorted(int(g[1:]) - 1 for g in grp.split(",")) for grp in re.findall(r"\[([^\]]*)\]", s))


def test_vanilla_grouping_with_two_generation_stages():
    g = dict(tuple(s.strip() for s in line.split("=", 1)) for line in _lines("vanilla_pg2_groups.txt"))
    assert g["train p-t-d"] == "2-4-1" and g["gen p_g-t_g-d_g-d"] == "2-2-2-1"
    m = Model(4, 32, 4, 4, 8, 24, 64)
    v = ReshardOracle(m, TrainLayout(2, 4, 1), GenLayout(2, 2, "vanilla"))
    assert v.dg == 2
    assert v.gen_tp_groups() == _groups(g["vanilla_gen_tp_groups"])
    assert v.gen_pp_groups() == _groups(g["vanilla_gen_pp_groups"])
    assert v.micro_dp_groups() == _groups(g["vanilla_micro_dp_groups"])
    # which GPUs find their TP-sharded training weights inside their generation partition
    ranks = list(range(8))
    src, owner, gb = source_index_map(v, ranks), owner_of_train_offset(v), v.gen_region_offsets(ranks)
    overlap = []
    for i, r in enumerate(ranks):
        sharded = np.zeros(gb[i + 1] - gb[i], bool)
        for e in v.gen_table(r)[0]:
            if e.kind not in ("ln1", "ln2", "lnf"):
                sharded[e.offset:e.offset + e.n] = True
        reg = src[gb[i]:gb[i + 1]]
        if (owner[reg[sharded]] == r).any():
            overlap.append(r)
    assert overlap == [int(x[1:]) - 1 for x in g["vanilla_overlap"].split()]
    h = ReshardOracle(m, TrainLayout(2, 4, 1), GenLayout(2, 2, "hybridflow"))
    assert h.gen_tp_groups() == _groups(g["hybridflow_gen_tp_groups"])
    assert h.gen_pp_groups() == _groups(g["hybridflow_gen_pp_groups"])
    assert h.micro_dp_groups() == _groups(g["hybridflow_micro_dp_groups"])
