"""Pins of the oracle's parallel-group arithmetic against the paper's worked example
(Section 5.3, Figure 8) and the size identity of Section 5.1."""
import os
import re

import numpy as np
import pytest

from oracle.reshard_oracle import GenLayout, Model, ReshardOracle, TrainLayout
from tests.oracle_util import owner_of_train_offset, source_index_map

GOLD = os.path.join(os.path.dirname(__file__), "golden", "fig8_groups.txt")
M = Model(2, 32, 4, 4, 8, 24, 64)


def _load():
    out = {}
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        k, v = [s.strip() for s in line.split("=", 1)]
        out[k] = v
    return out


def _groups(s):
    return sorted(sorted(int(g[1:]) - 1 for g in grp.split(",")) for grp in re.findall(r"\[([^\]]*)\]", s))


def test_fig8_training_groups():
    g = _load()
    assert g["train p-t-d"] == "1-4-2"
    o = ReshardOracle(M, TrainLayout(1, 4, 2), GenLayout(1, 2))
    assert o.train_tp_groups() == _groups(g["train_tp_groups"])
    assert o.train_dp_groups() == _groups(g["train_dp_groups"])
    assert o.train_pp_groups() == [[r] for r in range(8)]


def test_fig8_hybridflow_generation_groups():
    g = _load()
    o = ReshardOracle(M, TrainLayout(1, 4, 2), GenLayout(1, 2, "hybridflow"))
    assert o.gen_tp_groups() == _groups(g["hybridflow_gen_tp_groups"])
    assert o.micro_dp_groups() == _groups(g["hybridflow_micro_dp_groups"])
    assert o.dg == 2


def _ranks_without_overlap(o):
    ranks = list(range(o.n_ranks))
    src = source_index_map(o, ranks)
    owner = owner_of_train_offset(o)
    gb = o.gen_region_offsets(ranks)
    none = []
    for i, r in enumerate(ranks):
        reg = src[gb[i]:gb[i + 1]]
        # TP-sharded tensors only: norms are replicated everywhere and say nothing
        sharded = np.zeros(reg.shape, bool)
        for e in o.gen_table(r)[0]:
            if e.kind not in ("ln1", "ln2", "lnf"):
                sharded[e.offset:e.offset + e.n] = True
        s = reg[sharded]
        if not (owner[s] == r).any():
            none.append(r)
    return none


def test_fig8_vanilla_has_no_overlap_on_the_papers_gpus():
    g = _load()
    want = sorted(int(x[1:]) - 1 for x in g["vanilla_no_overlap"].split())
    o = ReshardOracle(M, TrainLayout(1, 4, 2), GenLayout(1, 2, "vanilla"))
    assert _ranks_without_overlap(o) == want
    # vanilla groups are the training rule with the smaller sizes: consecutive TP ranks
    assert o.gen_tp_groups() == [[0, 1], [2, 3], [4, 5], [6, 7]]
    o2 = ReshardOracle(M, TrainLayout(1, 4, 2), GenLayout(1, 2, "hybridflow"))
    assert _ranks_without_overlap(o2) == []


def test_fig7_example_four_gpus():
    # Figure 7: 4 GPUs, training 1-2-2, generation 1-1-2-2
    o = ReshardOracle(M, TrainLayout(1, 2, 2), GenLayout(1, 1))
    assert o.dg == 2
    assert o.micro_dp_groups() == [[0, 1], [2, 3]]
    assert o.gen_tp_groups() == [[0], [1], [2], [3]]
    assert o.train_dp_groups() == [[0, 2], [1, 3]]


@pytest.mark.parametrize("p,t,d,pg,tg", [(1, 4, 2, 1, 2), (2, 4, 1, 1, 2), (4, 8, 1, 1, 4), (4, 4, 2, 2, 2), (2, 2, 3, 2, 1)])
@pytest.mark.parametrize("grouping", ["hybridflow", "vanilla"])
def test_size_identity_and_group_shapes(p, t, d, pg, tg, grouping):
    # Section 5.1: N_a = p t d = p_g t_g d_g d
    m = Model(8, 32, 8, 8, 4, 32, 64)
    o = ReshardOracle(m, TrainLayout(p, t, d), GenLayout(pg, tg, grouping))
    assert o.n_ranks == p * t * d == pg * tg * o.dg * d
    for groups, size in [(o.train_tp_groups(), t), (o.train_pp_groups(), p), (o.train_dp_groups(), d),
                         (o.gen_tp_groups(), tg), (o.gen_pp_groups(), pg), (o.micro_dp_groups(), o.dg)]:
        assert all(len(g) == size for g in groups)
        assert sorted(r for g in groups for r in g) == list(range(o.n_ranks))
    if grouping == "hybridflow":
        a, b = t // tg, p // pg
        for g in o.gen_tp_groups():          # stride t/t_g
            assert all(y - x == a for x, y in zip(g, g[1:]))
        for g in o.gen_pp_groups():          # stride (p/p_g) stages = (p/p_g)*t ranks
            assert all(y - x == b * t for x, y in zip(g, g[1:]))
        for g in o.train_dp_groups():        # stride p*t
            assert all(y - x == p * t for x, y in zip(g, g[1:]))
