"""Pins of the oracle's tables and of its training-shard conventions against
hand-written fixtures (tests/golden/*.txt)."""
import os

import numpy as np
import pytest

from oracle.reshard_oracle import GenLayout, Model, ReshardOracle, TrainLayout
from tests.cases import BASELINE
from tests.oracle_util import make_oracle, seeded_train_buf

G = os.path.join(os.path.dirname(__file__), "golden")


def _lines(name):
    for line in open(os.path.join(G, name)):
        line = line.strip()
        if line and not line.startswith("#"):
            yield line


@pytest.mark.parametrize("fixture,orc", [
    ("tiny_layout_offsets.txt", make_oracle(BASELINE[0])),
    ("odd_rows_layout_offsets.txt", ReshardOracle(Model(1, 6, 2, 2, 3, 10, 8), TrainLayout(1, 2), GenLayout(1, 1))),
])
def test_hand_computed_offsets(fixture, orc):
    n = 0
    for line in _lines(fixture):
        f = line.split()
        if f[0] == "train_region":
            assert orc.train_table(0)[1] * 2 == int(f[1])
            assert orc.train_region_offsets()[1] * 2 == int(f[1])
        elif f[0] == "gen_region":
            assert orc.gen_table(0)[1] * 2 == int(f[1])
        else:
            e = (orc.train_entry if f[0] == "train" else orc.gen_entry)(0, f[1], int(f[2]))
            assert e.offset * 2 == int(f[3]), line
        n += 1
    assert n > 15


def test_hand_derived_fused_layout_spots():
    n = 0
    for line in _lines("fused_layout_spots.txt"):
        left, right = line.split("|")
        L, h, nq, nkv, hd, F, V, t = map(int, left.split())
        f = right.split()
        rank, kind, lrow, lcol, name, frow, fcol = int(f[0]), f[1], int(f[2]), int(f[3]), f[5], int(f[6]), int(f[7])
        orc = ReshardOracle(Model(L, h, nq, nkv, hd, F, V), TrainLayout(1, t), GenLayout(1, 1))
        buf = seeded_train_buf(orc, 5)
        layer = -1 if kind in ("embed", "head", "lnf") else 0
        e = orc.train_entry(rank, kind, layer)
        val = buf[orc.train_region_offsets()[rank] + e.offset + lrow * e.cols + lcol]
        # (1) array formulation  (2) element formulation
        full = orc.full_from_train(lambda o, k: buf[o:o + k], 0, name, layer)
        assert full[frow, fcol] == val, line
        (r, off), = orc.where_train(0, name, layer, frow, fcol)
        assert (r, off) == (rank, orc.train_region_offsets()[rank] + e.offset + lrow * e.cols + lcol), line
        n += 1
    assert n == 16


def test_region_sizes_of_baseline_configs():
    # model bytes M = 2 * parameter count; known parameter counts of the shapes
    want_params = {
        "tiny": 2 * 1024 * 256 + 2 * (4 * 256 * 256 + 3 * 688 * 256 + 2 * 256) + 256,
        "llama7b": 6_738_415_616,      # Llama-7B parameter count
        "llama13b": 13_015_864_320,    # Llama-13B parameter count
    }
    for case in BASELINE:
        o = make_oracle(case)
        if case["name"] in want_params:
            assert o.model_bytes() == 2 * want_params[case["name"]]
        # a training shard is M/(p t) plus replicated norms, to within alignment padding
        for r in range(o.n_ranks):
            entries, size = o.train_table(r)
            payload = sum(e.n for e in entries)
            assert 0 <= size - payload < len(entries) * 128 + 2048
        offs = o.train_region_offsets()
        assert all(x % 2048 == 0 for x in offs)


def test_validation_errors():
    m = Model(4, 32, 8, 4, 4, 24, 64)
    for tl, gl in [(TrainLayout(1, 4), GenLayout(1, 3)), (TrainLayout(3, 1), GenLayout(1, 1)),
                   (TrainLayout(1, 8), GenLayout(1, 1)), (TrainLayout(4, 1), GenLayout(3, 1))]:
        with pytest.raises(ValueError):
            ReshardOracle(m, tl, gl)
    with pytest.raises(ValueError):
        ReshardOracle(Model(4, 32, 6, 4, 4, 24, 64), TrainLayout(1, 1), GenLayout(1, 1))
    with pytest.raises(ValueError):
        ReshardOracle(Model(0, 32, 8, 4, 4, 24, 64), TrainLayout(1, 1), GenLayout(1, 1))
