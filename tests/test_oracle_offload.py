"""Pins of the oracle's offload image of the remote pieces (Section 7: the generation copy
of the weights is moved to host memory during training; Section 5.3 / 5.4: the own shard
stays, only the d_g-1 peers' pieces are "remote")."""
import os

import numpy as np
import pytest

from oracle.reshard_oracle import ELEM_BYTES, GenLayout, Model, ReshardOracle, TrainLayout
from tests.cases import BASELINE, MEDIUM, SMALL
from tests.oracle_util import POISON, make_oracle, seeded_train_buf

G = os.path.join(os.path.dirname(__file__), "golden")
CASES = SMALL + [BASELINE[0]]


def _fixture():
    head, spots = {}, []
    for line in open(os.path.join(G, "offload_image_spots.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        left, right = [s.strip() for s in line.split("=", 1)]
        if left[0].isdigit():
            r, off = map(int, left.split())
            kind, layer, lrow, lcol = right.split()
            spots.append((r, off, kind, int(layer), int(lrow), int(lcol)))
        else:
            head[left] = [int(x) for x in right.split()]
    return head, spots


def test_hand_worked_image_offsets():
    head, spots = _fixture()
    orc = ReshardOracle(Model(*head["model"]), TrainLayout(*head["train"]), GenLayout(*head["gen"]))
    ranks = list(range(orc.n_ranks))
    _, rank_offsets, total = orc.remote_layout(ranks)
    assert rank_offsets == head["rank_offsets"] and [total] == head["total"]
    gb = orc.gen_region_offsets(ranks)
    gen = np.arange(gb[-1], dtype=np.int64)            # every element carries its own gen offset
    image = orc.pack_remote(gen, ranks, np.full(total, -1, dtype=np.int64))
    for r, off, kind, layer, lrow, lcol in spots:
        e = orc.gen_entry(r, kind, layer)
        assert image[off] == gb[r] + e.offset + lrow * e.cols + lcol, (r, off, kind)
    assert len(spots) >= 12


@pytest.mark.parametrize("case", SMALL, ids=lambda c: c["name"])
def test_image_against_the_element_definition(case):
    """Brute force: walk every element of every generation tensor in row-major order; it is
    remote iff none of the training locations that hold it (where_train; t copies for the
    norms) lies on the rank itself.  The remote ones, in that order, are the tensor's part."""
    orc = make_oracle(case)
    ranks = list(range(orc.n_ranks))
    gb = orc.gen_region_offsets(ranks)
    holders = {}                                         # gen offset -> ranks holding the source
    for dp in range(orc.d):
        for name, layer in orc.full_tensor_names():
            rows, cols = orc.full_shape(name)
            for row in range(rows):
                for col in range(cols):
                    src_ranks = {q for q, _ in orc.where_train(dp, name, layer, row, col)}
                    for r, off in orc.where_gen(dp, name, layer, row, col):
                        holders[gb[ranks.index(r)] + off] = src_ranks
    parts, rank_offsets, total = orc.remote_layout(ranks)
    gen = np.arange(gb[-1], dtype=np.int64)
    image = orc.pack_remote(gen, ranks, np.full(total, -1, dtype=np.int64))
    off = 0
    for i, r in enumerate(ranks):
        off = -(-off // 2048) * 2048
        assert rank_offsets[i] == off
        for e in orc.gen_table(r)[0]:
            remote = [gb[i] + e.offset + k for k in range(e.n) if r not in holders[gb[i] + e.offset + k]]
            if not remote:
                continue
            off = -(-off // 128) * 128
            assert np.array_equal(image[off:off + len(remote)], remote), (r, e.kind, e.layer)
            off += len(remote)
    assert total == -(-off // 2048) * 2048
    # everything that is not part of a tensor part is untouched
    assert int((image >= 0).sum()) == sum(int(m.sum()) for _, _, _, m in parts)


@pytest.mark.parametrize("case", CASES, ids=lambda c: c["name"])
def test_offload_then_reload_restores_the_remote_pieces_only(case):
    orc = make_oracle(case)
    ranks = list(range(orc.n_ranks))
    train = seeded_train_buf(orc, 77)
    gen = orc.reshard(train, np.full(orc.gen_region_offsets(ranks)[-1], POISON, np.uint16), ranks)
    parts, _, total = orc.remote_layout(ranks)
    image = orc.pack_remote(gen, ranks, np.full(total, 0xABCD, np.uint16))
    # the remote pieces are lost (the buffer is reused during training) ...
    scratch = gen.copy()
    remote = orc.owner_tags(ranks)
    for i, r in enumerate(ranks):
        lo, hi = orc.gen_region_offsets(ranks)[i:i + 2]
        reg = remote[lo:hi]
        scratch[lo:hi][(reg >= 0) & (reg != r)] = 0x0BAD
    assert not np.array_equal(scratch, gen) or all(m.sum() == 0 for *_, m in parts)
    # ... and come back; own pieces and padding were never written
    assert np.array_equal(orc.unpack_remote(image, scratch, ranks), gen)


@pytest.mark.parametrize("case", [BASELINE[0], SMALL[0], SMALL[2], SMALL[3], SMALL[4], MEDIUM[0], MEDIUM[2]], ids=lambda c: c["name"])
def test_image_size_is_the_communication_volume_of_table_2(case):
    """Section 5.4, Table 2: a GPU collects (d_g-1)/(t p) of the model in the transition.  The
    image of a rank holds exactly that many bytes of TP-sharded tensors; with merged pipeline
    stages (outside the table's p = p_g setting) it holds the generation partition
    M_s/(t_g p_g) minus the own shard, plus the norm vectors of the merged peer stages."""
    orc = make_oracle(case)
    ranks = list(range(orc.n_ranks))
    parts, _, _ = orc.remote_layout(ranks)
    norms = ("ln1", "ln2", "lnf")
    sharded_remote = {r: 0 for r in ranks}
    norm_remote = {r: 0 for r in ranks}
    for r, e, _, m in parts:
        (norm_remote if e.kind in norms else sharded_remote)[r] += int(m.sum())
    sharded = orc.model_bytes() - ELEM_BYTES * orc.m.hidden * (2 * orc.m.n_layers + 1)
    for r in ranks:
        if orc.p == orc.pg:
            assert sharded_remote[r] * ELEM_BYTES * orc.t * orc.p == (orc.dg - 1) * sharded
            assert norm_remote[r] == 0
        else:
            gen_sharded = sum(e.n for e in orc.gen_table(r)[0] if e.kind not in norms)
            own_sharded = sum(e.n for e in orc.train_table(r)[0] if e.kind not in norms)
            assert gen_sharded * ELEM_BYTES * orc.tg * orc.pg == sharded
            assert sharded_remote[r] == gen_sharded - own_sharded
            gen_norms = sum(e.n for e in orc.gen_table(r)[0] if e.kind in norms)
            own_norms = sum(e.n for e in orc.train_table(r)[0] if e.kind in norms)
            assert norm_remote[r] == gen_norms - own_norms
