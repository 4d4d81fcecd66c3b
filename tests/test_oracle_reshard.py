"""Pins of the oracle's reshard (array formulation: concatenate + slice) against
things that do not depend on it: the element-by-element definition, the round trip,
the overlap (zero-redundancy) invariant, Table 2 of the paper, special cases that
reduce to a plain library concatenation, and planted mistakes that must be caught."""
import numpy as np
import pytest

from oracle.reshard_oracle import REPLICATED, GenLayout, Model, ReshardOracle, TrainLayout
from tests.cases import BASELINE, SMALL
from tests.oracle_util import (POISON, make_oracle, owner_of_train_offset, seeded_train_buf, source_index_map)

CASES = SMALL + [BASELINE[0]]
IDS = [c["name"] for c in CASES]


def _gen(orc, train_buf, ranks):
    gen = np.full(orc.gen_region_offsets(ranks)[-1], POISON, dtype=np.uint16)
    return orc.reshard(train_buf, gen, ranks)


def brute_force_check(orc, train_buf, gen_buf, ranks, stride=1):
    """Every `stride`-th element of every full tensor, one by one (pure Python)."""
    gb = dict(zip(ranks, orc.gen_region_offsets(ranks)))
    hits = np.zeros(gen_buf.shape, dtype=np.int32)
    fetch = lambda o, n: train_buf[o:o + n]
    k = 0
    for dp in range(orc.d):
        for name, layer in orc.full_tensor_names():
            full = orc.full_from_train(fetch, dp, name, layer)
            rows, cols = orc.full_shape(name)
            assert full.shape == (rows, cols)
            for row in range(rows):
                for col in range(cols):
                    k += 1
                    if k % stride:
                        continue
                    v = full[row, col]
                    locs = orc.where_train(dp, name, layer, row, col)
                    assert len(locs) == (orc.t if name in REPLICATED else 1)
                    for _, off in locs:
                        assert train_buf[off] == v
                    holders = orc.where_gen(dp, name, layer, row, col)
                    assert len(holders) == (orc.dg * orc.tg if name in REPLICATED else orc.dg)
                    for r, off in holders:
                        if r in gb:
                            assert gen_buf[gb[r] + off] == v, (name, layer, row, col, r)
                            hits[gb[r] + off] += 1
    return hits


@pytest.mark.parametrize("case", CASES, ids=IDS)
def test_array_formulation_equals_element_definition(case):
    orc = make_oracle(case)
    ranks = list(range(orc.n_ranks))
    train = seeded_train_buf(orc, 1234)
    gen = _gen(orc, train, ranks)
    stride = 1 if case["name"] != "tiny" else 7
    hits = brute_force_check(orc, train, gen, ranks, stride)
    if stride == 1:
        # every generation element is defined exactly once; padding is never written
        payload = np.zeros(gen.shape, bool)
        for i, r in enumerate(ranks):
            for e in orc.gen_table(r)[0]:
                s = orc.gen_region_offsets(ranks)[i] + e.offset
                payload[s:s + e.n] = True
        assert (hits[payload] == 1).all() and (hits[~payload] == 0).all()
        assert (gen[~payload] == POISON).all()


@pytest.mark.parametrize("case", CASES, ids=IDS)
def test_round_trip_restores_training_shards(case):
    orc = make_oracle(case)
    ranks = list(range(orc.n_ranks))
    train = seeded_train_buf(orc, 77)
    gen = _gen(orc, train, ranks)
    back = orc.reshard_back(gen, ranks, np.full(train.shape, 0xBEEF, dtype=np.uint16))
    payload = train != POISON  # seeded values can equal POISON by chance; compare both ways
    assert np.array_equal(back[payload], train[payload])
    pad = np.ones(train.shape, bool)
    offs = orc.train_region_offsets()
    for r in ranks:
        for e in orc.train_table(r)[0]:
            pad[offs[r] + e.offset: offs[r] + e.offset + e.n] = False
    assert (back[pad] == 0xBEEF).all() and np.array_equal(back[~pad], train[~pad])


@pytest.mark.parametrize("case", CASES, ids=IDS)
def test_overlap_invariant_own_shard_inside_generation_partition(case):
    """Section 5.3: with the HybridFlow grouping a rank's training weights are reused in
    generation, i.e. every element of its shard appears in its own generation buffer."""
    orc = make_oracle(case)
    ranks = list(range(orc.n_ranks))
    src = source_index_map(orc, ranks)
    gb = orc.gen_region_offsets(ranks)
    offs = orc.train_region_offsets()
    for i, r in enumerate(ranks):
        held = src[gb[i]:gb[i + 1]]
        for e in orc.train_table(r)[0]:
            mine = np.arange(offs[r] + e.offset, offs[r] + e.offset + e.n)
            assert np.isin(mine, held).all(), (r, e.kind, e.layer)


def test_overlap_invariant_fails_under_vanilla_grouping():
    orc = ReshardOracle(Model(2, 32, 4, 4, 8, 24, 64), TrainLayout(1, 4, 2), GenLayout(1, 2, "vanilla"))
    ranks = list(range(orc.n_ranks))
    src = source_index_map(orc, ranks)
    gb, offs = orc.gen_region_offsets(ranks), orc.train_region_offsets()
    missing = []
    for i, r in enumerate(ranks):
        e = orc.train_entry(r, "qkv", 0)
        mine = np.arange(offs[r] + e.offset, offs[r] + e.offset + e.n)
        if not np.isin(mine, src[gb[i]:gb[i + 1]]).all():
            missing.append(r)
    assert missing == [1, 2, 5, 6]  # G2, G3, G6, G7 of Figure 8(a)


def _remote_and_own_elems(orc, sharded_only=True):
    ranks = list(range(orc.n_ranks))
    src = source_index_map(orc, ranks)
    owner = owner_of_train_offset(orc)
    gb = orc.gen_region_offsets(ranks)
    out = []
    for i, r in enumerate(ranks):
        remote = own = 0
        for e in orc.gen_table(r)[0]:
            if sharded_only and e.kind in REPLICATED:
                continue
            s = src[gb[i] + e.offset: gb[i] + e.offset + e.n]
            own += int((owner[s] == r).sum())
            remote += int((owner[s] != r).sum())
        out.append((remote, own))
    return out


@pytest.mark.parametrize("case", [c for c in CASES if c["train"].pp == c["gen"].pp], ids=lambda c: c["name"])
def test_table2_comm_volume_peak_memory_redundancy(case):
    """Table 2 (Section 5.4), HybridFlow column, for the TP-sharded part M_s of the model
    (the closed forms ignore the replicated norm vectors): per-GPU volume (d_g-1)/(tp) M_s
    = (tp - t_g p_g)/(t_g p_g t p) M_s, peak M_s/(t_g p_g), redundancy 0."""
    orc = make_oracle(case)
    Ms = sum(int(np.prod(orc.full_shape(n))) for n, _ in orc.full_tensor_names() if n not in REPLICATED)
    t2 = orc.table2(Ms)["hybridflow"]
    tp = orc.t * orc.p
    assert t2["comm"] == pytest.approx((orc.dg - 1) / tp * Ms)
    per_rank = _remote_and_own_elems(orc)
    if orc.p == 1:
        for remote, own in per_rank:
            assert remote == t2["comm"]
            assert remote + own == t2["peak"]
            assert own == Ms / tp          # whole shard reused -> redundancy 0
    else:
        # stages differ in size (embed / head): the closed form holds for the average GPU
        assert sum(r for r, _ in per_rank) / len(per_rank) == pytest.approx(t2["comm"])
        assert sum(r + o for r, o in per_rank) / len(per_rank) == pytest.approx(t2["peak"])


def test_table2_vanilla_redundancy():
    """HybridFlow-V column: GPUs without overlap must keep their training shard besides the
    generation partition: redundancy M_s/(tp) on exactly those GPUs."""
    orc = ReshardOracle(Model(2, 32, 4, 4, 8, 24, 64), TrainLayout(1, 4, 2), GenLayout(1, 2, "vanilla"))
    Ms = sum(int(np.prod(orc.full_shape(n))) for n, _ in orc.full_tensor_names() if n not in REPLICATED)
    per_rank = _remote_and_own_elems(orc)
    for r, (remote, own) in enumerate(per_rank):
        assert remote + own == Ms // orc.tg
        assert own == (0 if r in (1, 2, 5, 6) else Ms // orc.t)
    assert orc.table2(Ms)["hybridflow_v"]["redundancy"] == Ms / (orc.t * orc.p)
    assert orc.table2(Ms)["hybridflow_v"]["comm"] == pytest.approx((orc.t * orc.p - 1) / (orc.t * orc.p) * Ms)
    assert orc.table2(Ms)["ds_chat"]["comm"] == pytest.approx(7 / 8 * Ms)


# ---------------------------------------------------------------- special cases
def _random_logical_model(orc, seed):
    rng = np.random.default_rng(seed)
    return {(n, l): rng.integers(0, 1 << 16, size=orc.full_shape(n), dtype=np.uint16) for n, l in orc.full_tensor_names()}


def _train_buf_from_logical(orc, logical):
    buf = np.full(orc.train_region_offsets()[-1], POISON, dtype=np.uint16)
    offs = orc.train_region_offsets()
    for r in range(orc.n_ranks):
        for e in orc.train_table(r)[0]:
            val = orc.train_tensor_from_full(lambda name, _l=e.layer: logical[(name, _l)], r, e.kind)
            buf[offs[r] + e.offset: offs[r] + e.offset + e.n] = val.reshape(-1)
    return buf


@pytest.mark.parametrize("case", SMALL, ids=[c["name"] for c in SMALL])
def test_tg1_pg1_generation_buffer_is_the_whole_model(case):
    """t_g = p_g = 1: every rank's generation partition is the full logical model, and
    sharding a known model then gathering it must give that model back (the fuse/slice and
    the concatenate/split code are written separately)."""
    orc = ReshardOracle(case["model"], case["train"], GenLayout(1, 1))
    logical = _random_logical_model(orc, 3)
    train = _train_buf_from_logical(orc, logical)
    ranks = [0, orc.n_ranks - 1]
    gen = _gen(orc, train, ranks)
    gb = orc.gen_region_offsets(ranks)
    gname = orc._GEN_TO_FULL
    for i, r in enumerate(ranks):
        for e in orc.gen_table(r)[0]:
            got = gen[gb[i] + e.offset: gb[i] + e.offset + e.n].reshape(e.rows, e.cols)
            assert np.array_equal(got, logical[(gname[e.kind], e.layer)]), (r, e.kind, e.layer)


def test_one_kv_group_per_rank_fused_qkv_is_plain_concat():
    """n_kv/t = 1: the fused tensor of TP rank i is literally [q-heads of group i; k_i; v_i]."""
    m = Model(1, 16, 8, 4, 4, 12, 8)
    orc = ReshardOracle(m, TrainLayout(1, 4), GenLayout(1, 1))
    logical = _random_logical_model(orc, 4)
    train = _train_buf_from_logical(orc, logical)
    offs = orc.train_region_offsets()
    for tp in range(4):
        e = orc.train_entry(tp, "qkv", 0)
        got = train[offs[tp] + e.offset: offs[tp] + e.offset + e.n].reshape(e.rows, e.cols)
        want = np.concatenate([logical[("wq", 0)][tp * 8:(tp + 1) * 8], logical[("wk", 0)][tp * 4:(tp + 1) * 4],
                               logical[("wv", 0)][tp * 4:(tp + 1) * 4]])
        assert np.array_equal(got, want)


def test_same_layout_means_nothing_is_remote():
    case = [c for c in SMALL if c["name"] == "same_layout"][0]
    orc = make_oracle(case)
    assert orc.dg == 1
    for remote, own in _remote_and_own_elems(orc, sharded_only=False):
        assert remote == 0 and own > 0


def test_reverse_needs_only_the_ranks_own_generation_buffer():
    """Step 4 for rank r uses nothing but r's own generation buffer: corrupting every other
    buffer of its generation TP group does not change the result for r."""
    case = SMALL[0]
    orc = make_oracle(case)
    ranks = list(range(orc.n_ranks))
    train = seeded_train_buf(orc, 5)
    gen = _gen(orc, train, ranks)
    gb = orc.gen_region_offsets(ranks)
    offs = orc.train_region_offsets()
    for r in ranks:
        g2 = np.full(gen.shape, 0x1111, dtype=np.uint16)
        g2[gb[r]:gb[r + 1]] = gen[gb[r]:gb[r + 1]]
        out = orc.reshard_back(g2, ranks, np.zeros(train.shape, np.uint16), ranks=[r])
        for e in orc.train_table(r)[0]:
            s = slice(offs[r] + e.offset, offs[r] + e.offset + e.n)
            assert np.array_equal(out[s], train[s])


# ---------------------------------------------------------------- planted mistakes
class _SwappedKV(ReshardOracle):
    def full_from_train(self, fetch, dp, name, layer, take_tp=0):
        name = {"wk": "wv", "wv": "wk"}.get(name, name)
        return super().full_from_train(fetch, dp, name, layer, take_tp)


class _RowParallelAsColumn(ReshardOracle):
    def gen_tensor(self, fetch, r, kind, layer):
        if kind == "down":
            dp, _, tp = self.train_coords(r)
            full = self.full_from_train(fetch, dp, "wd", layer, take_tp=tp)
            rows, cols = self._gen_shape(kind)
            gtp = self.gen_coords(r)[1]
            return np.ascontiguousarray(full.reshape(-1)[gtp * rows * cols:(gtp + 1) * rows * cols].reshape(rows, cols))
        return super().gen_tensor(fetch, r, kind, layer)


class _WrongMicroGroup(ReshardOracle):
    def gen_coords(self, r):
        gpp, gtp, micro = super().gen_coords(r)
        return gpp, (gtp + 1) % self.tg, micro


@pytest.mark.parametrize("cls", [_SwappedKV, _RowParallelAsColumn, _WrongMicroGroup])
def test_planted_mistakes_are_caught(cls):
    case = SMALL[0]
    orc = cls(case["model"], case["train"], case["gen"])
    ranks = list(range(orc.n_ranks))
    train = seeded_train_buf(orc, 9)
    gen = _gen(orc, train, ranks)
    caught = False
    try:
        if cls is _WrongMicroGroup:
            # the element definition uses the same coordinates: the overlap invariant catches it
            src = source_index_map(orc, ranks)
            gb, offs = orc.gen_region_offsets(ranks), orc.train_region_offsets()
            e = orc.train_entry(0, "qkv", 0)
            assert np.isin(np.arange(offs[0] + e.offset, offs[0] + e.offset + e.n), src[gb[0]:gb[1]]).all()
        else:
            brute_force_check(ReshardOracle(case["model"], case["train"], case["gen"]), train, gen, ranks)
    except AssertionError:
        caught = True
    assert caught
