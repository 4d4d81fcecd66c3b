"""Helpers shared by the oracle tests and the GPU parity tests (test-side only)."""
import numpy as np

from oracle.reshard_oracle import ReshardOracle
from seeded_inputs import fill_regions_numpy, tensor_uid

POISON = 0xDEAD


def make_oracle(case):
    return ReshardOracle(case["model"], case["train"], case["gen"])


def mat_ranks(case, orc):
    m = case.get("mat", "all")
    return list(range(orc.n_ranks)) if m == "all" else list(m)


def seeded_train_buf(orc, seed):
    """Host train_buf (uint16) with every shard tensor filled from the seeded streams."""
    total = orc.train_region_offsets()[-1]
    buf = np.full(total, POISON, dtype=np.uint16)
    fill_regions_numpy(buf, orc.input_regions(tensor_uid), seed)
    return buf


def index_train_buf(orc):
    """train_buf whose items are their own element offsets (to transport indices)."""
    return np.arange(orc.train_region_offsets()[-1], dtype=np.int64)


def source_index_map(orc, ranks):
    """gen_buf-shaped int64 array: train_buf element offset each gen element comes from
    (-1 for padding), obtained by pushing offsets through the oracle's concat/slice code."""
    orc.check_replicas = False
    try:
        gen = np.full(orc.gen_region_offsets(ranks)[-1], -1, dtype=np.int64)
        return orc.reshard(index_train_buf(orc), gen, ranks)
    finally:
        orc.check_replicas = True


def owner_of_train_offset(orc):
    """int32 array over train_buf elements: rank whose region holds the element."""
    offs = orc.train_region_offsets()
    own = np.empty(offs[-1], dtype=np.int32)
    for r in range(orc.n_ranks):
        own[offs[r]:offs[r + 1]] = r
    return own
