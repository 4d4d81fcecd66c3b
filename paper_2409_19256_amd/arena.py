"""Device-memory plumbing for callers that use PyTorch: one HBM allocation that holds
the training shards of all simulated ranks followed by the generation buffers of the
materialised ranks, and a seeded fill of the training shards.  torch is used only to
allocate, to fill and to hand out pointers/streams; all resharding is in the library.
"""
from __future__ import annotations

import torch

from . import binding as B
from .plan import Plan


class Arena:
    """train_buf at byte 0, gen_buf at the next 4096-byte boundary, in one allocation."""

    def __init__(self, plan: Plan, device="cuda:0"):
        if not torch.cuda.is_available():
            raise RuntimeError("no HIP device: the reshard library has no CPU path")
        self.plan = plan
        self.device = torch.device(device)
        self.train_elems = plan.train_bytes // 2
        self.gen_elems = plan.gen_bytes // 2
        self.gen_start = (self.train_elems + 2047) // 2048 * 2048
        self.buf = torch.empty(self.gen_start + self.gen_elems, dtype=torch.int16, device=self.device)
        assert self.buf.data_ptr() % 256 == 0
        self.train = self.buf[: self.train_elems]
        self.gen = self.buf[self.gen_start: self.gen_start + self.gen_elems]

    @property
    def train_ptr(self) -> int:
        return self.train.data_ptr()

    @property
    def gen_ptr(self) -> int:
        return self.gen.data_ptr()

    @staticmethod
    def stream_handle() -> int:
        """hipStream_t of torch's current stream (so torch events time the launches)."""
        return torch.cuda.current_stream().cuda_stream

    def execute(self):
        self.plan.execute(self.train_ptr, self.gen_ptr, self.stream_handle())

    def back(self):
        self.plan.back(self.train_ptr, self.gen_ptr, self.stream_handle())

    def install_own(self):
        self.plan.install_own(self.train_ptr, self.gen_ptr, self.stream_handle())

    def seeded_regions(self):
        """(element offset, n, stream uid) of every training-shard tensor, from the library's
        own tensor tables: TP-sharded tensors get one stream per TP index, replicated norms
        the same stream on every rank, DP replicas identical streams."""
        from seeded_inputs import tensor_uid
        regs = []
        for r in range(self.plan.n_ranks):
            for t in self.plan.tensors(B.HF_BUF_TRAIN, r):
                uid = tensor_uid(B.TENSOR_NAMES[t.tensor_id], max(t.layer, 0), t.tp_index)
                regs.append((t.offset // 2, t.rows * t.cols, uid))
        return regs

    def fill_train_seeded(self, seed: int):
        from seeded_inputs import fill_regions_torch
        fill_regions_torch(self.train, self.seeded_regions(), seed)
