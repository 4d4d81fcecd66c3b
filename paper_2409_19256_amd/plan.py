"""Thin object wrapper over the C ABI: owns an hf_plan* and marshals arguments.  Holds
no resharding logic of its own."""
from __future__ import annotations

import ctypes as C
from typing import List, Optional, Sequence

from . import binding as B


class Plan:
    def __init__(self, model: dict, train: Sequence[int], gen: Sequence[int], flags: int = B.HF_SKIP_OWN,
                 mat_ranks: Optional[Sequence[int]] = None):
        """model: dict with n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab
        train: (p, t, d);  gen: (p_g, t_g);  flags: HF_* plan flags."""
        md = B.hf_model_desc(model["n_layers"], model["hidden"], model["n_q_heads"], model["n_kv_heads"],
                             model["head_dim"], model["ffn"], model["vocab"], model.get("elem_bytes", 2),
                             model.get("tied_embed", 0))
        tl = B.hf_train_layout(*train)
        if mat_ranks is not None:
            arr = (C.c_int32 * len(mat_ranks))(*mat_ranks)
            gl = B.hf_gen_layout(gen[0], gen[1], flags, C.cast(arr, C.POINTER(C.c_int32)), len(mat_ranks))
        else:
            gl = B.hf_gen_layout(gen[0], gen[1], flags, None, 0)
        self._h = B.hf_plan_p()
        B.check(B.hf_reshard_plan(C.byref(md), C.byref(tl), C.byref(gl), C.byref(self._h)), "hf_reshard_plan")
        self.flags = flags

    def close(self):
        if getattr(self, "_h", None):
            B.hf_plan_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:  # interpreter shutdown: the binding module may already be gone
            pass

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.close()

    # ---- execution (device pointers as ints; stream as int, 0 = default stream) -------
    def execute(self, train_ptr: int, gen_ptr: int, stream: int = 0):
        B.check(B.hf_reshard_execute(self._h, train_ptr, gen_ptr, stream), "hf_reshard_execute")

    def execute_static(self, train_ptr: int, gen_ptr: int, stream: int = 0):
        B.check(B.hf_reshard_execute_static(self._h, train_ptr, gen_ptr, stream), "hf_reshard_execute_static")

    def back(self, train_ptr: int, gen_ptr: int, stream: int = 0):
        B.check(B.hf_reshard_back(self._h, train_ptr, gen_ptr, stream), "hf_reshard_back")

    def install_own(self, train_ptr: int, gen_ptr: int, stream: int = 0):
        B.check(B.hf_reshard_install_own(self._h, train_ptr, gen_ptr, stream), "hf_reshard_install_own")

    def offload_remote(self, gen_ptr: int, host_ptr: int, stream: int = 0):
        B.check(B.hf_offload_remote(self._h, gen_ptr, host_ptr, stream), "hf_offload_remote")

    def reload_remote(self, host_ptr: int, gen_ptr: int, stream: int = 0):
        B.check(B.hf_reload_remote(self._h, host_ptr, gen_ptr, stream), "hf_reload_remote")

    def check_buffers(self, train_ptr: int, train_len: int, gen_ptr: int, gen_len: int):
        B.check(B.hf_plan_check_buffers(self._h, train_ptr, train_len, gen_ptr, gen_len), "hf_plan_check_buffers")

    def gather_responses(self, in_ptr: int, out_ptr: int, slot_bytes: int, stream: int = 0):
        B.check(B.hf_gather_responses(self._h, in_ptr, out_ptr, slot_bytes, stream), "hf_gather_responses")

    def micro_dp_peers(self, rank: int) -> List[int]:
        return [B.hf_plan_micro_dp_peer(self._h, rank, j) for j in range(self.micro_dp_size)]

    def set_param(self, param: int, value: int):
        B.check(B.hf_plan_set_param(self._h, param, value), "hf_plan_set_param")

    def get_param(self, param: int) -> int:
        return B.hf_plan_get_param(self._h, param)

    def validate(self):
        B.check(B.hf_plan_validate(self._h), "hf_plan_validate")

    # ---- queries ---------------------------------------------------------------------
    @property
    def train_bytes(self) -> int:
        return B.hf_plan_train_bytes(self._h)

    @property
    def gen_bytes(self) -> int:
        return B.hf_plan_gen_bytes(self._h)

    @property
    def n_ranks(self) -> int:
        return B.hf_plan_num_ranks(self._h)

    @property
    def mat_ranks(self) -> List[int]:
        return [B.hf_plan_mat_rank(self._h, i) for i in range(B.hf_plan_num_mat(self._h))]

    @property
    def micro_dp_size(self) -> int:
        return B.hf_plan_micro_dp_size(self._h)

    def rank_train_offset(self, r: int) -> int:
        return B.hf_plan_rank_train_offset(self._h, r)

    def rank_gen_offset(self, r: int) -> int:
        return B.hf_plan_rank_gen_offset(self._h, r)

    @property
    def remote_bytes(self) -> int:
        return B.hf_plan_remote_bytes(self._h)

    def remote_rank_offset(self, r: int) -> int:
        return B.hf_plan_remote_rank_offset(self._h, r)

    def rank_coords(self, r: int):
        out = (C.c_int32 * 6)()
        B.check(B.hf_plan_rank_coords(self._h, r, out), "hf_plan_rank_coords")
        return tuple(out)

    def tensors(self, which: int, rank: int) -> List[B.hf_tensor_info]:
        res = []
        for i in range(B.hf_plan_num_tensors(self._h, which, rank)):
            t = B.hf_tensor_info()
            B.check(B.hf_plan_get_tensor(self._h, which, rank, i, C.byref(t)), "hf_plan_get_tensor")
            res.append(t)
        return res

    def num_desc(self, direction: int) -> int:
        return B.hf_plan_num_desc(self._h, direction)

    def descs(self, direction: int) -> List[B.hf_desc]:
        res = []
        for i in range(self.num_desc(direction)):
            d = B.hf_desc()
            B.check(B.hf_plan_get_desc(self._h, direction, i, C.byref(d)), "hf_plan_get_desc")
            res.append(d)
        return res

    def own_view(self, rank: int) -> List[B.hf_desc]:
        res = []
        for i in range(B.hf_plan_num_own_view(self._h, rank)):
            d = B.hf_desc()
            B.check(B.hf_plan_get_own_view(self._h, rank, i, C.byref(d)), "hf_plan_get_own_view")
            res.append(d)
        return res

    def num_tiles(self, direction: int) -> int:
        return B.hf_plan_num_tiles(self._h, direction)

    def tiles(self, direction: int):
        """[(hf_tile, [destination offsets])] of the active work list of a direction."""
        res = []
        off = C.c_uint64()
        for i in range(self.num_tiles(direction)):
            t = B.hf_tile()
            B.check(B.hf_plan_get_tile(self._h, direction, i, C.byref(t)), "hf_plan_get_tile")
            dsts = []
            for k in range(t.n_dst):
                B.check(B.hf_plan_get_tile_dst(self._h, direction, i, k, C.byref(off)), "hf_plan_get_tile_dst")
                dsts.append(off.value)
            res.append((t, dsts))
        return res

    def bytes_moved(self, direction: int) -> int:
        return B.hf_plan_bytes_moved(self._h, direction)

    def unique_src_bytes(self, direction: int) -> int:
        return B.hf_plan_unique_src_bytes(self._h, direction)
