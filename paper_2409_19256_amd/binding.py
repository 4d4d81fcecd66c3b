"""ctypes binding of libhfreshard: same names as include/hfreshard.h, argument
marshalling only.  Every step of the reshard runs inside the library's HIP kernels;
there is no Python or CPU fallback: a missing library raises at import of this module.
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhfreshard.so")

# PyTorch wheels carry their own copy of the HIP runtime.  If this library pulled in the
# system's copy first, a later `import torch` would start a second runtime that sees no
# GPU; loading torch first makes both use the same one.  Callers without torch are fine.
try:
    import torch  # noqa: F401
except ImportError:
    pass

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it with `python -m paper_2409_19256_amd.build` "
        "(there is no fallback path)")
_lib = C.CDLL(LIB_PATH)

# ---- constants (mirror the header) ----------------------------------------------------
HF_OK, HF_EINVAL, HF_EDIVIS, HF_ERANGE, HF_ENOMEM, HF_EHIP = 0, -1, -2, -3, -4, -5
HF_SKIP_OWN, HF_COPY_OWN, HF_GROUPING_VANILLA, HF_PLAN_HOST_ONLY, HF_PLAN_OFFLOAD, HF_GATHER_FROM_GEN = 0x0, 0x1, 0x2, 0x4, 0x8, 0x10
(HF_T_EMBED, HF_T_LN1, HF_T_QKV, HF_T_O, HF_T_LN2, HF_T_GATE_UP, HF_T_DOWN, HF_T_LNF, HF_T_HEAD) = range(9)
(HF_G_EMBED, HF_G_LN1, HF_G_Q, HF_G_K, HF_G_V, HF_G_O, HF_G_LN2, HF_G_GATE, HF_G_UP, HF_G_DOWN, HF_G_LNF,
 HF_G_HEAD) = range(16, 28)
HF_COL, HF_ROW, HF_REPL, HF_QKV_DEINT, HF_GATEUP_DEINT = range(5)
HF_DESC_OWN, HF_DESC_ALIGN16, HF_DESC_ALIGN8, HF_DESC_ALIGN4, HF_DESC_ALIGN2 = 0x1, 0x10, 0x20, 0x40, 0x80
HF_DIR_TRAIN_TO_GEN, HF_DIR_GEN_TO_TRAIN, HF_DIR_OFFLOAD, HF_DIR_RELOAD = 0, 1, 2, 3
HF_BUF_TRAIN, HF_BUF_GEN = 0, 1
(HF_PARAM_TILE_BYTES, HF_PARAM_GRID_WGS, HF_PARAM_VARIANT, HF_PARAM_MULTICAST, HF_PARAM_CACHE_POLICY, HF_PARAM_PART_BYTES,
 HF_PARAM_MC_BLOCK_BYTES) = range(7)
HF_PARAM_MAX_WGS_PER_LAUNCH, HF_PARAM_WG_THREADS, HF_PARAM_OFFLOAD_WGS, HF_PARAM_ROW_INTERLEAVE, HF_PARAM_PREFETCH_BLOCK_BYTES = 8, 9, 10, 11, 12
HF_PARAM_PREFETCH_MERGE = 13
HF_MAX_PREFETCH_CHUNKS = 8
HF_MULTICAST_AUTO = -1
HF_MULTICAST_OFF, HF_MULTICAST_REGISTERS, HF_MULTICAST_CACHE_BLOCKED, HF_MULTICAST_PREFETCHED = 0, 1, 2, 3
HF_STATIC_SCRATCH_BYTES = 16 << 20
HF_FANOUT_REGISTERS, HF_FANOUT_CACHE_BLOCKED, HF_FANOUT_PREFETCHED = 0, 1, 2
HF_VARIANT_PERSISTENT, HF_VARIANT_ONE_WG_PER_TILE, HF_VARIANT_LDS_STAGED, HF_VARIANT_WAVE_PERSISTENT, HF_VARIANT_PARTS = 0, 1, 2, 3, 4

TENSOR_NAMES = {
    HF_T_EMBED: "embed", HF_T_LN1: "ln1", HF_T_QKV: "qkv", HF_T_O: "o", HF_T_LN2: "ln2", HF_T_GATE_UP: "gate_up",
    HF_T_DOWN: "down", HF_T_LNF: "lnf", HF_T_HEAD: "head",
    HF_G_EMBED: "embed", HF_G_LN1: "ln1", HF_G_Q: "q", HF_G_K: "k", HF_G_V: "v", HF_G_O: "o", HF_G_LN2: "ln2",
    HF_G_GATE: "gate", HF_G_UP: "up", HF_G_DOWN: "down", HF_G_LNF: "lnf", HF_G_HEAD: "head",
}


class hf_model_desc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim", "ffn", "vocab",
                                        "elem_bytes", "tied_embed")]


class hf_train_layout(C.Structure):
    _fields_ = [("pp", C.c_int32), ("tp", C.c_int32), ("dp", C.c_int32)]


class hf_gen_layout(C.Structure):
    _fields_ = [("pp", C.c_int32), ("tp", C.c_int32), ("flags", C.c_uint32), ("mat_ranks", C.POINTER(C.c_int32)),
                ("n_mat", C.c_int32)]


class hf_desc(C.Structure):
    _fields_ = [("src_rank", C.c_int32), ("dst_rank", C.c_int32), ("tensor_id", C.c_int32), ("layer", C.c_int32),
                ("kind", C.c_uint32), ("flags", C.c_uint32), ("src_off", C.c_uint64), ("dst_off", C.c_uint64),
                ("n_blocks", C.c_uint32), ("rows", C.c_uint32), ("row_bytes", C.c_uint32), ("_pad", C.c_uint32),
                ("src_block_stride", C.c_uint64), ("dst_block_stride", C.c_uint64), ("src_row_stride", C.c_uint64),
                ("dst_row_stride", C.c_uint64)]


class hf_tensor_info(C.Structure):
    _fields_ = [("tensor_id", C.c_int32), ("layer", C.c_int32), ("rows", C.c_uint32), ("cols", C.c_uint32),
                ("offset", C.c_uint64), ("tp_index", C.c_int32), ("replicated", C.c_int32)]


class hf_tile(C.Structure):
    _fields_ = [("src_off", C.c_uint64), ("dst_off", C.c_uint64), ("rows", C.c_uint32), ("row_bytes", C.c_uint32),
                ("src_row_stride", C.c_uint32), ("dst_row_stride", C.c_uint32), ("vec_bytes", C.c_uint32),
                ("n_dst", C.c_uint32), ("dst_list", C.c_uint32), ("_pad", C.c_uint32)]


hf_plan_p = C.c_void_p
_P = hf_plan_p

# name -> (restype, argtypes); every symbol declared in the header
SIGNATURES = {
    "hf_reshard_plan": (C.c_int, [C.POINTER(hf_model_desc), C.POINTER(hf_train_layout), C.POINTER(hf_gen_layout),
                                  C.POINTER(hf_plan_p)]),
    "hf_plan_destroy": (None, [_P]),
    "hf_reshard_execute": (C.c_int, [_P, C.c_void_p, C.c_void_p, C.c_void_p]),
    "hf_reshard_back": (C.c_int, [_P, C.c_void_p, C.c_void_p, C.c_void_p]),
    "hf_reshard_install_own": (C.c_int, [_P, C.c_void_p, C.c_void_p, C.c_void_p]),
    "hf_reshard_execute_static": (C.c_int, [_P, C.c_void_p, C.c_void_p, C.c_void_p]),
    "hf_plan_set_param": (C.c_int, [_P, C.c_int, C.c_int64]),
    "hf_plan_get_param": (C.c_int64, [_P, C.c_int]),
    "hf_plan_train_bytes": (C.c_size_t, [_P]),
    "hf_plan_gen_bytes": (C.c_size_t, [_P]),
    "hf_plan_num_ranks": (C.c_int, [_P]),
    "hf_plan_num_mat": (C.c_int, [_P]),
    "hf_plan_mat_rank": (C.c_int, [_P, C.c_int]),
    "hf_plan_rank_train_offset": (C.c_size_t, [_P, C.c_int]),
    "hf_plan_rank_gen_offset": (C.c_size_t, [_P, C.c_int]),
    "hf_plan_rank_coords": (C.c_int, [_P, C.c_int, C.POINTER(C.c_int32)]),
    "hf_plan_micro_dp_size": (C.c_int, [_P]),
    "hf_plan_num_tensors": (C.c_size_t, [_P, C.c_int, C.c_int]),
    "hf_plan_get_tensor": (C.c_int, [_P, C.c_int, C.c_int, C.c_size_t, C.POINTER(hf_tensor_info)]),
    "hf_plan_num_desc": (C.c_size_t, [_P, C.c_int]),
    "hf_plan_get_desc": (C.c_int, [_P, C.c_int, C.c_size_t, C.POINTER(hf_desc)]),
    "hf_plan_bytes_moved": (C.c_size_t, [_P, C.c_int]),
    "hf_plan_unique_src_bytes": (C.c_size_t, [_P, C.c_int]),
    "hf_plan_num_own_view": (C.c_size_t, [_P, C.c_int]),
    "hf_plan_get_own_view": (C.c_int, [_P, C.c_int, C.c_size_t, C.POINTER(hf_desc)]),
    "hf_plan_num_tiles": (C.c_size_t, [_P, C.c_int]),
    "hf_plan_get_tile": (C.c_int, [_P, C.c_int, C.c_size_t, C.POINTER(hf_tile)]),
    "hf_plan_get_tile_dst": (C.c_int, [_P, C.c_int, C.c_size_t, C.c_uint32, C.POINTER(C.c_uint64)]),
    "hf_gather_responses": (C.c_int, [_P, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "hf_plan_micro_dp_peer": (C.c_int, [_P, C.c_int, C.c_int]),
    "hf_calib_copy": (C.c_int, [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "hf_calib_fanout": (C.c_int, [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int, C.c_size_t, C.c_int, C.c_size_t, C.c_int, C.c_void_p]),
    "hf_offload_remote": (C.c_int, [_P, C.c_void_p, C.c_void_p, C.c_void_p]),
    "hf_reload_remote": (C.c_int, [_P, C.c_void_p, C.c_void_p, C.c_void_p]),
    "hf_plan_remote_bytes": (C.c_size_t, [_P]),
    "hf_plan_remote_rank_offset": (C.c_size_t, [_P, C.c_int]),
    "hf_plan_check_buffers": (C.c_int, [_P, C.c_void_p, C.c_size_t, C.c_void_p, C.c_size_t]),
    "hf_debug_restrict_kinds": (C.c_int, [_P, C.c_int]),
    "hf_plan_validate": (C.c_int, [_P]),
    "hf_last_error": (C.c_char_p, []),
    "hf_version": (C.c_char_p, []),
}

for _name, (_res, _args) in SIGNATURES.items():
    _fn = getattr(_lib, _name)   # AttributeError here = the library does not export it
    _fn.restype = _res
    _fn.argtypes = _args
    globals()[_name] = _fn


class HfError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: status {code}: {hf_last_error().decode()}")  # noqa: F821


def check(code: int, where: str) -> None:
    if code != HF_OK:
        raise HfError(code, where)
