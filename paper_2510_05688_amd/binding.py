"""ctypes binding of libvatt (include/vatt.h): argument marshalling only.

Every step of the decode path runs inside the HIP library; PyTorch is used here
for device memory and streams.  The functions carry the names of the C entry
points.  Importing this module loads the in-tree libvatt.so and fails loudly if
it has not been built (python -m paper_2510_05688_amd.build).
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libvatt.so")

VATT_OK = 0
VATT_E_INVALID_ARG = -1
VATT_E_UNSUPPORTED_SHAPE = -2
VATT_E_WORKSPACE_TOO_SMALL = -3
VATT_E_HIP = -4
VATT_E_NO_DEVICE = -5
VATT_TARGET_D, VATT_TARGET_N, VATT_TARGET_SDPA = 0, 1, 2
VATT_LAYOUT_CONTIGUOUS, VATT_LAYOUT_PAGED = 0, 1
VATT_WS_SCORES = 0
VATT_WS_DEBUG = 1
VATT_OPT_SAMPLER_SMALL_BATCHES = 1
VATT_OPT_SAMPLER_DRAW_CAP = 2
VATT_OPT_TOPK_GENERAL_PATH = 3
VATT_OPT_BUDGET_BOUND = 4
VATT_OPT_NESTED_SAMPLES = 5
VATT_OPT_HEAD_THREADS = 6
VATT_OPT_BUDGET_MULTIPLE = 7
VATT_OPT_SCORE_ORDER = 8
VATT_OPT_FUSED_GATHER = 9
VATT_OPT_SCORE_PREWORK = 10
VATT_OPT_ASCENDING_SAMPLES = 12
VATT_OPT_CACHE_SLOTS = 13
VATT_OPT_GIVEN_SPLITS = 14
VATT_OPT_SPARSE_SPLITS = 15
VATT_OPT_GIVEN_FUSED = 16
VATT_BOUND_CLT = 0
VATT_BOUND_HOEFFDING = 1
VATT_BOUND_HOEFFDING_RANGE = 2

EXPORTS = [
    "vatt_plan_create", "vatt_plan_create_chunk", "vatt_plan_query_len", "vatt_plan_destroy", "vatt_plan_set_option", "vatt_plan_workspace_bytes",
    "vatt_plan_workspace_offset", "vatt_plan_score_stride", "vatt_plan_index_capacity",
    "vatt_plan_index_segment", "vatt_decode", "vatt_decode_static", "vatt_static_scratch_bytes", "vatt_decode_given_topk", "vatt_dense_decode", "vatt_score", "vatt_append_kv", "vatt_stream_read", "vatt_row_read",
    "vatt_random_cache_bytes", "vatt_random_cache_slots", "vatt_random_cache_fill", "vatt_append_kv_cached",
    "vatt_decode_given_topk_cached", "vatt_random_cache_read",
    "vatt_host_kv_device_pointer", "vatt_status_string",
]


class vatt_params(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("n_max", ctypes.c_int32), ("kv_layout", ctypes.c_int32),
        ("page_size", ctypes.c_int32), ("num_blocks", ctypes.c_int32), ("sink", ctypes.c_int32),
        ("window", ctypes.c_int32), ("topk_abs", ctypes.c_int32), ("topk_frac", ctypes.c_float),
        ("base_abs", ctypes.c_int32), ("base_frac", ctypes.c_float), ("epsilon", ctypes.c_float),
        ("delta", ctypes.c_float), ("target", ctypes.c_int32), ("sm_scale", ctypes.c_float),
        ("budget_cap_frac", ctypes.c_float),
    ]


class VattError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s (%d)" % (where, vatt_status_string(status), status))


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            "libvatt.so is not built: run `python -m paper_2510_05688_amd.build` (needs hipcc). "
            "There is no fallback path.")
    lib = ctypes.CDLL(LIB_PATH)
    vp, sz, i32, i64 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32, ctypes.c_int64
    lib.vatt_plan_create.argtypes = [ctypes.POINTER(vatt_params), ctypes.c_int, ctypes.POINTER(vp)]
    lib.vatt_plan_create.restype = ctypes.c_int
    lib.vatt_plan_create_chunk.argtypes = [ctypes.POINTER(vatt_params), ctypes.c_int, ctypes.c_int,
                                           ctypes.POINTER(vp)]
    lib.vatt_plan_create_chunk.restype = ctypes.c_int
    lib.vatt_plan_query_len.argtypes = [vp]
    lib.vatt_plan_query_len.restype = ctypes.c_int
    lib.vatt_plan_destroy.argtypes = [vp]
    lib.vatt_plan_destroy.restype = None
    lib.vatt_plan_set_option.argtypes = [vp, ctypes.c_int, ctypes.c_int]
    lib.vatt_plan_set_option.restype = ctypes.c_int
    lib.vatt_plan_workspace_bytes.argtypes = [vp]
    lib.vatt_plan_workspace_bytes.restype = sz
    lib.vatt_plan_workspace_offset.argtypes = [vp, ctypes.c_int]
    lib.vatt_plan_workspace_offset.restype = sz
    lib.vatt_plan_score_stride.argtypes = [vp]
    lib.vatt_plan_score_stride.restype = sz
    lib.vatt_plan_index_capacity.argtypes = [vp]
    lib.vatt_plan_index_capacity.restype = sz
    lib.vatt_plan_index_segment.argtypes = [vp, ctypes.c_int]
    lib.vatt_plan_index_segment.restype = i64
    lib.vatt_decode.argtypes = [vp] * 8 + [sz] + [vp] * 7
    lib.vatt_decode.restype = ctypes.c_int
    lib.vatt_decode_static.argtypes = [vp] * 14
    lib.vatt_decode_static.restype = ctypes.c_int
    lib.vatt_static_scratch_bytes.argtypes = []
    lib.vatt_static_scratch_bytes.restype = sz
    lib.vatt_decode_given_topk.argtypes = [vp] * 10 + [sz] + [vp] * 7
    lib.vatt_decode_given_topk.restype = ctypes.c_int
    lib.vatt_dense_decode.argtypes = [vp] * 7 + [sz] + [vp] * 3
    lib.vatt_dense_decode.restype = ctypes.c_int
    lib.vatt_score.argtypes = [vp] * 6 + [sz, vp]
    lib.vatt_score.restype = ctypes.c_int
    lib.vatt_append_kv.argtypes = [vp] * 8
    lib.vatt_append_kv.restype = ctypes.c_int
    lib.vatt_host_kv_device_pointer.argtypes = [vp, ctypes.POINTER(vp)]
    lib.vatt_host_kv_device_pointer.restype = ctypes.c_int
    lib.vatt_stream_read.argtypes = [vp, sz, vp, vp]
    lib.vatt_row_read.argtypes = [vp, sz, vp, sz, vp, vp]
    lib.vatt_row_read.restype = ctypes.c_int
    lib.vatt_stream_read.restype = ctypes.c_int
    lib.vatt_random_cache_bytes.argtypes = [vp]
    lib.vatt_random_cache_bytes.restype = sz
    lib.vatt_random_cache_slots.argtypes = [vp]
    lib.vatt_random_cache_slots.restype = ctypes.c_int
    lib.vatt_random_cache_fill.argtypes = [vp] * 8
    lib.vatt_random_cache_fill.restype = ctypes.c_int
    lib.vatt_append_kv_cached.argtypes = [vp] * 10
    lib.vatt_append_kv_cached.restype = ctypes.c_int
    lib.vatt_decode_given_topk_cached.argtypes = [vp] * 11 + [sz] + [vp] * 7
    lib.vatt_decode_given_topk_cached.restype = ctypes.c_int
    lib.vatt_random_cache_read.argtypes = [vp] * 5
    lib.vatt_random_cache_read.restype = ctypes.c_int
    lib.vatt_status_string.argtypes = [ctypes.c_int]
    lib.vatt_status_string.restype = ctypes.c_char_p
    return lib


_lib = _load()


def _ptr(x) -> Optional[int]:
    """Device/host address of a tensor-like (anything with data_ptr()), an int, or None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return int(x.data_ptr())


def _nbytes(x) -> int:
    return int(x.numel() * x.element_size())


def make_params(d: Dict) -> vatt_params:
    p = vatt_params()
    for name, _ in vatt_params._fields_:
        if name in d:
            setattr(p, name, d[name])
    return p


def vatt_status_string(status: int) -> str:
    return _lib.vatt_status_string(int(status)).decode()


def vatt_plan_create(params, device: int) -> int:
    """Returns an opaque plan handle (int).  `params` is a vatt_params or a dict of its fields."""
    if isinstance(params, dict):
        params = make_params(params)
    out = ctypes.c_void_p()
    rc = _lib.vatt_plan_create(ctypes.byref(params), int(device), ctypes.byref(out))
    if rc != VATT_OK:
        raise VattError(rc, "vatt_plan_create")
    return out.value


def vatt_plan_create_chunk(params, q_len: int, device: int) -> int:
    """A plan for steps with q_len query tokens per sequence; otherwise as vatt_plan_create."""
    if isinstance(params, dict):
        params = make_params(params)
    out = ctypes.c_void_p()
    rc = _lib.vatt_plan_create_chunk(ctypes.byref(params), int(q_len), int(device), ctypes.byref(out))
    if rc != VATT_OK:
        raise VattError(rc, "vatt_plan_create_chunk")
    return out.value


def vatt_plan_query_len(plan: int) -> int:
    return int(_lib.vatt_plan_query_len(plan))


def vatt_plan_destroy(plan: int) -> None:
    _lib.vatt_plan_destroy(plan)


def vatt_plan_set_option(plan: int, option: int, value: int) -> None:
    rc = _lib.vatt_plan_set_option(plan, option, value)
    if rc != VATT_OK:
        raise VattError(rc, "vatt_plan_set_option")


def vatt_plan_workspace_bytes(plan: int) -> int:
    return int(_lib.vatt_plan_workspace_bytes(plan))


def vatt_plan_workspace_offset(plan: int, region: int) -> int:
    return int(_lib.vatt_plan_workspace_offset(plan, region))


def vatt_plan_score_stride(plan: int) -> int:
    return int(_lib.vatt_plan_score_stride(plan))


def vatt_plan_index_capacity(plan: int) -> int:
    return int(_lib.vatt_plan_index_capacity(plan))


def vatt_plan_index_segment(plan: int, segment: int) -> int:
    return int(_lib.vatt_plan_index_segment(plan, segment))


def vatt_decode(plan, q, k, v, block_table, seq_lens, seq_seeds, workspace, out_o, out_lse, out_idx,
                out_counts, out_budget_raw, out_stats, stream=None) -> None:
    rc = _lib.vatt_decode(plan, _ptr(q), _ptr(k), _ptr(v), _ptr(block_table), _ptr(seq_lens), _ptr(seq_seeds),
                          _ptr(workspace), _nbytes(workspace), _ptr(out_o), _ptr(out_lse), _ptr(out_idx),
                          _ptr(out_counts), _ptr(out_budget_raw), _ptr(out_stats), _ptr(stream))
    if rc != VATT_OK:
        raise VattError(rc, "vatt_decode")


def vatt_static_scratch_bytes() -> int:
    return int(_lib.vatt_static_scratch_bytes())


def vatt_decode_static(plan, q, k, v, block_table, seq_lens, seq_seeds, out_o, out_lse, out_idx, out_counts,
                       out_budget_raw, out_stats, stream=None) -> None:
    """vatt_decode on the library's own scratch array (no workspace argument, nothing allocated)."""
    rc = _lib.vatt_decode_static(plan, _ptr(q), _ptr(k), _ptr(v), _ptr(block_table), _ptr(seq_lens),
                                 _ptr(seq_seeds), _ptr(out_o), _ptr(out_lse), _ptr(out_idx), _ptr(out_counts),
                                 _ptr(out_budget_raw), _ptr(out_stats), _ptr(stream))
    if rc != VATT_OK:
        raise VattError(rc, "vatt_decode_static")


def vatt_decode_given_topk(plan, q, k, v, block_table, seq_lens, seq_seeds, topk_idx, topk_cnt, workspace, out_o,
                           out_lse, out_idx, out_counts, out_budget_raw, out_stats, stream=None) -> None:
    rc = _lib.vatt_decode_given_topk(plan, _ptr(q), _ptr(k), _ptr(v), _ptr(block_table), _ptr(seq_lens),
                                     _ptr(seq_seeds), _ptr(topk_idx), _ptr(topk_cnt), _ptr(workspace),
                                     _nbytes(workspace), _ptr(out_o), _ptr(out_lse), _ptr(out_idx),
                                     _ptr(out_counts), _ptr(out_budget_raw), _ptr(out_stats), _ptr(stream))
    if rc != VATT_OK:
        raise VattError(rc, "vatt_decode_given_topk")


def vatt_dense_decode(plan, q, k, v, block_table, seq_lens, workspace, out_o, out_lse, stream=None) -> None:
    rc = _lib.vatt_dense_decode(plan, _ptr(q), _ptr(k), _ptr(v), _ptr(block_table), _ptr(seq_lens),
                                _ptr(workspace), _nbytes(workspace), _ptr(out_o), _ptr(out_lse), _ptr(stream))
    if rc != VATT_OK:
        raise VattError(rc, "vatt_dense_decode")


def vatt_score(plan, q, k, block_table, seq_lens, workspace, stream=None) -> None:
    rc = _lib.vatt_score(plan, _ptr(q), _ptr(k), _ptr(block_table), _ptr(seq_lens), _ptr(workspace),
                         _nbytes(workspace), _ptr(stream))
    if rc != VATT_OK:
        raise VattError(rc, "vatt_score")


def vatt_append_kv(plan, k_new, v_new, k, v, block_table, seq_lens, stream=None) -> None:
    rc = _lib.vatt_append_kv(plan, _ptr(k_new), _ptr(v_new), _ptr(k), _ptr(v), _ptr(block_table),
                             _ptr(seq_lens), _ptr(stream))
    if rc != VATT_OK:
        raise VattError(rc, "vatt_append_kv")


def vatt_random_cache_bytes(plan) -> int:
    return int(_lib.vatt_random_cache_bytes(plan))


def vatt_random_cache_slots(plan) -> int:
    return int(_lib.vatt_random_cache_slots(plan))


def vatt_random_cache_fill(plan, k, v, block_table, seq_lens, cache_seeds, rcache, stream=None) -> None:
    rc = _lib.vatt_random_cache_fill(plan, _ptr(k), _ptr(v), _ptr(block_table), _ptr(seq_lens), _ptr(cache_seeds),
                                     _ptr(rcache), _ptr(stream))
    if rc != VATT_OK:
        raise VattError(rc, "vatt_random_cache_fill")


def vatt_append_kv_cached(plan, k_new, v_new, k, v, block_table, seq_lens, cache_seeds, rcache, stream=None) -> None:
    rc = _lib.vatt_append_kv_cached(plan, _ptr(k_new), _ptr(v_new), _ptr(k), _ptr(v), _ptr(block_table),
                                    _ptr(seq_lens), _ptr(cache_seeds), _ptr(rcache), _ptr(stream))
    if rc != VATT_OK:
        raise VattError(rc, "vatt_append_kv_cached")


def vatt_decode_given_topk_cached(plan, q, k, v, block_table, seq_lens, seq_seeds, topk_idx, topk_cnt, rcache,
                                  workspace, out_o, out_lse, out_idx, out_counts, out_budget_raw, out_stats,
                                  stream=None) -> None:
    rc = _lib.vatt_decode_given_topk_cached(plan, _ptr(q), _ptr(k), _ptr(v), _ptr(block_table), _ptr(seq_lens),
                                            _ptr(seq_seeds), _ptr(topk_idx), _ptr(topk_cnt), _ptr(rcache),
                                            _ptr(workspace), _nbytes(workspace), _ptr(out_o), _ptr(out_lse),
                                            _ptr(out_idx), _ptr(out_counts), _ptr(out_budget_raw), _ptr(out_stats),
                                            _ptr(stream))
    if rc != VATT_OK:
        raise VattError(rc, "vatt_decode_given_topk_cached")


def vatt_random_cache_read(plan, rcache, out_tokens, out_counts, stream=None) -> None:
    """Test hook: token of every cache slot (int32 [B, Hkv, slots], -1 where unused) and slots in use ([B, Hkv])."""
    rc = _lib.vatt_random_cache_read(plan, _ptr(rcache), _ptr(out_tokens), _ptr(out_counts), _ptr(stream))
    if rc != VATT_OK:
        raise VattError(rc, "vatt_random_cache_read")


def vatt_row_read(src, rows_total: int, rows, count: int, sink, stream=None) -> None:
    """Measurement aid: read the listed 256-byte rows of the device buffer src and discard them."""
    rc = _lib.vatt_row_read(_ptr(src), int(rows_total), _ptr(rows), int(count), _ptr(sink), _ptr(stream))
    if rc != VATT_OK:
        raise VattError(rc, "vatt_row_read")


def vatt_host_kv_device_pointer(host) -> int:
    """Address to pass as k or v for a cache in pinned host memory (a tensor-like or an int address)."""
    out = ctypes.c_void_p()
    rc = _lib.vatt_host_kv_device_pointer(_ptr(host), ctypes.byref(out))
    if rc != VATT_OK:
        raise VattError(rc, "vatt_host_kv_device_pointer")
    return int(out.value)


def vatt_stream_read(src, nbytes: int, sink, stream=None) -> None:
    """Measurement aid: read nbytes of the device buffer src and discard them (sink: >= 4 KiB device buffer)."""
    rc = _lib.vatt_stream_read(_ptr(src), int(nbytes), _ptr(sink), _ptr(stream))
    if rc != VATT_OK:
        raise VattError(rc, "vatt_stream_read")
