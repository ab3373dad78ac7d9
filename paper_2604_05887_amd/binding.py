"""ctypes binding of libhkv.so: one Python function per C entry point of include/hkv.h,
with the same name.  Argument marshalling only -- every step of the method runs in the
HIP kernels.  PyTorch supplies device memory (tensors) and streams.

Importing this module does not need a GPU; calling a compute entry point does.
If the shared library has not been built the import of the library fails loudly.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence, Tuple

import numpy as np

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libhkv.so")

HKV_OK = 0
HKV_EINVAL, HKV_ESHAPE, HKV_EBUDGET, HKV_EALIGN, HKV_ENOSPACE, HKV_ESTATE, HKV_EHIP = -1, -2, -3, -4, -5, -6, -7
HKV_F32, HKV_BF16 = 0, 1
HKV_STATIC, HKV_DYNAMIC = 0, 1
(HKV_X_KEPT_IDX, HKV_X_SCORES, HKV_X_CHUNK_SEL, HKV_X_CHUNK_SIGMA, HKV_X_CHUNK_MEAN, HKV_X_K_ROWS,
 HKV_X_V_ROWS) = range(7)
HKV_ABI_VERSION = 1
HKV_NOALLOC_SCRATCH_BYTES = 16 << 20

EXPORTED_SYMBOLS = (
    "hkv_query_sizes", "hkv_cache_create", "hkv_query_tier_sizes", "hkv_cache_create_tiered", "hkv_compress", "hkv_decode_attn", "hkv_decode_attn_noalloc", "hkv_full_workspace_size",
    "hkv_full_decode_attn", "hkv_cache_rewind", "hkv_cache_unit_info", "hkv_plan_unit_info", "hkv_cache_step_bytes",
    "hkv_cache_decode_shape", "hkv_cache_call_tiling", "hkv_cache_set_decode_dynamic", "hkv_cache_set_stamps", "hkv_cache_set_device_tail",    "hkv_cache_export", "hkv_cache_import", "hkv_compress_from_scores", "hkv_reselect_chunks",
    "hkv_profile_enable", "hkv_profile_read", "hkv_profile_disable", "hkv_probe_stream_read", "hkv_head_scores_workspace_size", "hkv_head_scores", "hkv_focus_counts_workspace_size", "hkv_focus_counts", "hkv_allocate_budgets",
    "hkv_cache_destroy", "hkv_strerror", "hkv_abi_version",
)


class HkvError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {hkv_strerror(status)} ({status})")


class hkv_config(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("abi_version", C.c_uint32), ("n_layers", C.c_int32),
                ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("dtype", C.c_int32), ("window", C.c_int32), ("chunk_size", C.c_int32),
                ("score_causal", C.c_int32), ("max_new_tokens", C.c_int32), ("softmax_scale", C.c_float),
                ("decode_tile_rows", C.c_int32), ("decode_dynamic", C.c_int32),
                ("chunk_score_group", C.c_int32), ("index_generated", C.c_int32)]


class hkv_plan(C.Structure):
    _fields_ = [("batch", C.c_int32), ("cu_seqlens", C.POINTER(C.c_int32)), ("is_visual", C.POINTER(C.c_uint8)),
                ("head_type", C.POINTER(C.c_uint8)), ("budget", C.POINTER(C.c_int32)),
                ("chunk_size", C.POINTER(C.c_int32))]


_lib = None


def load_library() -> C.CDLL:
    """Load libhkv.so (built in-tree by paper_2604_05887_amd.build).  Raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} not found: build it with `python -m paper_2604_05887_amd.build` "
                          "(there is no CPU fallback)")
    lib = C.CDLL(_LIB_PATH)
    vp, i32, sz = C.c_void_p, C.c_int, C.c_size_t
    lib.hkv_query_sizes.argtypes = [C.POINTER(hkv_config), C.POINTER(hkv_plan), C.POINTER(sz), C.POINTER(sz)]
    lib.hkv_cache_create.argtypes = [C.POINTER(hkv_config), C.POINTER(hkv_plan), vp, sz, C.POINTER(vp)]
    lib.hkv_query_tier_sizes.argtypes = [C.POINTER(hkv_config), C.POINTER(hkv_plan), C.POINTER(sz), C.POINTER(sz),
                                         C.POINTER(sz)]
    lib.hkv_cache_create_tiered.argtypes = [C.POINTER(hkv_config), C.POINTER(hkv_plan), vp, sz, vp, sz, C.POINTER(vp)]
    lib.hkv_compress.argtypes = [vp, i32, i32, vp, vp, vp, vp, sz, vp]
    lib.hkv_decode_attn.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp, sz, vp]
    lib.hkv_decode_attn_noalloc.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp]
    lib.hkv_full_workspace_size.argtypes = [C.POINTER(hkv_config), C.c_int32, C.POINTER(C.c_int32), i32, C.POINTER(sz)]
    lib.hkv_full_decode_attn.argtypes = [C.POINTER(hkv_config), C.c_int32, C.POINTER(C.c_int32), i32, vp, vp, vp, vp,
                                         vp, sz, vp]
    lib.hkv_cache_rewind.argtypes = [vp, vp]
    lib.hkv_cache_unit_info.argtypes = [vp, i32, i32, i32, C.POINTER(C.c_int32), C.POINTER(C.c_int32),
                                        C.POINTER(C.c_int32)]
    lib.hkv_plan_unit_info.argtypes = [C.POINTER(hkv_config), C.POINTER(hkv_plan), i32, i32, i32,
                                       C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
    lib.hkv_cache_step_bytes.argtypes = [vp, i32, i32, i32, C.POINTER(C.c_uint64)]
    lib.hkv_cache_decode_shape.argtypes = [vp, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
    lib.hkv_cache_call_tiling.argtypes = [vp, C.c_int, C.c_int, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
    lib.hkv_cache_set_decode_dynamic.argtypes = [vp, C.c_int32]
    lib.hkv_cache_set_stamps.argtypes = [vp, vp, C.c_int32]
    lib.hkv_cache_set_device_tail.argtypes = [vp, i32, vp]
    lib.hkv_cache_export.argtypes = [vp, i32, i32, i32, i32, vp, sz, C.POINTER(sz), vp]
    lib.hkv_cache_import.argtypes = [vp, i32, i32, i32, i32, vp, sz, vp]
    lib.hkv_compress_from_scores.argtypes = [vp, i32, i32, vp, vp, vp]
    lib.hkv_reselect_chunks.argtypes = [vp, i32, i32, vp]
    lib.hkv_profile_enable.argtypes = [vp, i32]
    lib.hkv_profile_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_int)]
    lib.hkv_profile_disable.argtypes = [vp]
    lib.hkv_probe_stream_read.argtypes = [vp, sz, sz, i32, vp, C.POINTER(C.c_double)]
    lib.hkv_head_scores_workspace_size.argtypes = [C.POINTER(hkv_config), C.c_int32, C.POINTER(C.c_int32),
                                                   C.POINTER(C.c_uint8), C.POINTER(sz), C.POINTER(sz)]
    lib.hkv_head_scores.argtypes = [C.POINTER(hkv_config), C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_uint8), i32, vp, vp,
                                    C.c_double, vp, vp, sz, vp]
    lib.hkv_focus_counts_workspace_size.argtypes = [C.POINTER(hkv_config), C.c_int32, C.c_int32, C.POINTER(sz),
                                                    C.POINTER(sz)]
    lib.hkv_focus_counts.argtypes = [C.POINTER(hkv_config), C.c_int32, C.c_int32, vp, vp, C.c_double, vp, vp, sz, vp]
    lib.hkv_allocate_budgets.argtypes = [C.c_int32, C.POINTER(C.c_float), C.c_float, C.c_int64, C.c_float, C.c_float,
                                         C.c_int32, C.POINTER(C.c_uint8), C.POINTER(C.c_int32)]
    lib.hkv_cache_destroy.argtypes = [vp]
    lib.hkv_cache_destroy.restype = None
    lib.hkv_strerror.argtypes = [i32]
    lib.hkv_strerror.restype = C.c_char_p
    lib.hkv_abi_version.argtypes = []
    lib.hkv_abi_version.restype = C.c_uint32
    _lib = lib
    return lib


def _check(status: int, where: str) -> None:
    if status != HKV_OK:
        raise HkvError(status, where)


def _ptr(t) -> Optional[int]:
    """Device (or host) address of a torch tensor, or None."""
    return None if t is None else int(t.data_ptr())


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return int(torch.cuda.current_stream().cuda_stream) or None
    if isinstance(stream, int):
        return stream or None
    return int(stream.cuda_stream) or None


def make_config(*, n_layers: int, n_q_heads: int, n_kv_heads: int, dtype: int, window: int, chunk_size: int = 32,
                max_new_tokens: int = 0, head_dim: int = 128, score_causal: int = 0,
                softmax_scale: float = 0.0, decode_tile_rows: int = 0, decode_dynamic: int = 0,
                chunk_score_group: int = 0, index_generated: int = 0) -> hkv_config:
    return hkv_config(C.sizeof(hkv_config), HKV_ABI_VERSION, n_layers, n_q_heads, n_kv_heads, head_dim, dtype,
                      window, chunk_size, score_causal, max_new_tokens, softmax_scale, decode_tile_rows, decode_dynamic,
                      chunk_score_group, index_generated)


class PlanArrays:
    """Keeps the host arrays of an hkv_plan alive and exposes the ctypes struct."""

    def __init__(self, cu_seqlens: Sequence[int], is_visual, head_type, budget, chunk_size=None):
        self.cu = np.ascontiguousarray(cu_seqlens, dtype=np.int32)
        self.vis = np.ascontiguousarray(is_visual, dtype=np.uint8)
        self.ht = np.ascontiguousarray(head_type, dtype=np.uint8)
        self.bud = np.ascontiguousarray(budget, dtype=np.int32)
        self.cs = None if chunk_size is None else np.ascontiguousarray(chunk_size, dtype=np.int32)
        self.struct = hkv_plan(
            len(self.cu) - 1, self.cu.ctypes.data_as(C.POINTER(C.c_int32)),
            self.vis.ctypes.data_as(C.POINTER(C.c_uint8)), self.ht.ctypes.data_as(C.POINTER(C.c_uint8)),
            self.bud.ctypes.data_as(C.POINTER(C.c_int32)),
            None if self.cs is None else self.cs.ctypes.data_as(C.POINTER(C.c_int32)))


# ---------------------------------------------------------------------------------------------
# one function per C entry point
# ---------------------------------------------------------------------------------------------
def hkv_abi_version() -> int:
    return int(load_library().hkv_abi_version())


def hkv_strerror(status: int) -> str:
    return load_library().hkv_strerror(int(status)).decode()


def hkv_query_sizes(cfg: hkv_config, plan: PlanArrays) -> Tuple[int, int]:
    cb, wb = C.c_size_t(0), C.c_size_t(0)
    _check(load_library().hkv_query_sizes(C.byref(cfg), C.byref(plan.struct), C.byref(cb), C.byref(wb)),
           "hkv_query_sizes")
    return int(cb.value), int(wb.value)


def hkv_cache_create(cfg: hkv_config, plan: PlanArrays, cache_dev, cache_bytes: int) -> int:
    h = C.c_void_p(None)
    _check(load_library().hkv_cache_create(C.byref(cfg), C.byref(plan.struct), _ptr(cache_dev), cache_bytes,
                                           C.byref(h)), "hkv_cache_create")
    return int(h.value)


def hkv_query_tier_sizes(cfg: hkv_config, plan: PlanArrays) -> Tuple[int, int, int]:
    cb, hb, wb = C.c_size_t(0), C.c_size_t(0), C.c_size_t(0)
    _check(load_library().hkv_query_tier_sizes(C.byref(cfg), C.byref(plan.struct), C.byref(cb), C.byref(hb),
                                               C.byref(wb)), "hkv_query_tier_sizes")
    return int(cb.value), int(hb.value), int(wb.value)


def hkv_cache_create_tiered(cfg: hkv_config, plan: PlanArrays, cache_dev, cache_bytes: int, host_tier,
                            host_bytes: int) -> int:
    h = C.c_void_p(None)
    _check(load_library().hkv_cache_create_tiered(C.byref(cfg), C.byref(plan.struct), _ptr(cache_dev), cache_bytes,
                                                  _ptr(host_tier), host_bytes, C.byref(h)),
           "hkv_cache_create_tiered")
    return int(h.value)


def hkv_cache_destroy(handle: int) -> None:
    load_library().hkv_cache_destroy(handle)


def hkv_compress(handle: int, layer_begin: int, layer_end: int, q_window, k, v, workspace, workspace_bytes: int,
                 stream=None) -> None:
    _check(load_library().hkv_compress(handle, layer_begin, layer_end, _ptr(q_window), _ptr(k), _ptr(v),
                                       _ptr(workspace), workspace_bytes, _stream(stream)), "hkv_compress")


def hkv_compress_from_scores(handle: int, layer_begin: int, layer_end: int, k, v, stream=None) -> None:
    _check(load_library().hkv_compress_from_scores(handle, layer_begin, layer_end, _ptr(k), _ptr(v),
                                                   _stream(stream)), "hkv_compress_from_scores")


def hkv_decode_attn(handle: int, layer_begin: int, layer_end: int, q, k_new, v_new, out, workspace,
                    workspace_bytes: int, stream=None) -> None:
    _check(load_library().hkv_decode_attn(handle, layer_begin, layer_end, _ptr(q), _ptr(k_new), _ptr(v_new),
                                          _ptr(out), _ptr(workspace), workspace_bytes, _stream(stream)),
           "hkv_decode_attn")


def hkv_decode_attn_noalloc(handle: int, layer_begin: int, layer_end: int, q, k_new, v_new, out, stream=None) -> None:
    _check(load_library().hkv_decode_attn_noalloc(handle, layer_begin, layer_end, _ptr(q), _ptr(k_new), _ptr(v_new),
                                                  _ptr(out), _stream(stream)), "hkv_decode_attn_noalloc")


def hkv_reselect_chunks(handle: int, layer_begin: int, layer_end: int, stream=None) -> None:
    _check(load_library().hkv_reselect_chunks(handle, layer_begin, layer_end, _stream(stream)),
           "hkv_reselect_chunks")


def hkv_full_workspace_size(cfg: hkv_config, cu_seqlens, n_layers_call: int) -> int:
    cu = np.ascontiguousarray(cu_seqlens, dtype=np.int32)
    wb = C.c_size_t(0)
    _check(load_library().hkv_full_workspace_size(C.byref(cfg), len(cu) - 1, cu.ctypes.data_as(C.POINTER(C.c_int32)),
                                                  n_layers_call, C.byref(wb)), "hkv_full_workspace_size")
    return int(wb.value)


def hkv_full_decode_attn(cfg: hkv_config, cu_seqlens, n_layers_call: int, q, k, v, out, workspace,
                         workspace_bytes: int, stream=None) -> None:
    cu = np.ascontiguousarray(cu_seqlens, dtype=np.int32)
    _check(load_library().hkv_full_decode_attn(C.byref(cfg), len(cu) - 1, cu.ctypes.data_as(C.POINTER(C.c_int32)),
                                               n_layers_call, _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(workspace),
                                               workspace_bytes, _stream(stream)), "hkv_full_decode_attn")


def hkv_cache_rewind(handle: int, stream=None) -> None:
    _check(load_library().hkv_cache_rewind(handle, _stream(stream)), "hkv_cache_rewind")


def hkv_cache_unit_info(handle: int, seq: int, layer: int, head: int) -> Tuple[int, int, int]:
    a, b, c = C.c_int32(0), C.c_int32(0), C.c_int32(0)
    _check(load_library().hkv_cache_unit_info(handle, seq, layer, head, C.byref(a), C.byref(b), C.byref(c)),
           "hkv_cache_unit_info")
    return int(a.value), int(b.value), int(c.value)


def hkv_plan_unit_info(cfg: hkv_config, plan: PlanArrays, seq: int, layer: int, head: int) -> Tuple[int, int, int]:
    a, b, c = C.c_int32(0), C.c_int32(0), C.c_int32(0)
    _check(load_library().hkv_plan_unit_info(C.byref(cfg), C.byref(plan.struct), seq, layer, head, C.byref(a),
                                             C.byref(b), C.byref(c)), "hkv_plan_unit_info")
    return int(a.value), int(b.value), int(c.value)


def hkv_cache_step_bytes(handle: int, layer_begin: int, layer_end: int, tail: int) -> int:
    v = C.c_uint64(0)
    _check(load_library().hkv_cache_step_bytes(handle, layer_begin, layer_end, tail, C.byref(v)),
           "hkv_cache_step_bytes")
    return int(v.value)


def hkv_cache_decode_shape(handle: int) -> Tuple[int, int]:
    """(rows per split-K tile, dynamic mode) the cache's decode steps run with."""
    t, m = C.c_int32(0), C.c_int32(0)
    _check(load_library().hkv_cache_decode_shape(handle, C.byref(t), C.byref(m)), "hkv_cache_decode_shape")
    return int(t.value), int(m.value)


def hkv_cache_call_tiling(handle: int, layer_begin: int, layer_end: int) -> Tuple[int, int]:
    """(rows per tile, tiles) of a decode call over the given layers."""
    t, n = C.c_int32(0), C.c_int32(0)
    _check(load_library().hkv_cache_call_tiling(handle, layer_begin, layer_end, C.byref(t), C.byref(n)),
           "hkv_cache_call_tiling")
    return int(t.value), int(n.value)


def hkv_cache_set_decode_dynamic(handle: int, mode: int) -> None:
    _check(load_library().hkv_cache_set_decode_dynamic(handle, mode), "hkv_cache_set_decode_dynamic")


HKV_STAMP_WORDS = 8


def hkv_cache_set_stamps(handle: int, stamps, n_records: int) -> None:
    """stamps: device tensor of n_records * HKV_STAMP_WORDS int64 (or None to clear the setting)."""
    _check(load_library().hkv_cache_set_stamps(handle, _ptr(stamps), int(n_records)), "hkv_cache_set_stamps")


def hkv_cache_set_device_tail(handle: int, enable: bool, stream=None) -> None:
    _check(load_library().hkv_cache_set_device_tail(handle, 1 if enable else 0, _stream(stream)), "hkv_cache_set_device_tail")


def hkv_head_scores_workspace_size(cfg: hkv_config, cu_seqlens, is_visual) -> Tuple[int, int]:
    cu = np.ascontiguousarray(cu_seqlens, dtype=np.int32)
    vis = np.ascontiguousarray(is_visual, dtype=np.uint8)
    lo, hi = C.c_size_t(0), C.c_size_t(0)
    _check(load_library().hkv_head_scores_workspace_size(C.byref(cfg), len(cu) - 1, cu.ctypes.data_as(C.POINTER(C.c_int32)),
                                                         vis.ctypes.data_as(C.POINTER(C.c_uint8)), C.byref(lo), C.byref(hi)),
           "hkv_head_scores_workspace_size")
    return int(lo.value), int(hi.value)


def hkv_head_scores(cfg: hkv_config, cu_seqlens, is_visual, n_layers_call: int, q_prompt, k, focus_fraction: float,
                    scores, workspace, workspace_bytes: int, stream=None) -> None:
    cu = np.ascontiguousarray(cu_seqlens, dtype=np.int32)
    vis = np.ascontiguousarray(is_visual, dtype=np.uint8)
    _check(load_library().hkv_head_scores(C.byref(cfg), len(cu) - 1, cu.ctypes.data_as(C.POINTER(C.c_int32)),
                                          vis.ctypes.data_as(C.POINTER(C.c_uint8)), n_layers_call, _ptr(q_prompt), _ptr(k),
                                          focus_fraction, _ptr(scores), _ptr(workspace), workspace_bytes, _stream(stream)),
           "hkv_head_scores")


def hkv_focus_counts_workspace_size(cfg: hkv_config, n_steps: int, context_len: int) -> Tuple[int, int]:
    lo, hi = C.c_size_t(0), C.c_size_t(0)
    _check(load_library().hkv_focus_counts_workspace_size(C.byref(cfg), n_steps, context_len, C.byref(lo), C.byref(hi)),
           "hkv_focus_counts_workspace_size")
    return int(lo.value), int(hi.value)


def hkv_focus_counts(cfg: hkv_config, n_steps: int, context_len: int, q_steps, k, focus_fraction: float, counts,
                     workspace, workspace_bytes: int, stream=None) -> None:
    _check(load_library().hkv_focus_counts(C.byref(cfg), n_steps, context_len, _ptr(q_steps), _ptr(k), focus_fraction,
                                           _ptr(counts), _ptr(workspace), workspace_bytes, _stream(stream)),
           "hkv_focus_counts")


def hkv_allocate_budgets(scores, theta: float, total_budget: int, share_ratio: float, alpha: float,
                         pad_pow2: bool = True) -> Tuple[np.ndarray, np.ndarray]:
    """(head_type uint8, budget int32), same shape as `scores` (host arrays)."""
    sc = np.ascontiguousarray(scores, dtype=np.float32)
    types = np.zeros(sc.shape, np.uint8)
    budget = np.zeros(sc.shape, np.int32)
    _check(load_library().hkv_allocate_budgets(sc.size, sc.ctypes.data_as(C.POINTER(C.c_float)), theta, total_budget,
                                               share_ratio, alpha, 1 if pad_pow2 else 0,
                                               types.ctypes.data_as(C.POINTER(C.c_uint8)),
                                               budget.ctypes.data_as(C.POINTER(C.c_int32))), "hkv_allocate_budgets")
    return types, budget


def hkv_probe_stream_read(buf_ptr: int, buf_bytes: int, read_bytes: int, reps: int, stream: int = 0) -> float:
    """Average microseconds of a kernel that only reads read_bytes of the device buffer."""
    v = C.c_double(0.0)
    _check(load_library().hkv_probe_stream_read(buf_ptr, buf_bytes, read_bytes, reps, stream, C.byref(v)),
           "hkv_probe_stream_read")
    return float(v.value)


def hkv_profile_enable(handle: int, max_calls: int) -> None:
    _check(load_library().hkv_profile_enable(handle, max_calls), "hkv_profile_enable")


def hkv_profile_read(handle: int) -> Tuple[Tuple[float, float, float], int]:
    ms = (C.c_double * 3)()
    n = C.c_int(0)
    _check(load_library().hkv_profile_read(handle, ms, C.byref(n)), "hkv_profile_read")
    return (float(ms[0]), float(ms[1]), float(ms[2])), int(n.value)


def hkv_profile_disable(handle: int) -> None:
    _check(load_library().hkv_profile_disable(handle), "hkv_profile_disable")


_EXPORT_NP = {HKV_X_KEPT_IDX: np.int32, HKV_X_SCORES: np.float32, HKV_X_CHUNK_SEL: np.int32,
              HKV_X_CHUNK_SIGMA: np.float32}


def hkv_cache_export(handle: int, what: int, seq: int, layer: int, head: int, dtype: int, stream=None) -> np.ndarray:
    """Returns a host array: int32/float32 for indices and scores; for summaries and K/V rows a
    float32 [rows, 128] array holding the stored values exactly (bf16 widened)."""
    lib = load_library()
    need = C.c_size_t(0)
    st = lib.hkv_cache_export(handle, what, seq, layer, head, None, 0, C.byref(need), _stream(stream))
    if st not in (HKV_OK, HKV_ENOSPACE):
        _check(st, "hkv_cache_export")
    n = int(need.value)
    raw = np.empty(max(n, 1), np.uint8)
    if n:
        _check(lib.hkv_cache_export(handle, what, seq, layer, head, raw.ctypes.data, n, C.byref(need),
                                    _stream(stream)), "hkv_cache_export")
    raw = raw[:n]
    if what in _EXPORT_NP:
        return raw.view(_EXPORT_NP[what]).copy()
    if dtype == HKV_F32:
        return raw.view(np.float32).reshape(-1, 128).copy()
    u16 = raw.view(np.uint16).astype(np.uint32) << np.uint32(16)
    return u16.view(np.float32).reshape(-1, 128).copy()


def hkv_cache_import(handle: int, what: int, seq: int, layer: int, head: int, values: np.ndarray, dtype: int,
                     stream=None) -> None:
    """values: float32 array (scores / sigma / summaries); summaries are narrowed to the cache dtype
    and must already be exactly representable in it."""
    arr = np.ascontiguousarray(values, dtype=np.float32)
    if what == HKV_X_CHUNK_MEAN and dtype == HKV_BF16:
        bits = arr.view(np.uint32)
        if np.any(bits & np.uint32(0xFFFF)):
            raise ValueError("summary values are not bf16-representable")
        arr = (bits >> np.uint32(16)).astype(np.uint16)
    _check(load_library().hkv_cache_import(handle, what, seq, layer, head, arr.ctypes.data, arr.nbytes,
                                           _stream(stream)), "hkv_cache_import")


# ---------------------------------------------------------------------------------------------
# convenience holder: device memory from torch + the handle (no arithmetic)
# ---------------------------------------------------------------------------------------------
class HybridKVCache:
    """Allocates the cache arena and workspace as torch tensors and forwards to the C entry points."""

    def __init__(self, cfg: hkv_config, plan: PlanArrays, device="cuda:0", host_tier: bool = False):
        """host_tier: keep the dynamic heads' prompt rows in page-locked host memory (bf16 caches)."""
        import torch
        self.cfg, self.plan = cfg, plan
        self.host_bytes = 0
        if host_tier:
            self.cache_bytes, self.host_bytes, self.workspace_bytes = hkv_query_tier_sizes(cfg, plan)
        else:
            self.cache_bytes, self.workspace_bytes = hkv_query_sizes(cfg, plan)
        self.arena = torch.empty(self.cache_bytes + 256, dtype=torch.uint8, device=device)
        pad = (-self.arena.data_ptr()) % 256
        self.arena_view = self.arena[pad:pad + self.cache_bytes]
        self.workspace = torch.empty(self.workspace_bytes, dtype=torch.uint8, device=device)
        if host_tier:
            self.host_arena = torch.empty(self.host_bytes + 256, dtype=torch.uint8, pin_memory=True)
            hpad = (-self.host_arena.data_ptr()) % 256
            self.host_view = self.host_arena[hpad:hpad + self.host_bytes]
            self.handle = hkv_cache_create_tiered(cfg, plan, self.arena_view, self.cache_bytes, self.host_view,
                                                  self.host_bytes)
        else:
            self.handle = hkv_cache_create(cfg, plan, self.arena_view, self.cache_bytes)

    def compress(self, q_window, k, v, layer_begin=0, layer_end=None, stream=None):
        le = self.cfg.n_layers if layer_end is None else layer_end
        hkv_compress(self.handle, layer_begin, le, q_window, k, v, self.workspace, self.workspace_bytes, stream)

    def compress_from_scores(self, k, v, layer_begin=0, layer_end=None, stream=None):
        le = self.cfg.n_layers if layer_end is None else layer_end
        hkv_compress_from_scores(self.handle, layer_begin, le, k, v, stream)

    def decode_attn(self, q, k_new, v_new, out, layer_begin=0, layer_end=None, stream=None):
        le = self.cfg.n_layers if layer_end is None else layer_end
        hkv_decode_attn(self.handle, layer_begin, le, q, k_new, v_new, out, self.workspace, self.workspace_bytes,
                        stream)

    def decode_attn_noalloc(self, q, k_new, v_new, out, layer_begin=0, layer_end=None, stream=None):
        le = self.cfg.n_layers if layer_end is None else layer_end
        hkv_decode_attn_noalloc(self.handle, layer_begin, le, q, k_new, v_new, out, stream)

    def export(self, what, seq, layer, head, stream=None):
        return hkv_cache_export(self.handle, what, seq, layer, head, self.cfg.dtype, stream)

    def import_(self, what, seq, layer, head, values, stream=None):
        hkv_cache_import(self.handle, what, seq, layer, head, values, self.cfg.dtype, stream)

    def unit_info(self, seq, layer, head):
        return hkv_cache_unit_info(self.handle, seq, layer, head)

    def step_bytes(self, tail, layer_begin=0, layer_end=None):
        le = self.cfg.n_layers if layer_end is None else layer_end
        return hkv_cache_step_bytes(self.handle, layer_begin, le, tail)

    def decode_shape(self):
        return hkv_cache_decode_shape(self.handle)

    def call_tiling(self, layer_begin=0, layer_end=None):
        le = self.cfg.n_layers if layer_end is None else layer_end
        return hkv_cache_call_tiling(self.handle, layer_begin, le)

    def set_decode_dynamic(self, mode: int):
        hkv_cache_set_decode_dynamic(self.handle, mode)

    def set_stamps(self, stamps, n_records: int = 0):
        hkv_cache_set_stamps(self.handle, stamps, n_records)

    def set_device_tail(self, enable: bool, stream=None):
        hkv_cache_set_device_tail(self.handle, enable, stream)

    def rewind(self, stream=None):
        hkv_cache_rewind(self.handle, stream)

    def close(self):
        if self.handle:
            hkv_cache_destroy(self.handle)
            self.handle = 0

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
