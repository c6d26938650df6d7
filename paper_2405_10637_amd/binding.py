"""ctypes binding of liblckv.so: the same names as include/lckv.h and include/lckv_tools.h, argument marshalling only.

Tensors are torch CUDA (ROCm) tensors used as plain device buffers; their ``data_ptr()`` and the current
torch stream are passed through.  There is no fallback: without the built library every call raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblckv.so")

LCKV_OK = 0
LCKV_ERR_NULL, LCKV_ERR_CONFIG, LCKV_ERR_LAYER, LCKV_ERR_NOT_PRODUCER, LCKV_ERR_BATCH = -1, -2, -3, -4, -5
LCKV_ERR_LENGTH, LCKV_ERR_WORKSPACE, LCKV_ERR_ALIGN, LCKV_ERR_BLOCK_TABLE, LCKV_ERR_HIP = -6, -7, -8, -9, -10
LCKV_ERR_MASK, LCKV_ERR_STORAGE, LCKV_ERR_RANGE = -11, -12, -13
LCKV_BF16, LCKV_F32 = 0, 1
LCKV_PAIR_TOP_OF_CONDENSED, LCKV_PAIR_LAST_LAYER = 0, 1
LCKV_DEV_ERR_CAPACITY, LCKV_DEV_ERR_BLOCK, LCKV_DEV_ERR_BARRIER = 1, 2, 4
LCKV_LOAD_AUTO, LCKV_LOAD_TEMPORAL, LCKV_LOAD_NONTEMPORAL = 0, 1, 2
LCKV_STATIC_SCRATCH_BYTES = 32 << 20

EXPORTS = [
    "lckv_cache_bytes", "lckv_plan_max_batch", "lckv_cache_alloc", "lckv_cache_free", "lckv_cache_set_block_table", "lckv_n_slots",
    "lckv_kv_slot", "lckv_slot_producer", "lckv_append_kv", "lckv_decode_attention", "lckv_prefill_attention",
    "lckv_set_prefill_tile", "lckv_project_qkv", "lckv_project_workspace_bytes", "lckv_pack_projection_weight", "lckv_step",
    "lckv_step_static_scratch", "lckv_step_one_launch", "lckv_step_one_launch_workspace_bytes", "lckv_set_barrier_wait_ms",
    "lckv_workspace_bytes", "lckv_set_split_tokens", "lckv_set_workgroup_waves", "lckv_set_load_policy", "lckv_cache_load_dense", "lckv_cache_read",
    "lckv_last_device_error", "lckv_profile_enable", "lckv_profile_read", "lckv_profile_launch_ms",
    "lckv_hbm_read_probe", "lckv_strerror",
]


class lckv_config(ctypes.Structure):
    _fields_ = [
        ("L", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32), ("D", ctypes.c_int32),
        ("dtype", ctypes.c_int32), ("B_max", ctypes.c_int32), ("T_max", ctypes.c_int32),
        ("page_size", ctypes.c_int32), ("num_blocks", ctypes.c_int64),
        ("warmup_mask", ctypes.POINTER(ctypes.c_uint8)), ("pairing_rule", ctypes.c_int32),
        ("scale", ctypes.c_float), ("sink_tokens", ctypes.c_int32), ("window_tokens", ctypes.c_int32),
    ]


class LckvError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__("%s failed: %d (%s)" % (where, code, lckv_strerror(code)))


_lib = None


def lib():
    """The loaded C-ABI library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("liblckv.so is not built: run `python -m paper_2405_10637_amd.build` "
                               "(there is no CPU or PyTorch fallback)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
        cfgp = ctypes.POINTER(lckv_config)
        L.lckv_cache_bytes.argtypes = [cfgp, ctypes.POINTER(sz)]
        L.lckv_plan_max_batch.argtypes = [cfgp, sz, ctypes.POINTER(i32)]
        L.lckv_cache_alloc.argtypes = [cfgp, vp, sz, ctypes.POINTER(vp)]
        L.lckv_cache_free.argtypes = [vp]
        L.lckv_cache_set_block_table.argtypes = [vp, vp, i32]
        L.lckv_n_slots.argtypes = [vp, ctypes.POINTER(i32)]
        L.lckv_kv_slot.argtypes = [vp, i32, ctypes.POINTER(i32), ctypes.POINTER(i32)]
        L.lckv_slot_producer.argtypes = [vp, i32, ctypes.POINTER(i32)]
        L.lckv_append_kv.argtypes = [vp, i32, vp, vp, vp, i32, vp]
        L.lckv_decode_attention.argtypes = [vp, i32, vp, vp, vp, vp, i32, i32, vp, sz, vp]
        L.lckv_prefill_attention.argtypes = [vp, i32, vp, vp, vp, i32, i32, vp]
        L.lckv_set_prefill_tile.argtypes = [vp, i32]
        L.lckv_project_qkv.argtypes = [vp, i32, vp, i32, vp, vp, vp, vp, vp, vp, vp, i32, ctypes.c_float, vp, sz, vp]
        L.lckv_project_workspace_bytes.argtypes = [vp, i32, i32, ctypes.POINTER(sz)]
        L.lckv_pack_projection_weight.argtypes = [vp, vp, vp, i32, i32, vp]
        L.lckv_step.argtypes =[vp, vp, vp, vp, vp, vp, i32, i32, vp, sz, vp]
        L.lckv_step_static_scratch.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, vp]
        L.lckv_step_one_launch.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, vp, sz, vp]
        L.lckv_step_one_launch_workspace_bytes.argtypes = [vp, i32, i32, ctypes.POINTER(sz)]
        L.lckv_set_barrier_wait_ms.argtypes = [vp, ctypes.c_double]
        L.lckv_workspace_bytes.argtypes = [vp, i32, i32, ctypes.POINTER(sz)]
        L.lckv_set_split_tokens.argtypes = [vp, i32]
        L.lckv_set_workgroup_waves.argtypes = [vp, i32]
        L.lckv_set_load_policy.argtypes = [vp, i32]
        L.lckv_cache_load_dense.argtypes = [vp, i32, vp, vp, vp, i32, i32, vp]
        L.lckv_cache_read.argtypes = [vp, i32, i32, i32, i32, vp, vp]
        L.lckv_last_device_error.argtypes = [vp, ctypes.POINTER(i32)]
        L.lckv_profile_enable.argtypes = [vp, i32]
        L.lckv_profile_read.argtypes = [vp, ctypes.POINTER(i32), ctypes.POINTER(ctypes.c_double)]
        L.lckv_hbm_read_probe.argtypes = [vp, vp, sz, i32, vp]
        L.lckv_profile_launch_ms.argtypes = [vp, vp, i32, ctypes.POINTER(i32)]
        L.lckv_strerror.argtypes = [ctypes.c_int]
        L.lckv_strerror.restype = ctypes.c_char_p
        for name in EXPORTS:
            if name != "lckv_strerror":
                getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def lckv_strerror(code: int) -> str:
    return lib().lckv_strerror(int(code)).decode()


def _check(rc: int, where: str):
    if rc != LCKV_OK:
        raise LckvError(rc, where)


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    h = stream if isinstance(stream, int) else stream.cuda_stream
    return h or None


def make_config(L, Hq, Hkv, D, dtype, B_max, T_max, warmup_mask, page_size=0, num_blocks=0,
                pairing_rule=LCKV_PAIR_TOP_OF_CONDENSED, scale=0.0, sink_tokens=0, window_tokens=0) -> lckv_config:
    mask = np.ascontiguousarray(np.asarray(warmup_mask, dtype=np.uint8))
    cfg = lckv_config(L, Hq, Hkv, D, dtype, B_max, T_max, page_size, num_blocks,
                      mask.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)), pairing_rule, scale, sink_tokens,
                      window_tokens)
    cfg._mask_keepalive = mask
    return cfg


def lckv_cache_bytes(cfg: lckv_config) -> int:
    out = ctypes.c_size_t(0)
    _check(lib().lckv_cache_bytes(ctypes.byref(cfg), ctypes.byref(out)), "lckv_cache_bytes")
    return out.value


def lckv_plan_max_batch(cfg: lckv_config, budget_bytes: int) -> int:
    out = ctypes.c_int32(0)
    _check(lib().lckv_plan_max_batch(ctypes.byref(cfg), budget_bytes, ctypes.byref(out)), "lckv_plan_max_batch")
    return out.value


def lckv_cache_alloc(cfg: lckv_config, kv_storage, kv_bytes: Optional[int] = None) -> int:
    """Returns the opaque handle (an integer address).  `kv_storage`: a device tensor (kept alive by the caller)."""
    if kv_bytes is None:
        kv_bytes = kv_storage.numel() * kv_storage.element_size()
    h = ctypes.c_void_p(None)
    _check(lib().lckv_cache_alloc(ctypes.byref(cfg), _ptr(kv_storage), kv_bytes, ctypes.byref(h)), "lckv_cache_alloc")
    return h.value


def lckv_cache_free(cache: int):
    _check(lib().lckv_cache_free(cache), "lckv_cache_free")


def lckv_cache_set_block_table(cache: int, dev_table, max_blocks_per_seq: int):
    _check(lib().lckv_cache_set_block_table(cache, _ptr(dev_table), max_blocks_per_seq), "lckv_cache_set_block_table")


def lckv_n_slots(cache: int) -> int:
    n = ctypes.c_int32(0)
    _check(lib().lckv_n_slots(cache, ctypes.byref(n)), "lckv_n_slots")
    return n.value


def lckv_kv_slot(cache: int, layer: int):
    s, v = ctypes.c_int32(0), ctypes.c_int32(0)
    _check(lib().lckv_kv_slot(cache, layer, ctypes.byref(s), ctypes.byref(v)), "lckv_kv_slot")
    return s.value, v.value


def lckv_slot_producer(cache: int, slot: int) -> int:
    l = ctypes.c_int32(0)
    _check(lib().lckv_slot_producer(cache, slot, ctypes.byref(l)), "lckv_slot_producer")
    return l.value


def lckv_append_kv(cache: int, layer: int, k_new, v_new, dev_seq_lens, B: int, stream=None):
    _check(lib().lckv_append_kv(cache, layer, _ptr(k_new), _ptr(v_new), _ptr(dev_seq_lens), B, _stream(stream)),
           "lckv_append_kv")


def lckv_decode_attention(cache: int, layer: int, q, out, dev_seq_lens, warmup_mask, B: int, max_len_hint: int,
                          workspace=None, workspace_bytes: Optional[int] = None, stream=None):
    mask = None
    if warmup_mask is not None:
        mask = np.ascontiguousarray(np.asarray(warmup_mask, dtype=np.uint8)).ctypes.data
    if workspace_bytes is None:
        workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().lckv_decode_attention(cache, layer, _ptr(q), _ptr(out), _ptr(dev_seq_lens), mask, B, max_len_hint,
                                       _ptr(workspace), workspace_bytes, _stream(stream)), "lckv_decode_attention")


def lckv_prefill_attention(cache: int, layer: int, q, out, dev_prompt_lens, B: int, S: int, stream=None):
    _check(lib().lckv_prefill_attention(cache, layer, _ptr(q), _ptr(out), _ptr(dev_prompt_lens), B, S,
                                        _stream(stream)), "lckv_prefill_attention")


def lckv_set_prefill_tile(cache: int, query_blocks_per_wave: int):
    _check(lib().lckv_set_prefill_tile(cache, query_blocks_per_wave), "lckv_set_prefill_tile")


def lckv_step(cache: int, q_all, k_new_all, v_new_all, out_all, dev_seq_lens, B: int, max_len_hint: int,
              workspace=None, workspace_bytes: Optional[int] = None, stream=None):
    if workspace_bytes is None:
        workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().lckv_step(cache, _ptr(q_all), _ptr(k_new_all), _ptr(v_new_all), _ptr(out_all), _ptr(dev_seq_lens), B,
                           max_len_hint, _ptr(workspace), workspace_bytes, _stream(stream)), "lckv_step")


def lckv_step_one_launch(cache: int, q_all, k_new_all, v_new_all, out_all, dev_seq_lens, B: int, max_len_hint: int,
                         workspace=None, workspace_bytes: Optional[int] = None, stream=None):
    if workspace_bytes is None:
        workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().lckv_step_one_launch(cache, _ptr(q_all), _ptr(k_new_all), _ptr(v_new_all), _ptr(out_all),
                                      _ptr(dev_seq_lens), B, max_len_hint, _ptr(workspace), workspace_bytes,
                                      _stream(stream)), "lckv_step_one_launch")


def lckv_step_one_launch_workspace_bytes(cache: int, B: int, max_len_hint: int) -> int:
    out = ctypes.c_size_t(0)
    _check(lib().lckv_step_one_launch_workspace_bytes(cache, B, max_len_hint, ctypes.byref(out)),
           "lckv_step_one_launch_workspace_bytes")
    return out.value


def lckv_set_barrier_wait_ms(cache: int, ms: float):
    _check(lib().lckv_set_barrier_wait_ms(cache, float(ms)), "lckv_set_barrier_wait_ms")


def lckv_step_static_scratch(cache: int, q_all, k_new_all, v_new_all, out_all, dev_seq_lens, B: int, max_len_hint: int,
                             stream=None):
    _check(lib().lckv_step_static_scratch(cache, _ptr(q_all), _ptr(k_new_all), _ptr(v_new_all), _ptr(out_all),
                                          _ptr(dev_seq_lens), B, max_len_hint, _stream(stream)),
           "lckv_step_static_scratch")


def lckv_pack_projection_weight(cache: int, w, w_packed, n_rows: int, hidden: int, stream=None):
    _check(lib().lckv_pack_projection_weight(cache, _ptr(w), _ptr(w_packed), n_rows, hidden, _stream(stream)),
           "lckv_pack_projection_weight")


def lckv_project_workspace_bytes(cache: int, B: int, hidden: int) -> int:
    out = ctypes.c_size_t(0)
    _check(lib().lckv_project_workspace_bytes(cache, B, hidden, ctypes.byref(out)), "lckv_project_workspace_bytes")
    return out.value


def lckv_project_qkv(cache: int, layer: int, x, hidden: int, w_q, w_k, w_v, q_out, dev_seq_lens, B: int,
                     rope_base: float, workspace, stream=None, k_out=None, v_out=None,
                     workspace_bytes: Optional[int] = None):
    if workspace_bytes is None:
        workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().lckv_project_qkv(cache, layer, _ptr(x), hidden, _ptr(w_q), _ptr(w_k), _ptr(w_v), _ptr(q_out),
                                  _ptr(k_out), _ptr(v_out), _ptr(dev_seq_lens), B,
                                  float(rope_base), _ptr(workspace), workspace_bytes, _stream(stream)),
           "lckv_project_qkv")


def lckv_workspace_bytes(cache: int, B: int, max_len_hint: int) -> int:
    out = ctypes.c_size_t(0)
    _check(lib().lckv_workspace_bytes(cache, B, max_len_hint, ctypes.byref(out)), "lckv_workspace_bytes")
    return out.value


def lckv_set_split_tokens(cache: int, tokens: int):
    _check(lib().lckv_set_split_tokens(cache, tokens), "lckv_set_split_tokens")


def lckv_set_workgroup_waves(cache: int, waves: int):
    _check(lib().lckv_set_workgroup_waves(cache, waves), "lckv_set_workgroup_waves")


def lckv_set_load_policy(cache: int, policy: int):
    _check(lib().lckv_set_load_policy(cache, policy), "lckv_set_load_policy")


def lckv_cache_load_dense(cache: int, slot: int, k, v, dev_seq_lens, B: int, T: int, stream=None):
    _check(lib().lckv_cache_load_dense(cache, slot, _ptr(k), _ptr(v), _ptr(dev_seq_lens), B, T, _stream(stream)),
           "lckv_cache_load_dense")


def lckv_cache_read(cache: int, slot: int, b: int, pos: int, n_pos: int, host_k: np.ndarray, host_v: np.ndarray):
    """host_k, host_v: writable C-contiguous numpy arrays of n_pos*Hkv*D elements (uint16 for bf16, float32)."""
    _check(lib().lckv_cache_read(cache, slot, b, pos, n_pos, host_k.ctypes.data, host_v.ctypes.data), "lckv_cache_read")


def lckv_last_device_error(cache: int) -> int:
    bits = ctypes.c_int32(0)
    _check(lib().lckv_last_device_error(cache, ctypes.byref(bits)), "lckv_last_device_error")
    return bits.value


def lckv_hbm_read_probe(cache: int, dev_buf, nbytes: int, nontemporal: bool = True, stream=None):
    _check(lib().lckv_hbm_read_probe(cache, _ptr(dev_buf), nbytes, int(nontemporal), _stream(stream)),
           "lckv_hbm_read_probe")


def lckv_profile_enable(cache: int, enable: bool):
    _check(lib().lckv_profile_enable(cache, int(bool(enable))), "lckv_profile_enable")


def lckv_profile_read(cache: int):
    n, ms = ctypes.c_int32(0), ctypes.c_double(0.0)
    _check(lib().lckv_profile_read(cache, ctypes.byref(n), ctypes.byref(ms)), "lckv_profile_read")
    return n.value, ms.value


def lckv_profile_launch_ms(cache: int, capacity: int = 8192) -> np.ndarray:
    ms = np.zeros(capacity, np.float32)
    n = ctypes.c_int32(0)
    _check(lib().lckv_profile_launch_ms(cache, ms.ctypes.data, capacity, ctypes.byref(n)), "lckv_profile_launch_ms")
    return ms[: n.value].copy()
