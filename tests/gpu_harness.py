"""Test-side plumbing for the GPU parity tests: device buffers (torch), the cache handle, and conversion of the
same seeded inputs to what the CPU oracle takes.  No arithmetic of the method lives here."""
from __future__ import annotations

import numpy as np
import torch

from paper_2405_10637_amd import binding as lk
from paper_2405_10637_amd import synth

DEV = "cuda"


def lk_dtype(wl):
    return lk.LCKV_BF16 if wl.dtype == "bf16" else lk.LCKV_F32


def to_f32_numpy(t: torch.Tensor) -> np.ndarray:
    """Exact widening of bf16/fp32 tensors to float32 numpy (what the oracle takes)."""
    return np.ascontiguousarray(t.detach().cpu().float().numpy())


def bits(t: torch.Tensor) -> np.ndarray:
    """Bit patterns of a bf16/fp32 tensor as uint16/uint32 numpy."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.view(torch.int32).numpy().view(np.uint32)


class GpuCache:
    """A cache on the GPU for workload `wl`: storage poisoned with NaN bit patterns, optional block table."""

    def __init__(self, wl: synth.Workload, T_cap: int, lens: np.ndarray, rule=lk.LCKV_PAIR_TOP_OF_CONDENSED,
                 split_tokens: int = 0, scale: float = 0.0, poison: bool = True, load_policy: int = 0, waves: int = 0,
                 sink: int = 0, window: int = 0):
        self.wl = wl
        self.lens0 = np.asarray(lens, np.int32).copy()
        self.table = None
        if wl.paged:
            table, num_blocks = synth.block_table(wl, np.full(wl.B, T_cap - 1, np.int32))
            self.cfg = lk.make_config(wl.L, wl.Hq, wl.Hkv, wl.D, lk_dtype(wl), wl.B, 0, wl.warmup_mask, page_size=16,
                                      num_blocks=num_blocks, pairing_rule=rule, scale=scale, sink_tokens=sink,
                                      window_tokens=window)
            self.table = torch.from_numpy(table).to(DEV)
            self.capacity = table.shape[1] * 16
        else:
            self.cfg = lk.make_config(wl.L, wl.Hq, wl.Hkv, wl.D, lk_dtype(wl), wl.B, T_cap, wl.warmup_mask,
                                      pairing_rule=rule, scale=scale, sink_tokens=sink, window_tokens=window)
            self.capacity = (T_cap + 15) // 16 * 16
        nbytes = lk.lckv_cache_bytes(self.cfg)
        self.storage = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
        if poison:
            self.storage.fill_(0xFF)  # every bf16 / fp32 there is a NaN: stale data must never reach a result
        self.h = lk.lckv_cache_alloc(self.cfg, self.storage)
        if self.table is not None:
            lk.lckv_cache_set_block_table(self.h, self.table, self.table.shape[1])
        if split_tokens:
            lk.lckv_set_split_tokens(self.h, split_tokens)
        if waves:
            lk.lckv_set_workgroup_waves(self.h, waves)
        lk.lckv_set_load_policy(self.h, load_policy)
        self.n_slots = lk.lckv_n_slots(self.h)
        self.lens = torch.from_numpy(self.lens0).to(DEV)
        self.max_len = int(self.lens0.max())
        self._ws = None

    def close(self):
        if self.h:
            lk.lckv_cache_free(self.h)
            self.h = None

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.close()

    def workspace(self, max_len_hint):
        need = lk.lckv_workspace_bytes(self.h, self.wl.B, max_len_hint)
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty(max(need, 256), dtype=torch.uint8, device=DEV)
        return self._ws

    def load_dense(self, slot: int, K: torch.Tensor, V: torch.Tensor):
        """K, V: [B][T][Hkv][D] tensors (any device) in the cache dtype."""
        K = K.to(DEV).contiguous()
        V = V.to(DEV).contiguous()
        lk.lckv_cache_load_dense(self.h, slot, K, V, None, K.shape[0], K.shape[1])
        torch.cuda.synchronize()

    def step(self, q, k_new, v_new, max_len_hint=None):
        q, k_new, v_new = q.to(DEV).contiguous(), k_new.to(DEV).contiguous(), v_new.to(DEV).contiguous()
        out = torch.full_like(q, float("nan"))
        hint = self.max_len if max_len_hint is None else max_len_hint
        ws = self.workspace(hint)
        lk.lckv_step(self.h, q, k_new, v_new, out, self.lens, self.wl.B, hint, ws)
        torch.cuda.synchronize()
        self.max_len += 1
        return out

    def read(self, slot, b, pos, n_pos):
        dt = np.uint16 if self.wl.dtype == "bf16" else np.uint32
        k = np.zeros((n_pos, self.wl.Hkv, self.wl.D), dt)
        v = np.zeros_like(k)
        lk.lckv_cache_read(self.h, slot, b, pos, n_pos, k, v)
        return k, v

    def device_error(self):
        return lk.lckv_last_device_error(self.h)


def check_close(got: torch.Tensor, want: np.ndarray, dtype: str, what: str = ""):
    """The parity bar: max-abs error 2e-2 for bf16 inputs, 1e-5 in fp32 mode, plus (bf16) a bound on the error
    relative to the largest expected magnitude, because with near-uniform softmax rows the outputs themselves
    are smaller than 2e-2."""
    g = got.detach().cpu().double().numpy()
    assert np.isfinite(g).all(), what + ": non-finite output"
    err = np.abs(g - want).max()
    ref = np.abs(want).max()
    if dtype == "bf16":
        assert err <= 2e-2, "%s: max-abs error %.3g > 2e-2" % (what, err)
        assert err <= 1e-2 * max(ref, 1e-3), "%s: max-abs error %.3g vs max |expected| %.3g" % (what, err, ref)
    else:
        assert err <= 1e-5, "%s: max-abs error %.3g > 1e-5" % (what, err)
    return err
