"""Device-side plumbing for running LCKV decode steps on a named synthetic workload: owns the torch buffers
(cache storage, lengths, block table, workspace), fills the cache from seeded dense tensors through
lckv_cache_load_dense, and calls lckv_step.  Used by bench.py and the full-size GPU tests.  No arithmetic of the
method lives here, and nothing here knows the cache's physical layout."""
from __future__ import annotations

from typing import Dict, Iterable, Tuple

import numpy as np
import torch

from . import binding as lk
from . import synth

DEV = "cuda"


class DecodeSession:
    def __init__(self, wl: synth.Workload, room: int = 16, rule: int = lk.LCKV_PAIR_TOP_OF_CONDENSED,
                 split_tokens: int = 0, waves: int = 0):
        """`room`: how many decode steps the cache must be able to take beyond the initial lengths."""
        self.wl = wl
        self.lens0 = synth.seq_lens(wl)
        dtype = lk.LCKV_BF16 if wl.dtype == "bf16" else lk.LCKV_F32
        self.table = None
        if wl.paged:
            table, num_blocks = synth.block_table(wl, self.lens0, extra_tokens=room)
            self.cfg = lk.make_config(wl.L, wl.Hq, wl.Hkv, wl.D, dtype, wl.B, 0, wl.warmup_mask, page_size=16,
                                      num_blocks=num_blocks, pairing_rule=rule)
            self.table = torch.from_numpy(table).to(DEV)
        else:
            self.cfg = lk.make_config(wl.L, wl.Hq, wl.Hkv, wl.D, dtype, wl.B, int(self.lens0.max()) + room,
                                      wl.warmup_mask, pairing_rule=rule)
        self.cache_bytes = lk.lckv_cache_bytes(self.cfg)
        self.storage = torch.empty(self.cache_bytes, dtype=torch.uint8, device=DEV)
        self.h = lk.lckv_cache_alloc(self.cfg, self.storage)
        if self.table is not None:
            lk.lckv_cache_set_block_table(self.h, self.table, self.table.shape[1])
        if split_tokens:
            lk.lckv_set_split_tokens(self.h, split_tokens)
        if waves:
            lk.lckv_set_workgroup_waves(self.h, waves)
        self.n_slots = lk.lckv_n_slots(self.h)
        self.kv_slot = [lk.lckv_kv_slot(self.h, l) for l in range(wl.L)]      # (slot, self_visible) per layer
        self.producer = [lk.lckv_slot_producer(self.h, s) for s in range(self.n_slots)]
        self.lens = torch.from_numpy(self.lens0).to(DEV)
        self.max_len = int(self.lens0.max())
        self.steps_left = room
        self.import_GBps = []     # read + write rate of each lckv_cache_load_dense call made by fill()
        ws = max(lk.lckv_workspace_bytes(self.h, wl.B, self.max_len + i) for i in range(room + 1))
        if wl.dtype == "bf16":   # the one-launch step sizes its own (two sets of partials, workgroups of four waves)
            ws = max([ws] + [lk.lckv_step_one_launch_workspace_bytes(self.h, wl.B, self.max_len + i) for i in range(room + 1)])
        self.workspace = torch.empty(max(ws, 256), dtype=torch.uint8, device=DEV)

    def close(self):
        if self.h:
            lk.lckv_cache_free(self.h)
            self.h = None
        self.storage = None

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.close()

    def fill(self, units: Iterable[Tuple[int, int, int]] = (), keep_dense: bool = False):
        """Fill every slot with sigma*N(0,1) values (seeded per slot) and return, for each requested
        (layer, b, query head) unit, the float32 copies of the K and V rows that unit's layer reads:
        arrays [lens0[b]][D] taken from the dense tensors BEFORE they enter the cache.  With `keep_dense` the
        dense tensors [B][T][Hkv][D] of every slot are also returned as CPU tensors (small workloads only)."""
        wl = self.wl
        T = int(self.lens0.max())
        G = wl.G
        by_slot: Dict[int, list] = {}
        for u in units:
            by_slot.setdefault(self.kv_slot[u[0]][0], []).append(u)
        got = {}
        dense = []
        shape = (wl.B, T, wl.Hkv, wl.D)
        for s in range(self.n_slots):
            Kd = torch.empty(shape, dtype=wl.torch_dtype, device=DEV)
            Vd = torch.empty(shape, dtype=wl.torch_dtype, device=DEV)
            synth.fill_normal_(Kd, wl.sigma, wl.seed * 31 + 2 * s)
            synth.fill_normal_(Vd, wl.sigma, wl.seed * 31 + 2 * s + 1)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            lk.lckv_cache_load_dense(self.h, s, Kd, Vd, self.lens, wl.B, T)
            e1.record()
            e1.synchronize()
            moved = 2 * 2 * int(self.lens0.astype(np.int64).sum()) * wl.Hkv * wl.D * wl.elem_bytes  # read + written
            self.import_GBps.append(moved / (e0.elapsed_time(e1) * 1e-3) / 1e9)
            for (l, b, h) in by_slot.get(s, []):
                n = int(self.lens0[b])
                got[(l, b, h)] = (Kd[b, :n, h // G].float().cpu().numpy(), Vd[b, :n, h // G].float().cpu().numpy())
            torch.cuda.synchronize()
            if keep_dense:
                dense.append((Kd.cpu(), Vd.cpu()))
            del Kd, Vd
        return (got, dense) if keep_dense else got

    def step(self, q, k_new, v_new, out):
        assert self.steps_left > 0, "cache capacity used up"
        lk.lckv_step(self.h, q, k_new, v_new, out, self.lens, self.wl.B, self.max_len, self.workspace)
        self.max_len += 1
        self.steps_left -= 1

    def step_one_launch(self, q, k_new, v_new, out):
        """The same step through lckv_step_one_launch (bf16 caches)."""
        assert self.steps_left > 0, "cache capacity used up"
        lk.lckv_step_one_launch(self.h, q, k_new, v_new, out, self.lens, self.wl.B, self.max_len, self.workspace)
        self.max_len += 1
        self.steps_left -= 1

    def kv_bytes_per_step(self, step_index: int = 0) -> int:
        """Algorithmic K/V bytes one step streams: sum over layers and sequences of visible keys * 2*Hkv*D*E."""
        wl = self.wl
        per_key = 2 * wl.Hkv * wl.D * wl.elem_bytes
        tot = 0
        for l in range(wl.L):
            n = self.lens0.astype(np.int64) + step_index + self.kv_slot[l][1]
            tot += int(n.sum()) * per_key
        return tot

    def step_chained(self, q_seed, k_new, v_new, q_work, out):
        """One decode step through the per-layer entry points with the model's layer-to-layer dependency made
        physical: layer l's query is q_seed[l] + out[l-1] (the residual stream carries layer l-1's attention
        output into layer l's query; Section 2.1, "bottom-up computation"), so no layer can start before the
        previous one has finished.  q_work receives the queries actually used.  The adds are plain torch ops on
        the same stream; appends and attention go through lckv_append_kv / lckv_decode_attention."""
        assert self.steps_left > 0, "cache capacity used up"
        wl = self.wl
        for l in range(wl.L):
            q_work[l].copy_(q_seed[l])
            if l > 0:
                q_work[l].add_(out[l - 1])
            slot, vis = self.kv_slot[l]
            mine = [s for s in range(self.n_slots) if self.producer[s] == l]
            if vis:      # a warmup layer sees itself: its K/V go in first
                for s in mine:
                    lk.lckv_append_kv(self.h, l, k_new[s], v_new[s], self.lens, wl.B)
            lk.lckv_decode_attention(self.h, l, q_work[l], out[l], self.lens, None, wl.B, self.max_len,
                                     self.workspace)
            if not vis:  # the shared slot's new K/V are invisible to this step's condensed layers
                for s in mine:
                    lk.lckv_append_kv(self.h, l, k_new[s], v_new[s], self.lens, wl.B)
        self.lens.add_(1)
        self.max_len += 1
        self.steps_left -= 1
