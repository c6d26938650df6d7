"""lckv_step_static_scratch, the decode step for callers that cannot allocate device memory (no workspace
argument: the split partials live in the library's own static scratch array), against lckv_step on a twin cache.
Same kernels, so the outputs, the lengths and the caches must agree bit for bit - on two calls in a row, the
second on a smaller batch with shorter sequences (the scratch keeps the first call's contents), and both sides
must match the oracle."""
import numpy as np
import pytest
import torch

from oracle import lckv_oracle as orc
from paper_2405_10637_amd import binding as lk
from paper_2405_10637_amd import synth

from gpu_harness import GpuCache, check_close, to_f32_numpy

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("paged", [False, True])
def test_static_scratch_step_equals_the_step_with_a_workspace(paged):
    big = synth.Workload("na-big", "bf16", L=5, w=2, Hq=8, Hkv=2, D=128, B=6, T=400, sigma=1.0, seed=81, paged=paged)
    small = big.with_(name="na-small", B=3, T=90, seed=82)
    for wl, lens in ((big, [400, 399, 17, 0, 256, 130]), (small, [90, 1, 33])):      # second call: smaller input
        lens = np.asarray(lens, np.int32)
        print("static-scratch case", wl.name, "B", wl.B, "lens", list(lens), "paged", paged, flush=True)
        T_cap = wl.T + 16
        K, V = synth.logical_cache(wl, 3, T_cap)
        with GpuCache(wl, T_cap, lens, split_tokens=64) as ref, GpuCache(wl, T_cap, lens, split_tokens=64) as sta:
            for gc in (ref, sta):
                for s in range(3):
                    gc.load_dense(s, K[s, :, : wl.T], V[s, :, : wl.T])
            assert 0 < lk.lckv_workspace_bytes(sta.h, wl.B, wl.T + 2) <= lk.LCKV_STATIC_SCRATCH_BYTES
            Kf, Vf = to_f32_numpy(K), to_f32_numpy(V)
            lens_o = lens.copy()
            for step in range(2):
                q, kn, vn = synth.step_inputs(wl, 3, step=step)
                want_gpu = ref.step(q, kn, vn)
                qd, knd, vnd = q.cuda(), kn.cuda(), vn.cuda()
                out = torch.full_like(qd, float("nan"))
                lk.lckv_step_static_scratch(sta.h, qd, knd, vnd, out, sta.lens, wl.B, sta.max_len)
                torch.cuda.synchronize()
                sta.max_len += 1
                assert torch.equal(out, want_gpu), "%s step %d: differs from lckv_step" % (wl.name, step)
                assert torch.equal(sta.lens, ref.lens)
                want, _ = orc.step(wl.warmup_mask, Kf, Vf, lens_o, to_f32_numpy(q), to_f32_numpy(kn),
                                   to_f32_numpy(vn), 1.0 / np.sqrt(wl.D))
                check_close(out, want, "bf16", "%s step %d vs oracle" % (wl.name, step))
            assert torch.equal(sta.storage, ref.storage), "the caches differ"
            assert sta.device_error() == 0 and ref.device_error() == 0


def test_static_scratch_rejects_a_split_plan_that_does_not_fit():
    wl = synth.Workload("na-fit", "bf16", L=2, w=0, Hq=32, Hkv=32, D=128, B=128, T=4096, sigma=0.5, seed=83)
    cfg = lk.make_config(wl.L, wl.Hq, wl.Hkv, wl.D, lk.LCKV_BF16, wl.B, 4112, wl.warmup_mask)
    storage = torch.empty(lk.lckv_cache_bytes(cfg), dtype=torch.uint8, device="cuda")
    h = lk.lckv_cache_alloc(cfg, storage)
    try:
        lk.lckv_set_split_tokens(h, 256)                      # 17 splits x 128 x 32 rows x 128 channels of fp32: 35 MiB
        assert lk.lckv_workspace_bytes(h, wl.B, 4096) > lk.LCKV_STATIC_SCRATCH_BYTES
        t = torch.zeros(wl.L * wl.B * wl.Hq * wl.D, dtype=torch.bfloat16, device="cuda")
        lens = torch.zeros(wl.B, dtype=torch.int32, device="cuda")
        with pytest.raises(lk.LckvError) as e:
            lk.lckv_step_static_scratch(h, t, t, t, t, lens, wl.B, 4096)
        assert e.value.code == lk.LCKV_ERR_WORKSPACE
        torch.cuda.synchronize()
        assert int(lens.sum()) == 0                           # nothing ran
    finally:
        lk.lckv_cache_free(h)
