"""lckv_step_one_launch (the whole decode step in one resident kernel, layers separated by a device-wide barrier)
against lckv_step on a twin cache: same units of work, same arithmetic, so outputs, lengths and caches must agree
bit for bit - over several steps, contiguous and paged, both pairing rules, with and without splits, ragged lengths
including 0, the sink + window policy past several wrap-arounds - and both must match the oracle.  The barrier's
bounded wait is walked through by setting the bound to zero from the host: every workgroup leaves the kernel, the
sticky error bit is raised, nothing hangs, and the next step (with the normal bound) is right again."""
import numpy as np
import pytest
import torch

from oracle import lckv_oracle as orc
from paper_2405_10637_amd import binding as lk
from paper_2405_10637_amd import synth

from gpu_harness import GpuCache, check_close, to_f32_numpy

pytestmark = pytest.mark.gpu


def one_launch_step(gc, q, kn, vn, hint):
    qd, knd, vnd = q.cuda().contiguous(), kn.cuda().contiguous(), vn.cuda().contiguous()
    out = torch.full_like(qd, float("nan"))
    need = lk.lckv_step_one_launch_workspace_bytes(gc.h, gc.wl.B, hint)
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")
    ws.fill_(0xFF)
    lk.lckv_step_one_launch(gc.h, qd, knd, vnd, out, gc.lens, gc.wl.B, hint, ws)
    torch.cuda.synchronize()
    return out


CASES = [
    # name, workload kwargs, lens, T_cap, split_tokens, rule, sink, window, steps
    ("gqa64 splits", dict(L=5, w=2, Hq=16, Hkv=2, D=64, B=6), [300, 255, 256, 257, 31, 0], 320, 64, 0, 0, 0, 3),
    ("mha128 ragged rule2", dict(L=4, w=2, Hq=3, Hkv=3, D=128, B=7), [0, 1, 15, 16, 17, 100, 149], 160, 32, 1, 0, 0, 3),
    ("paged gqa2", dict(L=3, w=1, Hq=4, Hkv=2, D=128, B=5, paged=True), [200, 47, 48, 49, 0], 208, 48, 0, 0, 0, 3),
    ("single split, no warmup layers", dict(L=3, w=0, Hq=16, Hkv=1, D=64, B=3), [90, 5, 64], 96, 0, 0, 0, 0, 3),
    ("all warmup", dict(L=3, w=3, Hq=4, Hkv=4, D=64, B=3), [70, 0, 33], 80, 32, 0, 0, 0, 2),
    ("sink+window rule1", dict(L=4, w=2, Hq=4, Hkv=2, D=64, B=4), [0, 10, 31, 32], 32, 16, 0, 4, 28, 40),
    ("sink+window rule2 paged", dict(L=4, w=2, Hq=4, Hkv=2, D=128, B=3, paged=True), [45, 3, 20], 48, 16, 1, 4, 41, 60),
    ("more units than resident workgroups", dict(L=3, w=1, Hq=8, Hkv=8, D=64, B=40), None, 272, 16, 0, 0, 0, 2),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_one_launch_step_equals_the_layer_by_layer_step(case):
    name, kw, lens, T_cap, split, rule, sink, window, steps = case
    wl = synth.Workload("ol-" + name, "bf16", T=T_cap, sigma=1.0, seed=101 + len(name), **kw)
    if lens is None:
        lens = (np.arange(wl.B) * 37) % 257
    lens = np.asarray(lens, np.int32)
    print("one-launch case", name, "lens", list(lens)[:8], "split", split, "rule", rule, "sink", sink, "window", window,
          flush=True)
    T_hist = int(lens.max()) + steps + 1
    mk = lambda: GpuCache(wl, T_cap, lens, rule=rule, split_tokens=split, sink=sink, window=window)
    with mk() as ref, mk() as one:
        ns = ref.n_slots
        K, V = synth.logical_cache(wl, ns, max(T_hist, T_cap))
        Kf, Vf = to_f32_numpy(K), to_f32_numpy(V)
        n0 = int(lens.max())
        if n0 > 0:
            for gc in (ref, one):
                for s in range(ns):
                    gc.load_dense(s, K[s, :, :n0], V[s, :, :n0])
        lens_o = lens.copy()
        for step in range(steps):
            q, kn, vn = synth.step_inputs(wl, ns, step=step)
            hint = ref.max_len
            want_gpu = ref.step(q, kn, vn)
            got = one_launch_step(one, q, kn, vn, hint)
            assert torch.equal(got, want_gpu), "%s step %d: differs from lckv_step" % (name, step)
            assert torch.equal(one.lens, ref.lens)
            if step < 3 or step == steps - 1:
                want, _ = orc.step(wl.warmup_mask, Kf, Vf, lens_o, to_f32_numpy(q), to_f32_numpy(kn), to_f32_numpy(vn),
                                   1.0 / np.sqrt(wl.D), rule, sink=sink, window=window)
                check_close(got, want, "bf16", "%s step %d vs oracle" % (name, step))
            else:   # the oracle's history still has to advance
                orc.step(wl.warmup_mask, Kf, Vf, lens_o, to_f32_numpy(q), to_f32_numpy(kn), to_f32_numpy(vn),
                         1.0 / np.sqrt(wl.D), rule, sink=sink, window=window)
        assert torch.equal(one.storage, ref.storage), "the caches differ"
        assert one.device_error() == 0 and ref.device_error() == 0


def test_barrier_wait_is_bounded_and_reports():
    wl = synth.Workload("ol-bound", "bf16", L=4, w=2, Hq=8, Hkv=4, D=64, B=32, T=200, sigma=1.0, seed=131)
    lens = np.full(wl.B, 200, np.int32)
    K, V = synth.logical_cache(wl, 3, 208)
    with GpuCache(wl, 208, lens, split_tokens=64) as ref, GpuCache(wl, 208, lens, split_tokens=64) as one:
        for gc in (ref, one):
            for s in range(3):
                gc.load_dense(s, K[s, :, :200], V[s, :, :200])
        q, kn, vn = synth.step_inputs(wl, 3)
        lk.lckv_set_barrier_wait_ms(one.h, 0.0)             # the first workgroup to arrive gives up at once
        one_launch_step(one, q, kn, vn, 200)                # returns: no workgroup waits for ever
        assert one.device_error() & lk.LCKV_DEV_ERR_BARRIER
        assert one.device_error() == 0                      # reading cleared it
        # with the normal bound the same cache works again (the failed launch left its barrier counter dirty;
        # the next launch uses the other one and clears the first)
        lk.lckv_set_barrier_wait_ms(one.h, 2000.0)
        one.lens.copy_(torch.from_numpy(lens))
        for s in range(3):
            one.load_dense(s, K[s, :, :200], V[s, :, :200])
        for step in range(3):
            q, kn, vn = synth.step_inputs(wl, 3, step=step)
            want = ref.step(q, kn, vn)
            got = one_launch_step(one, q, kn, vn, 200 + step)
            assert torch.equal(got, want), "step %d after the failed launch" % step
        assert one.device_error() == 0
        with pytest.raises(lk.LckvError):
            lk.lckv_set_barrier_wait_ms(one.h, -1.0)


def test_one_launch_step_argument_errors():
    wl = synth.Workload("ol-err", "f32", L=2, w=1, Hq=2, Hkv=2, D=64, B=2, T=20, sigma=1.0, seed=132)
    with GpuCache(wl, 32, np.array([20, 3], np.int32)) as gc:
        q, kn, vn = [t.cuda() for t in synth.step_inputs(wl, gc.n_slots)]
        with pytest.raises(lk.LckvError) as e:              # bf16 caches only
            lk.lckv_step_one_launch(gc.h, q, kn, vn, torch.empty_like(q), gc.lens, 2, 20, None)
        assert e.value.code == lk.LCKV_ERR_CONFIG
    wl = wl.with_(dtype="bf16")
    with GpuCache(wl, 32, np.array([20, 3], np.int32), split_tokens=16) as gc:
        q, kn, vn = [t.cuda() for t in synth.step_inputs(wl, gc.n_slots)]
        need = lk.lckv_step_one_launch_workspace_bytes(gc.h, 2, 20)
        assert need == 2 * lk.lckv_workspace_bytes(gc.h, 2, 20) > 0
        ws = torch.empty(need - 256, dtype=torch.uint8, device="cuda")
        with pytest.raises(lk.LckvError) as e:
            lk.lckv_step_one_launch(gc.h, q, kn, vn, torch.empty_like(q), gc.lens, 2, 20, ws)
        assert e.value.code == lk.LCKV_ERR_WORKSPACE
        with pytest.raises(lk.LckvError) as e:
            lk.lckv_step_one_launch(gc.h, q, kn, vn, torch.empty_like(q), gc.lens, 2, 32, ws)
        assert e.value.code == lk.LCKV_ERR_LENGTH
        torch.cuda.synchronize()
        assert gc.lens.cpu().tolist() == [20, 3]
