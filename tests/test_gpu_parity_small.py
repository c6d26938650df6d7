"""GPU parity, small shapes: the HIP path (through the C ABI) against the CPU oracle, element by element, on
the same seeded inputs.  Shapes are small enough for the oracle to finish in seconds but span several pages,
several splits and ragged tails; the cache memory is poisoned with NaN patterns first."""
import numpy as np
import pytest
import torch

from oracle import lckv_oracle as orc
from paper_2405_10637_amd import binding as lk
from paper_2405_10637_amd import synth

from gpu_harness import GpuCache, bits, check_close, to_f32_numpy

pytestmark = pytest.mark.gpu


def run_case(wl, lens, T_cap, rule=0, split_tokens=0, steps=2, scale=0.0, waves=0, load_policy=0):
    """Load seeded caches, run `steps` decode steps on GPU and oracle, compare outputs, caches and lengths."""
    print("case", wl.name, wl.dtype, "L", wl.L, "H", wl.Hq, wl.Hkv, "D", wl.D, "B", wl.B, "lens", list(lens)[:8],
          "paged", wl.paged, "split", split_tokens, "rule", rule, "waves", waves, flush=True)
    lens = np.asarray(lens, np.int32)
    slot_o, vis_o, prod_o = orc.pairing(wl.warmup_mask, rule)
    with GpuCache(wl, T_cap, lens, rule=rule, split_tokens=split_tokens, scale=scale, waves=waves,
                  load_policy=load_policy) as gc:
        # pairing table of the library against the oracle's
        assert gc.n_slots == len(prod_o)
        for l in range(wl.L):
            assert lk.lckv_kv_slot(gc.h, l) == (int(slot_o[l]), int(vis_o[l]))
        for s in range(gc.n_slots):
            assert lk.lckv_slot_producer(gc.h, s) == int(prod_o[s])

        K, V = synth.logical_cache(wl, gc.n_slots, T_cap)           # [slots][B][T_cap][Hkv][D], cache dtype
        Kf, Vf = to_f32_numpy(K), to_f32_numpy(V)
        Tmax = int(lens.max())
        for s in range(gc.n_slots):
            if Tmax > 0:
                Kg, Vg = K[s, :, :Tmax].clone(), V[s, :, :Tmax].clone()
                for b in range(wl.B):                                # what lies beyond a sequence's length is NaN
                    Kg[b, lens[b]:] = float("nan")
                    Vg[b, lens[b]:] = float("nan")
                gc.load_dense(s, Kg, Vg)
        lens_o = lens.copy()
        eff_scale = scale if scale > 0 else 1.0 / np.sqrt(wl.D)
        worst = 0.0
        for step in range(steps):
            q, kn, vn = synth.step_inputs(wl, gc.n_slots, step=step)
            out = gc.step(q, kn, vn)
            want, _ = orc.step(wl.warmup_mask, Kf, Vf, lens_o, to_f32_numpy(q), to_f32_numpy(kn), to_f32_numpy(vn),
                               eff_scale, rule)
            worst = max(worst, check_close(out, want, wl.dtype, "%s step %d" % (wl.name, step)))
            assert (gc.lens.cpu().numpy() == lens_o).all()
        assert gc.device_error() == 0
        # cache contents: every logical position below the new lengths, bit for bit
        dt = np.uint16 if wl.dtype == "bf16" else np.uint32
        for s in range(gc.n_slots):
            for b in range(wl.B):
                n = int(lens_o[b])
                if n == 0:
                    continue
                k, v = gc.read(s, b, 0, n)
                # oracle's cache holds floats that came from the same bits: narrow them back exactly
                Kb = torch.from_numpy(Kf[s, b, :n]).to(wl.torch_dtype)
                Vb = torch.from_numpy(Vf[s, b, :n]).to(wl.torch_dtype)
                assert np.array_equal(k, bits(Kb).astype(dt).reshape(k.shape)), "K bits differ slot %d b %d" % (s, b)
                assert np.array_equal(v, bits(Vb).astype(dt).reshape(v.shape)), "V bits differ slot %d b %d" % (s, b)
    return worst


def test_c1_tiny_fp32_config():
    wl = synth.C1
    err = run_case(wl, synth.seq_lens(wl), T_cap=wl.T + 4, steps=3)
    print("C1 max-abs error", err)


@pytest.mark.parametrize("rule", [lk.LCKV_PAIR_TOP_OF_CONDENSED, lk.LCKV_PAIR_LAST_LAYER])
def test_bf16_mha_d128_ragged_with_forced_splits(rule):
    wl = synth.Workload("t-mha128", "bf16", L=4, w=2, Hq=3, Hkv=3, D=128, B=7, T=150, sigma=1.0, seed=11)
    run_case(wl, [0, 1, 15, 16, 17, 100, 149], T_cap=160, rule=rule, split_tokens=32, steps=2)


def test_bf16_gqa8_d64_ragged_with_forced_splits():
    wl = synth.Workload("t-gqa64", "bf16", L=5, w=2, Hq=16, Hkv=2, D=64, B=6, T=300, sigma=1.0, seed=12)
    run_case(wl, [300, 255, 256, 257, 31, 0], T_cap=310, split_tokens=64, steps=2)


def test_bf16_gqa2_d128_paged():
    wl = synth.Workload("t-gqa2-paged", "bf16", L=3, w=1, Hq=4, Hkv=2, D=128, B=5, T=200, sigma=1.0, seed=13,
                        paged=True)
    run_case(wl, [200, 47, 48, 49, 0], T_cap=208, split_tokens=48, steps=3)


def test_bf16_gqa16_d64_single_split_no_workspace():
    wl = synth.Workload("t-gqa16", "bf16", L=2, w=0, Hq=16, Hkv=1, D=64, B=3, T=90, sigma=1.0, seed=14)
    run_case(wl, [90, 5, 64], T_cap=96, steps=2)


def test_bf16_auto_split_plan_spans_several_splits():
    # D = 128, 4 units: the planner's own choice is three splits of 576 keys (workgroups of four waves)
    wl = synth.Workload("t-auto", "bf16", L=3, w=2, Hq=8, Hkv=2, D=128, B=2, T=1700, sigma=0.5, seed=15)
    with GpuCache(wl, 1704, np.array([1700, 700], np.int32)) as gc:
        assert lk.lckv_workspace_bytes(gc.h, 2, 1700) == 3 * 2 * 8 * 128 * 4 + 512
    run_case(wl, [1700, 700], T_cap=1704, steps=1)


def test_bf16_auto_plan_of_two_splits_becomes_one_workgroup_of_eight_waves():
    wl = synth.Workload("t-auto8", "bf16", L=3, w=2, Hq=8, Hkv=2, D=128, B=2, T=1100, sigma=0.5, seed=15)
    with GpuCache(wl, 1104, np.array([1100, 700], np.int32)) as gc:
        assert lk.lckv_workspace_bytes(gc.h, 2, 1100) == 0          # no split partials: the waves merge in LDS
        lk.lckv_set_workgroup_waves(gc.h, 4)
        assert lk.lckv_workspace_bytes(gc.h, 2, 1100) == 2 * 2 * 8 * 128 * 4 + 2 * 2 * 8 * 8
    run_case(wl, [1100, 700], T_cap=1104, steps=2)


def test_bf16_auto_plan_of_three_splits_becomes_one_workgroup_of_sixteen_waves_at_d64():
    wl = synth.Workload("t-auto16", "bf16", L=3, w=1, Hq=16, Hkv=2, D=64, B=3, T=3100, sigma=0.5, seed=19)
    with GpuCache(wl, 3104, np.array([3100, 0, 1500], np.int32)) as gc:
        assert lk.lckv_workspace_bytes(gc.h, 3, 3100) == 0
        lk.lckv_set_workgroup_waves(gc.h, 4)
        assert lk.lckv_workspace_bytes(gc.h, 3, 3100) > 0
    run_case(wl, [3100, 0, 1500], T_cap=3104, steps=2)


@pytest.mark.parametrize("waves,D,paged,split", [(8, 128, False, 0), (8, 128, True, 48), (8, 64, False, 0),
                                                 (16, 64, False, 0), (16, 64, True, 64), (16, 128, False, 0)],
                         ids=["w8-d128", "w8-d128-paged-splits", "w8-d64", "w16-d64", "w16-d64-paged-splits",
                              "w16-asked-at-d128-runs-as-8"])
def test_bf16_forced_workgroup_widths(waves, D, paged, split):
    """Workgroups of 8 and 16 waves, alone and together with splits, on ragged lengths: fewer pages than waves,
    none at all, a partly filled last page; with plain and with nontemporal loads (separate kernel variants)."""
    wl = synth.Workload("t-wide", "bf16", L=3, w=1, Hq=8, Hkv=2, D=D, B=7, T=300, sigma=1.0, seed=20 + waves + D,
                        paged=paged)
    for policy in (lk.LCKV_LOAD_TEMPORAL, lk.LCKV_LOAD_NONTEMPORAL):
        run_case(wl, [300, 0, 1, 16, 17, 129, 255], T_cap=304, split_tokens=split, steps=2, waves=waves,
                 load_policy=policy)


def test_bf16_all_warmup_is_standard_attention():
    wl = synth.Workload("t-allwarm", "bf16", L=3, w=3, Hq=4, Hkv=4, D=64, B=3, T=70, sigma=1.0, seed=16)
    run_case(wl, [70, 0, 33], T_cap=80, split_tokens=32, steps=2)


def test_f32_gqa4_d128_paged_with_forced_splits():
    wl = synth.Workload("t-f32-paged", "f32", L=3, w=1, Hq=8, Hkv=2, D=128, B=4, T=130, sigma=1.0, seed=17,
                        paged=True)
    run_case(wl, [130, 0, 17, 64], T_cap=144, split_tokens=32, steps=2)


def test_f32_custom_scale_d64():
    wl = synth.Workload("t-f32-scale", "f32", L=2, w=1, Hq=2, Hkv=2, D=64, B=2, T=50, sigma=1.0, seed=18)
    run_case(wl, [50, 9], T_cap=64, steps=2, scale=0.3)


def test_first_token_condensed_layers_give_exact_zeros():
    # Section 2.1: nothing visible for the first token in condensed layers; warmup layers return their own V.
    for dtype in ("bf16", "f32"):
        wl = synth.Workload("t-first", dtype, L=4, w=2, Hq=4, Hkv=2, D=64, B=2, T=1, sigma=1.0, seed=19)
        with GpuCache(wl, 32, np.zeros(2, np.int32)) as gc:
            q, kn, vn = synth.step_inputs(wl, gc.n_slots)
            out = gc.step(q, kn, vn).cpu()
            assert (out[1] == 0).all() and (out[2] == 0).all()
            for l, s in [(0, 0), (3, 2)]:
                for h in range(wl.Hq):
                    assert torch.equal(out[l, :, h], vn[s, :, h // 2]), "warmup layer must return the new value"


def test_needles_at_page_and_split_edges():
    # One key aligned with q takes all the mass: the output names the position that was read.  Positions sweep
    # page edges (15,16,17), split edges (47,48,49 with 48-token splits), first, last cached, and the new token.
    T = 100
    for dtype, tol in (("bf16", 2e-2), ("f32", 1e-5)):
        for paged in (False, True):
            wl = synth.Workload("t-needle", dtype, L=2, w=1, Hq=2, Hkv=2, D=128, B=1, T=T, sigma=1.0, seed=20,
                                paged=paged, warm=(0,))
            for pos in [0, 15, 16, 17, 47, 48, 49, 95, 96, 99, 100]:
                with GpuCache(wl, 112, np.array([T], np.int32), split_tokens=48) as gc:
                    K, V = synth.logical_cache(wl, 2, T)
                    q, kn, vn = synth.step_inputs(wl, 2)
                    for l, s in [(0, 0), (1, 1)]:
                        for h in range(2):
                            needle = (6.0 * q[l, 0, h].float() / q[l, 0, h].float().norm()).to(wl.torch_dtype)
                            if pos < T:
                                K[s, 0, pos, h] = needle        # score = 6|q|/sqrt(128)*... dominates by > e^30
                            else:
                                kn[s, 0, h] = needle
                    q = q * 8.0
                    gc.load_dense(0, K[0], V[0])
                    gc.load_dense(1, K[1], V[1])
                    out = gc.step(q, kn, vn).cpu().float()
                    Vall = [torch.cat([V[s, 0], vn[s]], 0).float() for s in range(2)]   # [T+1][Hkv][D]
                    err0 = (out[0, 0] - Vall[0][pos]).abs().max().item()
                    assert err0 <= tol, "warmup layer, needle at %d (%s, paged=%s): err %.3g" % (pos, dtype, paged, err0)
                    if pos < T:
                        err1 = (out[1, 0] - Vall[1][pos]).abs().max().item()
                        assert err1 <= tol, "condensed layer, needle at %d: err %.3g" % (pos, err1)
                    else:   # the diagonal is masked: the condensed layer must NOT see the new token
                        assert (out[1, 0] - Vall[1][pos]).abs().max().item() > 0.1


def test_huge_scores_do_not_overflow():
    wl = synth.Workload("t-huge", "bf16", L=1, w=0, Hq=2, Hkv=2, D=128, B=1, T=64, sigma=1.0, seed=21)
    with GpuCache(wl, 80, np.array([64], np.int32), split_tokens=32) as gc:
        K, V = synth.logical_cache(wl, 1, 64)
        q, kn, vn = synth.step_inputs(wl, 1)
        for h in range(2):
            u = q[0, 0, h].float() / q[0, 0, h].float().norm()
            K[0, 0, 40, h] = (900.0 * u).to(torch.bfloat16)      # raw score ~ +900 * |q|: exp overflows fp32
            K[0, 0, 7, h] = (-900.0 * u).to(torch.bfloat16)
        gc.load_dense(0, K[0], V[0])
        out = gc.step(q, kn, vn).cpu().float()
        assert torch.isfinite(out).all()
        assert (out[0, 0] - V[0, 0, 40].float()).abs().max().item() <= 2e-2


def test_condensed_layers_with_equal_queries_give_bitwise_equal_outputs_and_batch_order_does_not_matter():
    wl = synth.Workload("t-share", "bf16", L=5, w=2, Hq=8, Hkv=2, D=64, B=6, T=333, sigma=1.0, seed=22)
    lens = np.array([333, 1, 100, 257, 64, 200], np.int32)
    perm = np.array([4, 0, 5, 2, 1, 3])
    K, V = synth.logical_cache(wl, 3, 333)
    q, kn, vn = synth.step_inputs(wl, 3)
    q[2] = q[1]
    q[3] = q[1]
    outs = []
    for order in (np.arange(6), perm):
        with GpuCache(wl, 340, lens[order], split_tokens=64) as gc:
            for s in range(3):
                gc.load_dense(s, K[s][order], V[s][order])
            outs.append(gc.step(q[:, order], kn[:, order], vn[:, order]).cpu())
    assert torch.equal(outs[0][1], outs[0][2]) and torch.equal(outs[0][1], outs[0][3])   # one shared cache
    assert torch.equal(outs[0][:, perm], outs[1])                                        # bitwise


@pytest.mark.parametrize("D,Hq,Hkv", [(128, 8, 4), (64, 16, 2), (64, 4, 4)])
@pytest.mark.parametrize("paged", [False, True])
def test_load_policy_does_not_change_a_bit(D, Hq, Hkv, paged):
    # plain and nontemporal loads read the same bytes: outputs must be bitwise equal (contiguous and paged, both
    # head dimensions, grouped and ungrouped heads), and the forced-nontemporal result must match the oracle
    wl = synth.Workload("t-policy", "bf16", L=3, w=1, Hq=Hq, Hkv=Hkv, D=D, B=3, T=260, sigma=1.0, seed=25,
                        paged=paged)
    lens = np.array([260, 33, 128], np.int32)
    K, V = synth.logical_cache(wl, 2, 272)
    q, kn, vn = synth.step_inputs(wl, 2)
    outs = []
    for policy in (lk.LCKV_LOAD_TEMPORAL, lk.LCKV_LOAD_NONTEMPORAL):
        with GpuCache(wl, 272, lens, split_tokens=64, load_policy=policy) as gc:
            for s in range(2):
                gc.load_dense(s, K[s, :, :260], V[s, :, :260])
            outs.append(gc.step(q, kn, vn).cpu())
            assert gc.device_error() == 0
    assert torch.equal(outs[0], outs[1]) and torch.isfinite(outs[0].float()).all()
    want, _ = orc.step(wl.warmup_mask, to_f32_numpy(K), to_f32_numpy(V), lens.copy(), to_f32_numpy(q),
                       to_f32_numpy(kn), to_f32_numpy(vn), 1.0 / np.sqrt(D))
    check_close(outs[1], want, "bf16", "nontemporal loads, D=%d paged=%s" % (D, paged))


def test_new_shared_kv_is_invisible_now_and_visible_next_step():
    # Section 2.1 (diagonal mask): the K/V appended to the shared slot this step change no condensed output
    # this step and change them at the next step.
    wl = synth.Workload("t-diag", "bf16", L=4, w=1, Hq=2, Hkv=2, D=64, B=2, T=40, sigma=1.0, seed=23, warm=(0,))
    lens = np.array([40, 16], np.int32)
    K, V = synth.logical_cache(wl, 2, 40)
    q, kn, vn = synth.step_inputs(wl, 2)
    res = []
    for factor in (1.0, -2.0):
        kn2, vn2 = kn.clone(), vn.clone()
        kn2[1] *= factor
        vn2[1] *= factor
        with GpuCache(wl, 48, lens) as gc:
            gc.load_dense(0, K[0], V[0])
            gc.load_dense(1, K[1], V[1])
            o1 = gc.step(q, kn2, vn2).cpu()
            o2 = gc.step(q, kn2, vn2).cpu()
            res.append((o1, o2))
    assert torch.equal(res[0][0], res[1][0])
    assert torch.equal(res[0][1][0], res[1][1][0])
    assert (res[0][1][1:].float() - res[1][1][1:].float()).abs().amax(-1).min().item() > 0


def test_call_errors_found_on_the_host_and_device_error_word():
    wl = synth.Workload("t-err", "bf16", L=3, w=1, Hq=2, Hkv=2, D=64, B=2, T=20, sigma=1.0, seed=24, warm=(0,))
    with GpuCache(wl, 32, np.array([20, 3], np.int32)) as gc:
        q, kn, vn = [t.cuda() for t in synth.step_inputs(wl, gc.n_slots)]
        out = torch.empty_like(q)
        L = lk.lib()
        st = torch.cuda.current_stream().cuda_stream or None

        def step_rc(B=2, hint=20, lens=gc.lens, qq=q):
            return L.lckv_step(gc.h, qq.data_ptr(), kn.data_ptr(), vn.data_ptr(), out.data_ptr(), lens.data_ptr(),
                               B, hint, None, 0, st)

        assert step_rc(B=3) == lk.LCKV_ERR_BATCH
        assert step_rc(B=0) == lk.LCKV_ERR_BATCH
        assert step_rc(hint=32) == lk.LCKV_ERR_LENGTH            # no room for the new token
        assert step_rc(hint=-1) == lk.LCKV_ERR_LENGTH
        assert L.lckv_step(gc.h, q.data_ptr() + 2, kn.data_ptr(), vn.data_ptr(), out.data_ptr(), gc.lens.data_ptr(),
                           2, 20, None, 0, st) == lk.LCKV_ERR_ALIGN
        assert L.lckv_append_kv(gc.h, 1, kn.data_ptr(), vn.data_ptr(), gc.lens.data_ptr(), 2, st) == \
            lk.LCKV_ERR_NOT_PRODUCER                               # layer 1 is condensed and not the top one
        assert L.lckv_append_kv(gc.h, 5, kn.data_ptr(), vn.data_ptr(), gc.lens.data_ptr(), 2, st) == lk.LCKV_ERR_LAYER
        bad_mask = np.array([0, 1, 0], np.uint8)
        assert L.lckv_decode_attention(gc.h, 0, q.data_ptr(), out.data_ptr(), gc.lens.data_ptr(), bad_mask.ctypes.data,
                                       2, 20, None, 0, st) == lk.LCKV_ERR_MASK
        lk.lckv_set_split_tokens(gc.h, 16)                         # several splits now need a workspace
        assert L.lckv_decode_attention(gc.h, 0, q.data_ptr(), out.data_ptr(), gc.lens.data_ptr(), None, 2, 20, None, 0,
                                       st) == lk.LCKV_ERR_WORKSPACE
        lk.lckv_set_split_tokens(gc.h, 0)
        k = np.zeros((1, 2, 64), np.uint16)
        with pytest.raises(lk.LckvError) as e:
            lk.lckv_cache_read(gc.h, 0, 0, 32, 1, k, k.copy())
        assert e.value.code == lk.LCKV_ERR_RANGE
        assert gc.device_error() == 0
        # a device-side length beyond the host's bound is clamped and reported, not followed out of bounds
        big = torch.tensor([31, 40], dtype=torch.int32, device="cuda")
        assert step_rc(hint=31, lens=big) == lk.LCKV_OK
        torch.cuda.synchronize()
        assert gc.device_error() & lk.LCKV_DEV_ERR_CAPACITY
        assert gc.device_error() == 0                              # reading clears it
    wlp = wl.with_(paged=True)
    with GpuCache(wlp, 32, np.array([20, 3], np.int32)) as gc:
        q, kn, vn = synth.step_inputs(wlp, gc.n_slots)
        K, V = synth.logical_cache(wlp, gc.n_slots, 20)
        for s in range(gc.n_slots):
            gc.load_dense(s, K[s], V[s])
        gc.table[1, 0] = 10 ** 6                                   # a block id outside the pool
        out = gc.step(q, kn, vn)
        assert gc.device_error() & lk.LCKV_DEV_ERR_BLOCK
        assert torch.isfinite(out[:, 0].float()).all()


def test_step_captured_in_a_hip_graph_replays_like_eager_steps():
    # lckv_step neither allocates nor synchronises, so a caller may capture it once (with a loose length bound)
    # and replay it for successive tokens: lengths advance on the device inside the graph.  Every replay is
    # checked against an eager step on a twin cache, with the program's own eager work between the replays.
    wl = synth.Workload("t-graph", "bf16", L=4, w=2, Hq=8, Hkv=2, D=64, B=3, T=150, sigma=1.0, seed=26)
    lens = np.array([150, 40, 97], np.int32)
    K, V = synth.logical_cache(wl, 3, 150)
    with GpuCache(wl, 176, lens, split_tokens=64) as eager, GpuCache(wl, 176, lens, split_tokens=64) as graphed:
        for gc in (eager, graphed):
            for s in range(3):
                gc.load_dense(s, K[s], V[s])
        q0, kn0, vn0 = synth.step_inputs(wl, 3)
        sq, sk, sv = q0.cuda(), kn0.cuda(), vn0.cuda()           # static buffers the graph reads
        sout = torch.zeros_like(sq)
        ws = graphed.workspace(170)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            lk.lckv_step(graphed.h, sq, sk, sv, sout, graphed.lens, wl.B, 170, ws)
        # capturing does not execute: lengths must be unchanged
        assert (graphed.lens.cpu().numpy() == lens).all()
        for step in range(5):
            q, kn, vn = synth.step_inputs(wl, 3, step=step)
            sq.copy_(q)
            sk.copy_(kn)
            sv.copy_(vn)
            g.replay()
            want = eager.step(q, kn, vn)                           # eager work and a sync between replays
            torch.cuda.synchronize()
            assert torch.equal(sout.cpu(), want.cpu()), "replay %d differs from the eager step" % step
            assert (graphed.lens.cpu().numpy() == lens + step + 1).all()
        assert graphed.device_error() == 0 and eager.device_error() == 0


def test_per_layer_entry_points_compose_to_the_step():
    # lckv_append_kv + lckv_decode_attention called layer by layer (producers appended first, lengths bumped by
    # the caller) must give exactly what lckv_step gives, and must match the oracle.
    for paged in (False, True):
        wl = synth.Workload("t-layered", "bf16", L=5, w=2, Hq=8, Hkv=4, D=128, B=4, T=90, sigma=1.0, seed=27,
                            paged=paged)
        lens = np.array([90, 0, 31, 64], np.int32)
        K, V = synth.logical_cache(wl, 3, 96)
        q, kn, vn = synth.step_inputs(wl, 3)
        with GpuCache(wl, 96, lens, split_tokens=32) as a, GpuCache(wl, 96, lens, split_tokens=32) as b:
            for gc in (a, b):
                for s in range(3):
                    gc.load_dense(s, K[s, :, :90], V[s, :, :90])
            want_step = a.step(q, kn, vn)
            qd, knd, vnd = q.cuda(), kn.cuda(), vn.cuda()
            out = torch.full_like(qd, float("nan"))
            ws = b.workspace(91)
            for l in range(wl.L):
                for s in range(b.n_slots):
                    if lk.lckv_slot_producer(b.h, s) == l:
                        lk.lckv_append_kv(b.h, l, knd[s], vnd[s], b.lens, wl.B)
                lk.lckv_decode_attention(b.h, l, qd[l], out[l], b.lens, wl.warmup_mask, wl.B, 90, ws)
            torch.cuda.synchronize()
            assert torch.equal(out.cpu(), want_step.cpu())
            assert (b.lens.cpu().numpy() == lens).all()          # only lckv_step bumps the lengths
            want, _ = orc.step(wl.warmup_mask, to_f32_numpy(K), to_f32_numpy(V), lens.copy(), to_f32_numpy(q),
                               to_f32_numpy(kn), to_f32_numpy(vn), 1.0 / np.sqrt(wl.D))
            check_close(out, want, "bf16", "per-layer calls")
            assert a.device_error() == 0 and b.device_error() == 0


def test_batch_smaller_than_capacity_and_group_of_16():
    # B < B_max, and G = 16 query heads per kv head (all 16 columns of the matrix tile in use)
    wl_cap = synth.Workload("t-cap", "bf16", L=3, w=1, Hq=32, Hkv=2, D=64, B=6, T=70, sigma=1.0, seed=28)
    wl = wl_cap.with_(B=3)
    lens = np.array([70, 17, 48, 0, 0, 0], np.int32)
    K, V = synth.logical_cache(wl_cap, 2, 80)
    with GpuCache(wl_cap, 80, lens, split_tokens=32) as gc:
        for s in range(2):
            gc.load_dense(s, K[s, :, :70], V[s, :, :70])
        q, kn, vn = synth.step_inputs(wl, 2)
        qd, knd, vnd = q.cuda(), kn.cuda(), vn.cuda()
        out = torch.full_like(qd, float("nan"))
        lk.lckv_step(gc.h, qd, knd, vnd, out, gc.lens, 3, 70, gc.workspace(71))
        torch.cuda.synchronize()
        lens3 = lens[:3].copy()
        want, _ = orc.step(wl.warmup_mask, to_f32_numpy(K[:, :3]), to_f32_numpy(V[:, :3]), lens3, to_f32_numpy(q),
                           to_f32_numpy(kn), to_f32_numpy(vn), 1.0 / np.sqrt(wl.D))
        check_close(out, want, "bf16", "B < B_max, G = 16")
        assert gc.lens.cpu().numpy().tolist() == [71, 18, 49, 0, 0, 0]       # the other sequences are untouched
        assert gc.device_error() == 0
