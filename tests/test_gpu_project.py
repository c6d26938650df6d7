"""GPU parity of lckv_project_qkv (Section 2.1: queries for every layer, keys and values - stored straight into
the cache - for producing layers only; rotary embedding at position t_b) against the oracle, element by element:
ragged positions including 0, batches that are not a multiple of 16 and that need two passes, GQA, D = 64 and 128,
contiguous and paged caches, bf16 and fp32, no rotation; then whole decode steps built from the projection and
the attention entry points against the same composition of oracle functions."""
import numpy as np
import pytest
import torch

from oracle import lckv_oracle as orc
from paper_2405_10637_amd import binding as lk
from paper_2405_10637_amd import synth

from gpu_harness import GpuCache, check_close, to_f32_numpy

pytestmark = pytest.mark.gpu


def cache_rows_f32(gc, slot, b, pos):
    """K and V of one position as float32 [Hkv][D]."""
    k, v = gc.read(slot, b, pos, 1)
    if gc.wl.dtype == "bf16":
        k, v = (k.astype(np.uint32) << 16), (v.astype(np.uint32) << 16)
    return k.view(np.float32)[0], v.view(np.float32)[0]


def weights(wl, hidden, layer, producer):
    n = lambda rows, seed: synth._normal((rows, hidden), 1.0 / np.sqrt(hidden), wl.torch_dtype, seed)
    wq = n(wl.Hq * wl.D, wl.seed + 100 * layer + 1)
    if not producer:
        return wq, None, None
    return wq, n(wl.Hkv * wl.D, wl.seed + 100 * layer + 2), n(wl.Hkv * wl.D, wl.seed + 100 * layer + 3)


def packed(h, w):
    """Row-major weight (CPU tensor) -> the device image lckv_project_qkv takes."""
    if w is None:
        return None
    wd = w.cuda().contiguous()
    wp = torch.full_like(wd, float("nan"))
    lk.lckv_pack_projection_weight(h, wd, wp, w.shape[0], w.shape[1])
    return wp


def run_project(wl, hidden, lens, T_cap, rope_base=10000.0):
    print("project case", wl.name, wl.dtype, "H", wl.Hq, wl.Hkv, "D", wl.D, "hidden", hidden, "lens", list(lens)[:8],
          "paged", wl.paged, "base", rope_base, flush=True)
    lens = np.asarray(lens, np.int32)
    with GpuCache(wl, T_cap, lens) as gc:
        ws = torch.empty(lk.lckv_project_workspace_bytes(gc.h, wl.B, hidden), dtype=torch.uint8, device="cuda")
        ws.fill_(0xFF)                                            # the call must not rely on a cleared workspace
        producers = {lk.lckv_slot_producer(gc.h, s): s for s in range(gc.n_slots)}
        pos = lens if rope_base > 0 else None
        for layer in range(wl.L):
            x = synth._normal((wl.B, hidden), 1.0, wl.torch_dtype, wl.seed + 7 * layer)
            wq, wk, wv = weights(wl, hidden, layer, layer in producers)
            dev = lambda t: packed(gc.h, t)
            before = gc.storage.clone()
            q_out = torch.full((wl.B, wl.Hq, wl.D), float("nan"), dtype=wl.torch_dtype, device="cuda")
            lk.lckv_project_qkv(gc.h, layer, x.cuda(), hidden, dev(wq), dev(wk), dev(wv), q_out, gc.lens, wl.B,
                                rope_base, ws)
            torch.cuda.synchronize()
            xf = to_f32_numpy(x)
            check_close(q_out, orc.project(xf, to_f32_numpy(wq), wl.Hq, pos=pos, rope_base=rope_base), wl.dtype,
                        "%s layer %d q" % (wl.name, layer))
            if layer not in producers:
                assert torch.equal(gc.storage, before), "a layer without K/V projections wrote to the cache"
                continue
            slot = producers[layer]
            want_k = orc.project(xf, to_f32_numpy(wk), wl.Hkv, pos=pos, rope_base=rope_base)
            want_v = orc.project(xf, to_f32_numpy(wv), wl.Hkv)
            changed = (gc.storage != before).sum().item()
            eb = 2 if wl.dtype == "bf16" else 4
            assert changed <= wl.B * 2 * wl.Hkv * wl.D * eb       # nothing but the new token's K/V bytes
            for b in range(wl.B):
                gk, gv = cache_rows_f32(gc, slot, b, int(lens[b]))
                check_close(torch.from_numpy(gk), want_k[b], wl.dtype, "%s layer %d k[%d]" % (wl.name, layer, b))
                check_close(torch.from_numpy(gv), want_v[b], wl.dtype, "%s layer %d v[%d]" % (wl.name, layer, b))
        assert gc.device_error() == 0


def test_project_bf16_gqa_d64_contiguous_ragged():
    wl = synth.Workload("pr-gqa64", "bf16", L=4, w=2, Hq=4, Hkv=2, D=64, B=5, T=48, sigma=1.0, seed=61)
    run_project(wl, 256, [0, 1, 17, 33, 47], 48)


def test_project_bf16_mha_d128_paged_two_passes():
    wl = synth.Workload("pr-mha128", "bf16", L=3, w=1, Hq=2, Hkv=2, D=128, B=130, T=40, sigma=1.0, seed=62,
                        paged=True, warm=(0,))
    lens = (np.arange(130) * 7) % 40
    run_project(wl, 512, lens, 48)


@pytest.mark.parametrize("B", [16, 17, 33, 48, 64, 65])
def test_project_bf16_batch_blocks(B):
    wl = synth.Workload("pr-b%d" % B, "bf16", L=2, w=1, Hq=3, Hkv=1, D=64, B=B, T=20, sigma=1.0, seed=63 + B,
                        warm=(0,))
    run_project(wl, 256, (np.arange(B) * 3) % 20, 32)


def test_project_without_rotation():
    wl = synth.Workload("pr-norope", "bf16", L=2, w=1, Hq=2, Hkv=2, D=64, B=3, T=20, sigma=1.0, seed=64, warm=(0,))
    run_project(wl, 256, [3, 0, 19], 32, rope_base=0.0)


def test_project_long_positions_keep_their_angle():
    # position 32767 at the highest frequency is 32767 rad: the angle must be formed in double
    wl = synth.Workload("pr-long", "bf16", L=2, w=1, Hq=2, Hkv=2, D=128, B=2, T=32768, sigma=1.0, seed=65, warm=(0,))
    run_project(wl, 256, [32767, 20011], 32768)


def test_project_f32():
    wl = synth.Workload("pr-f32", "f32", L=3, w=1, Hq=4, Hkv=2, D=64, B=4, T=30, sigma=1.0, seed=66, warm=(0,))
    run_project(wl, 96, [0, 5, 16, 29], 32)
    wl = synth.Workload("pr-f32p", "f32", L=2, w=1, Hq=2, Hkv=1, D=128, B=3, T=30, sigma=1.0, seed=67, paged=True)
    run_project(wl, 200, [7, 31, 2], 32)


def test_project_argument_errors():
    wl = synth.Workload("pr-err", "bf16", L=3, w=1, Hq=2, Hkv=2, D=64, B=2, T=32, sigma=1.0, seed=68, warm=(0,))
    with GpuCache(wl, 32, np.array([3, 4], np.int32)) as gc:
        L = lk.lib()
        t = torch.zeros(1 << 16, dtype=torch.bfloat16, device="cuda")
        assert lk.lckv_project_workspace_bytes(gc.h, 2, 256) == 0     # bf16: one launch, no partial sums in memory
        ws = torch.empty(4096, dtype=torch.uint8, device="cuda")
        p, w, n = t.data_ptr(), ws.data_ptr(), ws.numel()
        st = torch.cuda.current_stream().cuda_stream or None
        call = lambda layer, hidden=256, wk=p, wv=p, B=2, wsp=w, wsn=n, ko=None, vo=None: L.lckv_project_qkv(
            gc.h, layer, p, hidden, p, wk, wv, p, ko, vo, gc.lens.data_ptr(), B, 10000.0, wsp, wsn, st)
        producers = [lk.lckv_slot_producer(gc.h, s) for s in range(gc.n_slots)]
        other = [l for l in range(wl.L) if l not in producers][0]
        assert lk.lckv_project_workspace_bytes(gc.h, 2, 1024) == 0
        with pytest.raises(lk.LckvError):
            lk.lckv_project_workspace_bytes(gc.h, 2, 100)
        assert call(other) == lk.LCKV_ERR_NOT_PRODUCER            # such a layer has no W_K, W_V
        assert call(other, wk=None, wv=None) == lk.LCKV_OK
        assert call(other, wk=None, wv=None, ko=p, vo=p) == lk.LCKV_ERR_NOT_PRODUCER
        assert call(producers[0], ko=p) == lk.LCKV_ERR_NULL       # both of k_out, v_out or neither
        assert call(producers[0], wk=None) == lk.LCKV_ERR_NULL and call(producers[0], wv=None) == lk.LCKV_ERR_NULL
        assert call(producers[0], hidden=128) == lk.LCKV_ERR_CONFIG
        assert call(7) == lk.LCKV_ERR_LAYER and call(producers[0], B=3) == lk.LCKV_ERR_BATCH
        assert call(producers[0], wsp=None, wsn=0) == lk.LCKV_OK     # bf16 needs no workspace
        pack = lambda rows, hid, dst=ws.data_ptr(): L.lckv_pack_projection_weight(gc.h, p, dst, rows, hid, st)
        assert pack(96, 256) == lk.LCKV_ERR_CONFIG and pack(64, 128) == lk.LCKV_ERR_CONFIG   # whole heads; hidden % 256
        assert pack(64, 256, dst=p) == lk.LCKV_ERR_CONFIG and pack(64, 256, dst=None) == lk.LCKV_ERR_NULL
        torch.cuda.synchronize()
    with GpuCache(wl, 32, np.array([3, 4], np.int32), sink=4, window=28) as gc:
        shared = [l for l in producers if not lk.lckv_kv_slot(gc.h, l)[1]][0]
        assert L.lckv_project_qkv(gc.h, shared, p, 256, p, p, p, p, None, None, gc.lens.data_ptr(), 2, 10000.0, w, n,
                                  st) == lk.LCKV_ERR_CONFIG     # storing at once would overwrite a visible entry
        assert L.lckv_project_qkv(gc.h, shared, p, 256, p, p, p, p, p, p + 4096, gc.lens.data_ptr(), 2, 10000.0, w, n,
                                  st) == lk.LCKV_OK             # handed back instead: accepted
        torch.cuda.synchronize()


def test_decode_steps_from_hidden_states():
    # Whole steps from the hidden states: per layer, projection (+ fused append) then attention, lengths bumped by
    # the caller; the same composition of oracle functions beside it.  The hidden state of a layer is a seeded
    # input (what lies between the layers - output projection, MLP - is outside the path).
    wl = synth.Workload("pr-steps", "bf16", L=4, w=2, Hq=4, Hkv=2, D=64, B=3, T=40, sigma=1.0, seed=69)
    hidden, T_cap, steps = 256, 48, 4
    lens = np.array([5, 0, 30], np.int32)
    scale = 1.0 / np.sqrt(wl.D)
    with GpuCache(wl, T_cap, lens) as gc:
        ns = gc.n_slots
        K0, V0 = synth.logical_cache(wl, ns, T_cap)
        for s in range(ns):
            gc.load_dense(s, K0[s], V0[s])
        Kf, Vf = to_f32_numpy(K0), to_f32_numpy(V0)                      # oracle's caches [slot][B][T][Hkv][D]
        producers = {lk.lckv_slot_producer(gc.h, s): s for s in range(ns)}
        W = [weights(wl, hidden, l, l in producers) for l in range(wl.L)]
        Wd = [[packed(gc.h, t) for t in w] for w in W]
        ws = torch.empty(lk.lckv_project_workspace_bytes(gc.h, wl.B, hidden), dtype=torch.uint8, device="cuda")
        lens_o = lens.copy()
        for step in range(steps):
            hint = int(lens_o.max())
            aws = gc.workspace(hint)
            for l in range(wl.L):
                x = synth._normal((wl.B, hidden), 1.0, torch.bfloat16, 5000 + 10 * step + l)
                q = torch.empty((wl.B, wl.Hq, wl.D), dtype=torch.bfloat16, device="cuda")
                out = torch.full_like(q, float("nan"))
                lk.lckv_project_qkv(gc.h, l, x.cuda(), hidden, Wd[l][0], Wd[l][1], Wd[l][2], q, gc.lens, wl.B,
                                    10000.0, ws)
                lk.lckv_decode_attention(gc.h, l, q, out, gc.lens, None, wl.B, hint, workspace=aws)
                torch.cuda.synchronize()
                # the oracle: its own projection (rounded to bf16 as the stored K/V and the query are), then
                # the definition of the attention on its own cache
                xf = to_f32_numpy(x)
                rb = lambda a: to_f32_numpy(torch.from_numpy(a).to(torch.bfloat16))
                qo = rb(orc.project(xf, to_f32_numpy(W[l][0]), wl.Hq, pos=lens_o))
                if l in producers:
                    ko = rb(orc.project(xf, to_f32_numpy(W[l][1]), wl.Hkv, pos=lens_o))
                    vo = rb(orc.project(xf, to_f32_numpy(W[l][2]), wl.Hkv))
                    for b in range(wl.B):
                        Kf[producers[l], b, lens_o[b]], Vf[producers[l], b, lens_o[b]] = ko[b], vo[b]
                slot, vis = lk.lckv_kv_slot(gc.h, l)
                n = lens_o + (1 if vis else 0)
                want = np.zeros((wl.B, wl.Hq, wl.D))
                for b in range(wl.B):
                    for h in range(wl.Hq):
                        g = h // (wl.Hq // wl.Hkv)
                        want[b, h] = orc.attend(qo[b, h], Kf[slot, b, :n[b], g], Vf[slot, b, :n[b], g], scale)
                # the two sides round q, k, v to bf16 independently (an ulp apart now and then): looser bar
                g_ = out.float().cpu().numpy()
                assert np.isfinite(g_).all()
                assert np.abs(g_ - want).max() <= 4e-2, "step %d layer %d" % (step, l)
            gc.lens += 1
            lens_o += 1
        assert gc.device_error() == 0


def test_projection_attention_and_prompt_encoding_replay_from_a_hip_graph():
    # The entry points only enqueue, so a caller may capture them: one layer's projection (+ fused append) and
    # attention of a decode step, and a prompt-encoding pass, captured once and replayed with new inputs in the
    # static buffers; every replay is compared with the same calls made eagerly on a twin cache, with eager work
    # and a synchronisation between the replays.  Results are bitwise equal (fixed order of the partial sums).
    wl = synth.Workload("pr-graph", "bf16", L=3, w=1, Hq=4, Hkv=2, D=64, B=5, T=40, sigma=1.0, seed=70, warm=(0,))
    hidden, S = 256, 40
    lens = np.array([7, 0, 33, 16, 36], np.int32)                       # + 3 bumps stays within the S = 40 prompt rows
    with GpuCache(wl, 48, lens) as eager, GpuCache(wl, 48, lens) as graphed:
        K0, V0 = synth.logical_cache(wl, eager.n_slots, 48)
        for gc in (eager, graphed):
            for s in range(gc.n_slots):
                gc.load_dense(s, K0[s], V0[s])
        layer = lk.lckv_slot_producer(eager.h, eager.n_slots - 1)        # the condensed layer that owns the shared slot
        W = weights(wl, hidden, layer, True)
        Wp = {id(gc): [packed(gc.h, w) for w in W] for gc in (eager, graphed)}
        ws = {id(gc): torch.empty(lk.lckv_project_workspace_bytes(gc.h, wl.B, hidden), dtype=torch.uint8, device="cuda")
              for gc in (eager, graphed)}
        aws = {id(gc): gc.workspace(48) for gc in (eager, graphed)}
        sx = torch.zeros((wl.B, hidden), dtype=torch.bfloat16, device="cuda")            # static buffers of the graph
        sq = torch.zeros((wl.B, wl.Hq, wl.D), dtype=torch.bfloat16, device="cuda")
        sout = torch.zeros_like(sq)
        spq = torch.zeros((wl.B, S, wl.Hq, wl.D), dtype=torch.bfloat16, device="cuda")
        spout = torch.zeros_like(spq)

        def calls(gc, x, q, out, pq, pout):
            w = Wp[id(gc)]
            lk.lckv_project_qkv(gc.h, layer, x, hidden, w[0], w[1], w[2], q, gc.lens, wl.B, 10000.0, ws[id(gc)])
            lk.lckv_decode_attention(gc.h, layer, q, out, gc.lens, None, wl.B, 47, workspace=aws[id(gc)])
            lk.lckv_prefill_attention(gc.h, layer, pq, pout, gc.lens, wl.B, S)

        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            calls(graphed, sx, sq, sout, spq, spout)
        for rep in range(4):
            x = synth._normal((wl.B, hidden), 1.0, torch.bfloat16, 7000 + rep).cuda()
            pq = synth._normal((wl.B, S, wl.Hq, wl.D), 1.0, torch.bfloat16, 7100 + rep).cuda()
            sx.copy_(x)
            spq.copy_(pq)
            g.replay()
            q = torch.empty_like(sq)
            out = torch.empty_like(sq)
            pout = torch.empty_like(spq)
            calls(eager, x, q, out, pq, pout)
            torch.cuda.synchronize()
            assert torch.equal(sq, q) and torch.equal(sout, out) and torch.equal(spout, pout), "replay %d" % rep
            assert torch.equal(graphed.storage, eager.storage), "the appended K/V differ in replay %d" % rep
            graphed.lens += 1                                            # eager work between the replays
            eager.lens += 1
        assert graphed.device_error() == 0 and eager.device_error() == 0


@pytest.mark.parametrize("paged", [False, True])
def test_streaming_decode_steps_from_hidden_states(paged):
    # Sections 2.1 and 3.3 together: under the sink + window policy every layer is driven from its hidden state.
    # Warmup layers project and store at once (they see the new token); the condensed layer that owns the shared
    # slot gets its rotated K/V handed back (k_out, v_out) and they are appended after its attention, when no
    # condensed layer of the step reads the ring entry they replace any more.  The ring wraps several times.  The
    # oracle keeps the whole history and projects with its own routine.
    wl = synth.Workload("pr-stream", "bf16", L=4, w=2, Hq=4, Hkv=2, D=64, B=3, T=24, sigma=1.0, seed=71, paged=paged)
    hidden, sink, window, steps = 256, 4, 20, 55
    lens = np.array([24, 0, 9], np.int32)
    T_hist = int(lens.max()) + steps + 1
    scale = 1.0 / np.sqrt(wl.D)
    print("streaming from hidden states: sink", sink, "window", window, "steps", steps, "paged", paged, flush=True)
    with GpuCache(wl, 32 if paged else sink + window, lens, sink=sink, window=window) as gc:
        ns = gc.n_slots
        K0, V0 = synth.logical_cache(wl, ns, T_hist)
        for s in range(ns):
            gc.load_dense(s, K0[s, :, :24], V0[s, :, :24])
        Kf, Vf = to_f32_numpy(K0), to_f32_numpy(V0)                      # the oracle's full history
        producers = {lk.lckv_slot_producer(gc.h, s): s for s in range(ns)}
        W = [weights(wl, hidden, l, l in producers) for l in range(wl.L)]
        Wd = [[packed(gc.h, t) for t in w] for w in W]
        ws = torch.empty(lk.lckv_project_workspace_bytes(gc.h, wl.B, hidden), dtype=torch.uint8, device="cuda")
        kbuf = torch.full((wl.B, wl.Hkv, wl.D), float("nan"), dtype=torch.bfloat16, device="cuda")
        vbuf = torch.full_like(kbuf, float("nan"))
        lens_o = lens.copy()
        rb = lambda a: to_f32_numpy(torch.from_numpy(a).to(torch.bfloat16))
        for step in range(steps):
            hint = int(lens_o.max())
            aws = gc.workspace(hint)
            for l in range(wl.L):
                x = synth._normal((wl.B, hidden), 1.0, torch.bfloat16, 9000 + 10 * step + l)
                q = torch.empty((wl.B, wl.Hq, wl.D), dtype=torch.bfloat16, device="cuda")
                out = torch.full_like(q, float("nan"))
                slot, vis = lk.lckv_kv_slot(gc.h, l)
                deferred = l in producers and not vis
                lk.lckv_project_qkv(gc.h, l, x.cuda(), hidden, Wd[l][0], Wd[l][1], Wd[l][2], q, gc.lens, wl.B,
                                    10000.0, ws, k_out=kbuf if deferred else None, v_out=vbuf if deferred else None)
                lk.lckv_decode_attention(gc.h, l, q, out, gc.lens, None, wl.B, hint, workspace=aws)
                if deferred:
                    lk.lckv_append_kv(gc.h, l, kbuf, vbuf, gc.lens, wl.B)
                torch.cuda.synchronize()
                xf = to_f32_numpy(x)
                qo = rb(orc.project(xf, to_f32_numpy(W[l][0]), wl.Hq, pos=lens_o))
                if l in producers:
                    ko = rb(orc.project(xf, to_f32_numpy(W[l][1]), wl.Hkv, pos=lens_o))
                    vo = rb(orc.project(xf, to_f32_numpy(W[l][2]), wl.Hkv))
                    if deferred:                                     # what was handed back is what the oracle projects
                        assert np.abs(kbuf.float().cpu().numpy() - ko).max() <= 4e-2
                        assert np.abs(vbuf.float().cpu().numpy() - vo).max() <= 4e-2
                    for b in range(wl.B):
                        Kf[producers[l], b, lens_o[b]], Vf[producers[l], b, lens_o[b]] = ko[b], vo[b]
                want = np.zeros((wl.B, wl.Hq, wl.D))
                for b in range(wl.B):
                    n = int(lens_o[b]) + (1 if vis else 0)           # candidates; kept: sinks + the last `window`
                    kept = list(range(min(sink, n))) + list(range(max(sink, n - window), n))
                    for h in range(wl.Hq):
                        g = h // (wl.Hq // wl.Hkv)
                        if kept:
                            want[b, h] = orc.attend(qo[b, h], Kf[slot, b, kept, g], Vf[slot, b, kept, g], scale)
                g_ = out.float().cpu().numpy()
                assert np.isfinite(g_).all()
                assert np.abs(g_ - want).max() <= 4e-2, "step %d layer %d: %g" % (step, l, np.abs(g_ - want).max())
            gc.lens += 1
            lens_o += 1
        assert gc.device_error() == 0
