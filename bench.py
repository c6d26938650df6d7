#!/usr/bin/env python3
"""Benchmark of the LCKV decode-attention step on one MI355X.

A "step" is one lckv_step: for every layer, append of the new token's K/V where the layer produces a slot,
split-KV attention of that layer's queries over the slot it is paired with, merge of the splits; then the length
bump.  Inputs are synthetic and already resident in HBM when the timed region starts.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C3] [--no-cpu-baseline]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E bandwidth

METRIC = {
    "C3": "decode attention tokens/s (all layers, Llama-7B shape, B=128, T=4096) + HBM GB/s %peak",
}


def kernel_source_hash(files=("attn_bf16_mfma.hip", "bf16_mfma_common.h", "lckv_internal.h")):
    """sha256 over the sources the attention kernel is built from.  A counter summary under profiles/ carries the
    hash of the sources it was measured on; bench.py quotes its traffic figure only while the hash still matches."""
    import hashlib
    h = hashlib.sha256()
    for f in files:
        h.update(open(os.path.join(ROOT, "paper_2405_10637_amd", "csrc", f), "rb").read())
    return h.hexdigest()


def measured_traffic(workload):
    """(bytes per launch, note) from profiles/attn_kernel_<workload>_hbm_traffic.txt, or (None, why not)."""
    tpath = os.path.join(ROOT, "profiles", "attn_kernel_%s_hbm_traffic.txt" % workload)
    if not os.path.exists(tpath):
        return None, "no counter summary for this workload under profiles/"
    traffic = stamp = None
    for line in open(tpath):
        if line.startswith("traffic_bytes_per_launch:"):
            traffic = float(line.split(":")[1])
        if line.startswith("kernel_source_sha256:"):
            stamp = line.split(":")[1].strip()
    if stamp != kernel_source_hash():
        return None, "the counter summary under profiles/ was measured on other kernel sources (hash differs)"
    return traffic, "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs summarised in profiles/ (same kernel sources, by hash)"


def key_visits_per_step(lens, self_visible, Hq, step_index=0):
    """(query head, key) pairs one decode step evaluates: every layer l, sequence b and query head attends to
    lens[b] + step_index keys, plus the token itself in a warmup layer (Section 2.1).  The CPU oracle's sample is
    counted in the same unit (keys per (layer, sequence, query head) item), so sample time scales by the ratio."""
    total = 0
    for vis in self_visible:
        for n in lens:
            total += (int(n) + step_index + (1 if vis else 0)) * Hq
    return total


def cpu_baseline(sess, units, kv, q, k_new, v_new, out, target_cpu_s=12.0):
    """Time the CPU oracle (as it stands) on a bounded sample of (layer, b, head) units of this workload, check the
    GPU's output for those units against it, and extrapolate the sample's time to a whole step."""
    import numpy as np
    from oracle import lckv_oracle as orc

    wl = sess.wl
    G = wl.G
    T = int(sess.lens0.max()) + 1
    N = len(units)
    Kb = np.zeros((N, T, wl.D), np.float32)
    Vb = np.zeros((N, T, wl.D), np.float32)
    qb = np.zeros((N, wl.D), np.float32)
    nk = np.zeros(N, np.int64)
    kn_h, vn_h, q_h = k_new.float().cpu().numpy(), v_new.float().cpu().numpy(), q.float().cpu().numpy()
    for i, (l, b, h) in enumerate(units):
        Ku, Vu = kv[(l, b, h)]
        n = Ku.shape[0]
        Kb[i, :n], Vb[i, :n] = Ku, Vu
        slot, vis = sess.kv_slot[l]
        if vis:  # a warmup layer also sees the token being decoded (Section 2.1)
            Kb[i, n], Vb[i, n] = kn_h[slot, b, h // G], vn_h[slot, b, h // G]
            n += 1
        nk[i] = n
        qb[i] = q_h[l, b, h]
    scale = 1.0 / np.sqrt(wl.D)
    t0 = time.perf_counter()
    want, threads = orc.attend_many(qb, Kb, Vb, nk, scale)
    dt = time.perf_counter() - t0
    reps = 1
    spent = dt
    while spent * threads < target_cpu_s and reps < 256:   # repeat until about target_cpu_s core-seconds were spent
        t0 = time.perf_counter()
        orc.attend_many(qb, Kb, Vb, nk, scale)
        one = time.perf_counter() - t0
        spent += one
        dt = min(dt, one)
        reps += 1
    got = np.stack([out[l, b, h].float().cpu().numpy() for (l, b, h) in units]).astype(np.float64)
    err = float(np.abs(got - want).max())
    ref = float(np.abs(want).max())
    total_visits = key_visits_per_step(sess.lens0, [vis for (_, vis) in sess.kv_slot], wl.Hq)
    step_s = dt * (total_visits / float(nk.sum()))
    return {
        "value": wl.B / step_s, "unit": "tokens/s", "cores": threads, "kind": "oracle",
        "sample": "%d of %d (layer, sequence, head) units of the same step, best of %d runs (%.1f core-seconds "
                  "in all), time scaled by (query head, key) visits: %d in the sample, %d in the step (%.3g s for "
                  "the sample)" % (N, wl.L * wl.B * wl.Hq, reps, spent * threads, int(nk.sum()), total_visits, dt),
        "max_abs_err_vs_gpu": err, "max_abs_expected": ref,
    }


def residency_sweep(steps, warmup):
    """Does the shared slot, re-read by each successive condensed layer, stay in the 256 MB last-level cache?
    TinyLlama shape (C2) with the batch varied so that the shared slot goes from 32 MiB to 1 GiB; for plain and
    nontemporal loads, the effective bandwidth (algorithmic bytes / kernel time, HIP events per launch) of the
    condensed layers' launches (slot just read by the previous layer) and of the warmup layers' launches (slot
    last read one step ago).  Prints one JSON line."""
    import numpy as np
    import torch
    from paper_2405_10637_amd import binding as lk
    from paper_2405_10637_amd import synth
    from paper_2405_10637_amd.runner import DecodeSession

    rows = []
    for B in (16, 32, 48, 64, 96, 128, 192, 256, 512):
        wl = synth.C2.with_(B=B, name="C2-shape-B%d" % B)
        with DecodeSession(wl, room=2 * (steps + warmup) + 4) as sess:
            warm = [l for l in range(wl.L) if sess.kv_slot[l][1]]
            units = [(1, 0, 0), (wl.L // 2, B - 1, wl.Hq - 1), (warm[-1], B // 2, 5)]   # condensed, condensed, warmup
            kv = sess.fill(units)
            q, k_new, v_new = synth.step_inputs(wl, sess.n_slots, device="cuda")
            out = torch.empty_like(q)
            per_key = 2 * wl.Hkv * wl.D * wl.elem_bytes
            qo = 2 * wl.B * wl.Hq * wl.D * wl.elem_bytes
            row = {"B": B, "shared_slot_MiB": B * wl.T * per_key / 2 ** 20}
            for name, policy in (("plain", lk.LCKV_LOAD_TEMPORAL), ("nontemporal", lk.LCKV_LOAD_NONTEMPORAL)):
                lk.lckv_set_load_policy(sess.h, policy)
                if name == "plain":     # the first step of each policy is checked against the oracle on sampled units
                    lens_before = sess.lens.clone()
                else:
                    sess.lens.copy_(lens_before)      # the same step again with the other load policy
                    sess.max_len, sess.steps_left = int(sess.lens0.max()), sess.steps_left + steps + warmup + 1
                sess.step(q, k_new, v_new, out)
                torch.cuda.synchronize()
                base = cpu_baseline(sess, units, kv, q, k_new, v_new, out, target_cpu_s=0.0)
                if base["max_abs_err_vs_gpu"] > 2e-2 or base["max_abs_err_vs_gpu"] > 1e-2 * max(base["max_abs_expected"], 1e-3):
                    sys.exit("residency sweep, B=%d, %s loads: GPU output disagrees with the oracle: %r" % (B, name, base))
                row.setdefault("max_abs_err_vs_oracle", {})[name] = base["max_abs_err_vs_gpu"]
                for _ in range(warmup):
                    sess.step(q, k_new, v_new, out)
                torch.cuda.synchronize()
                lk.lckv_profile_read(sess.h)
                lk.lckv_profile_enable(sess.h, True)
                first = sess.max_len - int(sess.lens0.max())
                for _ in range(steps):
                    sess.step(q, k_new, v_new, out)
                ms = lk.lckv_profile_launch_ms(sess.h).reshape(steps, wl.L)
                lk.lckv_profile_read(sess.h)
                lk.lckv_profile_enable(sess.h, False)
                vis = np.array([v for (_, v) in sess.kv_slot])
                n_keys = wl.T + first + np.arange(steps)[:, None] + vis[None, :]
                gbps = (wl.B * n_keys * per_key + qo) / (ms * 1e-3) / 1e9
                row[name] = {"condensed_GBps": float(np.median(gbps[:, vis == 0][:, 1:])),   # skip the first: cold
                             "first_condensed_GBps": float(np.median(gbps[:, vis == 0][:, 0])),
                             "warmup_layer_GBps": float(np.median(gbps[:, vis == 1])),
                             "condensed_launch_us": float(np.median(ms[:, vis == 0][:, 1:]) * 1e3)}
            rows.append(row)
    print(json.dumps({"metric": "shared-slot residency sweep, TinyLlama shape (L=22, 32/4 heads, D=64, T=2048)",
                      "unit": "GB/s effective per attention launch", "hbm_peak_GBps": HBM_PEAK_GBPS,
                      "last_level_cache_MiB": 256, "rows": rows}))


def prefill_bench(steps, warmup, tile, with_import=False, S=2048, B=16):
    """Prompt-encoding attention (lckv_prefill_attention, one condensed layer over the whole prompt), Llama-7B
    shape, bf16: B=16 prompts of S=2048 tokens.  Compute-bound: reported against the bf16 matrix-core peak.
    Checks a sample of rows against the oracle.  With `with_import` a step is what one iteration of the prompt
    encoding does for this layer (Section 2.3): the import of the producing layer's K/V of all prompt tokens
    (lckv_cache_load_dense) followed by the attention that reads them.  Prints one JSON line."""
    import numpy as np
    import torch
    from oracle import lckv_oracle as orc
    from paper_2405_10637_amd import binding as lk
    from paper_2405_10637_amd import synth
    from paper_2405_10637_amd.runner import DecodeSession

    wl = synth.C3.with_(B=B, T=S, name="prefill-llama-7b-B%d-S%d" % (B, S))
    with DecodeSession(wl, room=16) as sess:
        if tile:
            lk.lckv_set_prefill_tile(sess.h, tile)
        layer = 1                                    # a condensed layer: reads the shared slot, diagonal masked
        slot, vis = sess.kv_slot[layer]
        units = [(layer, b, h) for b in (0, wl.B - 1) for h in (0, 13, wl.Hq - 1)]
        kv = sess.fill(units)
        q = synth._normal((wl.B, S, wl.Hq, wl.D), wl.sigma, wl.torch_dtype, wl.seed + 9, device="cuda")
        out = torch.empty_like(q)
        attend = lambda: lk.lckv_prefill_attention(sess.h, layer, q, out, sess.lens, wl.B, S)
        # the dense K/V the iteration's producing layer hands over (same seeds as fill(): the cache content stays)
        Kd = torch.empty((wl.B, S, wl.Hkv, wl.D), dtype=wl.torch_dtype, device="cuda")
        Vd = torch.empty_like(Kd)
        synth.fill_normal_(Kd, wl.sigma, wl.seed * 31 + 2 * slot)
        synth.fill_normal_(Vd, wl.sigma, wl.seed * 31 + 2 * slot + 1)
        load = lambda: lk.lckv_cache_load_dense(sess.h, slot, Kd, Vd, sess.lens, wl.B, S)

        def timed(fn, n):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            for _ in range(n):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / n

        load()
        import_ms = timed(load, max(steps, 3))
        import_gbps = 2 * 2 * Kd.numel() * 2 / (import_ms * 1e-3) / 1e9      # K and V, read and written
        run = (lambda: (load(), attend())) if with_import else attend
        run()
        torch.cuda.synchronize()
        err = ref = 0.0
        rows = [i for i in (0, 1, 15, 16, 17, 255, 256, 1023, S - 1) if i < S]
        for (_, b, h) in units:                       # oracle on sampled rows of sampled (sequence, head) pairs
            Ku, Vu = kv[(layer, b, h)]
            for i in rows:
                want = orc.attend(q[b, i, h].float().cpu().numpy(), Ku[:i], Vu[:i], 1.0 / np.sqrt(wl.D))
                got = out[b, i, h].float().cpu().numpy().astype(np.float64)
                err, ref = max(err, float(np.abs(got - want).max())), max(ref, float(np.abs(want).max()))
        if err > 2e-2 or err > 1e-2 * max(ref, 1e-3):
            sys.exit("prefill output disagrees with the oracle: err %g, max expected %g" % (err, ref))
        for _ in range(warmup):
            run()
        ms = timed(run, steps)
        attn_ms = timed(attend, steps) if with_import else ms
        pairs = wl.B * wl.Hq * (S * (S - 1) // 2)                  # (query, key) pairs below the diagonal
        flops = 4.0 * wl.D * pairs                                 # QK^T and PV, 2 flops per multiply-add
        tflops = flops / (attn_ms * 1e-3) / 1e12
        print(json.dumps({
            "metric": "prompt-encoding attention%s, one condensed layer (Llama-7B shape, B=%d, S=%d)"
                      % (" with the K/V import before it" if with_import else "", B, S),
            "value": wl.B * S / (ms * 1e-3), "unit": "prompt tokens/s per layer", "n_gpus": 1, "steps": steps,
            "warmup": warmup, "ms_per_step": ms, "higher_is_better": True, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": wl.name},
            "roofline": {"bound": "mfma", "kernel": "prefill_bf16_kernel", "achieved": tflops, "peak": 2500.0,
                         "unit": "TFLOP/s", "frac": tflops / 2500.0, "traffic": None, "avg_launch_ms": attn_ms},
            "import": {"kernel": "load_dense_bf16_kernel", "ms": import_ms, "read_plus_write_GBps": import_gbps,
                       "frac_of_hbm_peak": import_gbps / HBM_PEAK_GBPS, "in_timed_step": bool(with_import)},
            "max_abs_err_vs_oracle": err, "max_abs_expected": ref}))


def project_bench(steps, warmup, batch, graph=False):
    """The projections of one decode step (lckv_project_qkv for every layer: queries everywhere, keys and values
    - rotated and stored into the cache - for the producing layers only), Llama-7B shape, bf16, hidden 4096.
    Weight-streaming bound: reported against the HBM peak.  Checks sampled outputs against the oracle.
    Prints one JSON line."""
    import numpy as np
    import torch
    from oracle import lckv_oracle as orc
    from paper_2405_10637_amd import binding as lk
    from paper_2405_10637_amd import synth
    from paper_2405_10637_amd.runner import DecodeSession

    hidden, T = 4096, 64
    wl = synth.C3.with_(B=batch, T=T, name="project-llama-7b-B%d" % batch)
    with DecodeSession(wl, room=steps + warmup + 4) as sess:
        producers = {lk.lckv_slot_producer(sess.h, s): s for s in range(sess.n_slots)}
        g = torch.Generator(device="cuda")
        g.manual_seed(wl.seed + 77)
        rnd = lambda rows: (torch.randn((rows, hidden), generator=g, device="cuda") / hidden ** 0.5).to(torch.bfloat16)
        W = [(rnd(wl.Hq * wl.D),) + ((rnd(wl.Hkv * wl.D), rnd(wl.Hkv * wl.D)) if l in producers else (None, None))
             for l in range(wl.L)]                                           # row-major, as the oracle takes them

        def pack(w):                                                        # once, as at model load
            if w is None:
                return None
            wp = torch.empty_like(w)
            lk.lckv_pack_projection_weight(sess.h, w, wp, w.shape[0], hidden)
            return wp

        Wp = [tuple(pack(w) for w in ws_) for ws_ in W]
        x = torch.randn((wl.L, wl.B, hidden), generator=g, device="cuda").to(torch.bfloat16)
        q = torch.empty((wl.L, wl.B, wl.Hq, wl.D), dtype=torch.bfloat16, device="cuda")
        ws = torch.empty(lk.lckv_project_workspace_bytes(sess.h, wl.B, hidden), dtype=torch.uint8, device="cuda")

        def one_step():
            for l in range(wl.L):
                lk.lckv_project_qkv(sess.h, l, x[l], hidden, Wp[l][0], Wp[l][1], Wp[l][2], q[l], sess.lens, wl.B,
                                    10000.0, ws)

        one_step()
        torch.cuda.synchronize()
        err = ref = 0.0
        lens = sess.lens.cpu().numpy()
        f32 = lambda t: t.float().cpu().numpy()
        for l in sorted(set([0, 1, wl.L // 2] + list(producers))):
            for b in (0, wl.B - 1):
                for h in (0, wl.Hq - 1):
                    want = orc.project(f32(x[l, b:b + 1]), f32(W[l][0][h * wl.D:(h + 1) * wl.D]), 1, pos=lens[b:b + 1])
                    got = f32(q[l, b, h]).astype(np.float64)
                    err, ref = max(err, float(np.abs(got - want[0, 0]).max())), max(ref, float(np.abs(want).max()))
        if err > 2e-2 or err > 1e-2 * max(ref, 1e-3):
            sys.exit("projection disagrees with the oracle: err %g, max expected %g" % (err, ref))
        run = one_step
        if graph:                                    # the 64 launches of a step captured once, replayed per step
            torch.cuda.synchronize()
            g_ = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g_):
                one_step()
            run = g_.replay
        for _ in range(warmup):
            run()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(steps):
            run()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / steps
        rows = wl.L * wl.Hq * wl.D + 2 * len(producers) * wl.Hkv * wl.D       # weight rows a step streams
        full = wl.L * (wl.Hq + 2 * wl.Hkv) * wl.D                           # ... with K/V projections everywhere
        nbytes = 2.0 * rows * hidden + wl.L * wl.B * (hidden + wl.Hq * wl.D) * 2.0
        gbps = nbytes / (ms * 1e-3) / 1e9
        print(json.dumps({
            "metric": "q/k/v projections + rotary embedding + append of one decode step (Llama-7B shape, B=%d)" % batch,
            "value": wl.B / (ms * 1e-3), "unit": "tokens/s (projections only)", "n_gpus": 1, "steps": steps,
            "warmup": warmup, "ms_per_step": ms, "higher_is_better": True, "dtype": "bf16", "data": "synthetic",
            "launch": "graph replay" if graph else "eager",
            "config": {"workload": wl.name, "hidden": hidden, "producing_layers": sorted(producers)},
            "roofline": {"bound": "hbm", "kernel": "project_bf16_kernel (+ finish)", "achieved": gbps,
                         "peak": 8000.0, "unit": "GB/s", "frac": gbps / 8000.0, "traffic": None},
            "weight_rows_streamed": rows, "weight_rows_with_kv_everywhere": full,
            "max_abs_err_vs_oracle": err, "max_abs_expected": ref}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="C3")
    ap.add_argument("--split-tokens", type=int, default=0)
    ap.add_argument("--waves", type=int, default=0, help="waves per decode-attention workgroup (0 auto, 4, 8, 16)")
    ap.add_argument("--load-policy", type=int, default=0, help="0 auto, 1 plain loads, 2 nontemporal loads")
    ap.add_argument("--sample", type=int, default=768, help="units the CPU oracle is timed and checked on")
    ap.add_argument("--capacity", type=int, default=0,
                    help="positions per sequence the cache is built for (default: just enough for this run); the "
                         "distance between two sequences' streams in HBM follows from it")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--graph", action="store_true",
                    help="capture one lckv_step in a HIP graph (length bound = last timed step) and time replays")
    ap.add_argument("--one-launch", action="store_true",
                    help="the step through lckv_step_one_launch: one resident kernel, a device-wide barrier between "
                         "layers (for small slots, where a layer's pass lasts about as long as a launch)")
    ap.add_argument("--chain", action="store_true",
                    help="feed layer l's output into layer l+1's query (q[l+1] = q_seed[l+1] + out[l]) so the "
                         "layer-to-layer dependency of the model is physically real; per-layer entry points")
    ap.add_argument("--prefill", action="store_true",
                    help="instead of the decode benchmark: prompt-encoding attention of one layer (MFMA-bound)")
    ap.add_argument("--prefill-tile", type=int, default=0, help="query blocks per wave in the prefill kernel (2|4)")
    ap.add_argument("--with-import", action="store_true",
                    help="--prefill: a step is the K/V import (lckv_cache_load_dense) plus the attention that reads it")
    ap.add_argument("--prompt-len", type=int, default=2048, help="--prefill: tokens per prompt")
    ap.add_argument("--prompts", type=int, default=16, help="--prefill: prompts in the batch")
    ap.add_argument("--project", action="store_true",
                    help="instead of the decode benchmark: the q/k/v projections of one decode step (HBM-bound)")
    ap.add_argument("--batch", type=int, default=128, help="sequences in --project")
    ap.add_argument("--residency-sweep", action="store_true",
                    help="instead of the benchmark: effective bandwidth vs size of the shared slot (C2 shape)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)")
    if args.residency_sweep:
        return residency_sweep(args.steps, args.warmup)
    if args.prefill:
        return prefill_bench(args.steps, args.warmup, args.prefill_tile, args.with_import, args.prompt_len,
                             args.prompts)
    if args.project:
        return project_bench(args.steps, args.warmup, args.batch, args.graph)

    import numpy as np
    import torch
    from paper_2405_10637_amd import binding as lk
    from paper_2405_10637_amd import synth
    from paper_2405_10637_amd.runner import DecodeSession

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    lk.lib()  # fail loudly if the HIP library is not built
    wl = synth.WORKLOADS[args.workload]
    K, W = args.steps, args.warmup

    # capacity: the initial length plus every step this run takes (graph mode runs K replays and K eager steps)
    room = 2 * K + W + 2   # timed steps + a second pass (graph: with launch events; otherwise: without them)
    if args.capacity:
        if args.capacity < wl.T + room:
            sys.exit("--capacity must be at least %d for this run" % (wl.T + room))
        room = args.capacity - wl.T
    sess = DecodeSession(wl, room=room, split_tokens=args.split_tokens, waves=args.waves)
    lk.lckv_set_load_policy(sess.h, args.load_policy)
    units = []
    if not args.no_cpu_baseline:
        warm_layers = [l for l in range(wl.L) if sess.kv_slot[l][1]]
        units = synth.sample_units(wl, sess.lens0, args.sample, must_layers=warm_layers[:1] + warm_layers[-1:])
    kv = sess.fill(units)
    q, k_new, v_new = synth.step_inputs(wl, sess.n_slots, device="cuda")
    out = torch.empty_like(q)
    if args.chain:
        if args.graph:
            sys.exit("--chain and --graph are separate modes")
        q_seed, q = q, torch.empty_like(q)
        one_step = lambda: sess.step_chained(q_seed, k_new, v_new, q, out)
    elif args.one_launch:
        if args.graph:
            sys.exit("--one-launch and --graph are separate modes (a cooperative launch is not captured)")
        one_step = lambda: sess.step_one_launch(q, k_new, v_new, out)
    else:
        one_step = lambda: sess.step(q, k_new, v_new, out)

    base = None
    # first (untimed) step doubles as the check against the oracle
    one_step()
    torch.cuda.synchronize()
    if units:
        base = cpu_baseline(sess, units, kv, q, k_new, v_new, out)
        tol_ok = base["max_abs_err_vs_gpu"] <= 2e-2 and \
            base["max_abs_err_vs_gpu"] <= 1e-2 * max(base["max_abs_expected"], 1e-3)
        if wl.dtype == "f32":
            tol_ok = base["max_abs_err_vs_gpu"] <= 1e-5
        if not tol_ok:
            sys.exit("GPU output disagrees with the oracle: %r" % base)
    del kv
    for _ in range(max(W - 1, 0)):
        one_step()
    torch.cuda.synchronize()

    first_timed = 1 + max(W - 1, 0)
    if args.graph:
        # One captured step replayed K times; the per-launch events are taken in a second, eager pass of K steps.
        hint = sess.max_len + 2 * K
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            lk.lckv_step(sess.h, q, k_new, v_new, out, sess.lens, wl.B, hint, sess.workspace)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(K):
            graph.replay()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        sess.max_len += K
        sess.steps_left -= K
    lk.lckv_profile_read(sess.h)
    lk.lckv_profile_enable(sess.h, True)
    torch.cuda.synchronize()
    te0 = time.perf_counter()
    for _ in range(0 if args.graph and sess.steps_left < K else K):
        one_step()
    torch.cuda.synchronize()
    te1 = time.perf_counter()
    if not args.graph:
        t0, t1 = te0, te1
    n_launch, kern_ms = lk.lckv_profile_read(sess.h)
    lk.lckv_profile_enable(sess.h, False)
    assert lk.lckv_last_device_error(sess.h) == 0
    # The timed steps carry two HIP events per launch (the kernel's duration for the roofline comes from them).  An
    # event costs a few microseconds on the stream: nothing next to a 1 ms launch, a quarter of a step where a
    # launch lasts 20 us.  A second pass of K steps without them says what the step costs a caller who records none.
    ms_plain = None
    if not args.graph and sess.steps_left >= K:
        torch.cuda.synchronize()
        tp0 = time.perf_counter()
        for _ in range(K):
            one_step()
        torch.cuda.synchronize()
        ms_plain = (time.perf_counter() - tp0) * 1e3 / K

    # what a pure read with the same load pattern reaches on this device (context for the roofline fraction)
    probe_bytes = min(sess.cache_bytes, 16 << 30) // (2 << 20) * (2 << 20)
    lk.lckv_hbm_read_probe(sess.h, sess.storage, probe_bytes, True)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(3):
        lk.lckv_hbm_read_probe(sess.h, sess.storage, probe_bytes, True)
    e1.record()
    torch.cuda.synchronize()
    probe_gbps = 3 * probe_bytes / (e0.elapsed_time(e1) * 1e-3) / 1e9

    ms_per_step = (t1 - t0) * 1e3 / K
    kv_bytes = sum(sess.kv_bytes_per_step(first_timed + i) for i in range(K))
    qo_bytes = K * 2 * wl.L * wl.B * wl.Hq * wl.D * wl.elem_bytes
    ev_first = first_timed + (K if args.graph else 0)   # the steps whose launches carried the events
    ev_bytes = sum(sess.kv_bytes_per_step(ev_first + i) for i in range(K)) + qo_bytes
    alg_bytes_per_launch = ev_bytes / float(K * wl.L)
    if args.one_launch:   # one kernel per step: its duration is the step's (no per-layer events inside a launch)
        n_launch, kern_ms, alg_bytes_per_launch = K, ms_per_step * K, ev_bytes / float(K)
    avg_kernel_ms = kern_ms / max(n_launch, 1)
    achieved = alg_bytes_per_launch / (avg_kernel_ms * 1e-3) / 1e9
    step_gbps = (kv_bytes + qo_bytes) / K / (ms_per_step * 1e-3) / 1e9

    traffic, traffic_note = measured_traffic(args.workload)

    rec = {
        "metric": METRIC.get(args.workload, "decode attention tokens/s (all layers, %s)" % wl.name),
        "value": wl.B / (ms_per_step * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic", "launch": "hip-graph replay" if args.graph else ("eager, chained layers" if args.chain else
                                                         "one launch, device-wide barriers" if args.one_launch else "eager"),
        "config": {"workload": "%s: L=%d w=%d Hq=%d Hkv=%d D=%d B=%d T=%s%s" % (
            wl.name, wl.L, wl.w, wl.Hq, wl.Hkv, wl.D, wl.B,
            wl.T if wl.T_min is None else "U[%d,%d]" % (wl.T_min, wl.T), " paged16" if wl.paged else ""),
            "slots": sess.n_slots, "cache_GiB": round(sess.cache_bytes / 2 ** 30, 2)},
        "step_effective_GBps": step_gbps, "step_pct_of_hbm_peak": 100.0 * step_gbps / HBM_PEAK_GBPS,
        "ms_per_step_without_launch_events": ms_plain,
        "read_probe_GBps": probe_gbps,
        "cache_fill_import_GBps": [round(x, 1) for x in sess.import_GBps],   # lckv_cache_load_dense, read + write
        "roofline": {"bound": "hbm", "kernel": "step_bf16_kernel" if args.one_launch else
                     "attn_%s_kernel" % ("bf16" if wl.dtype == "bf16" else "f32"),
                     "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": traffic, "traffic_source": traffic_note, "launches": n_launch, "avg_launch_ms": avg_kernel_ms,
                     "alg_bytes_per_launch": alg_bytes_per_launch},
        "cpu_baseline": base,
    }
    sess.close()
    print(json.dumps(rec))


if __name__ == "__main__":
    main()
