"""GPU parity of the widened path at the sizes bench.py times it at, on sampled outputs the oracle computes one by
one: the prompt-encoding attention (Llama-7B shape, 16 prompts of 2048 tokens, a condensed and a warmup layer,
ragged prompt lengths; 2 prompts of 16384 tokens, contiguous and paged; TinyLlama shape with D = 64 at 2048 tokens) and the projections of a decode step (Llama-7B shape, hidden 4096, B = 128: a layer without
K/V projections and the three producing layers, with the keys and values read back from the cache)."""
import numpy as np
import pytest
import torch

from oracle import lckv_oracle as orc
from paper_2405_10637_amd import binding as lk
from paper_2405_10637_amd import synth
from paper_2405_10637_amd.runner import DecodeSession

from gpu_harness import check_close, to_f32_numpy

pytestmark = pytest.mark.gpu


def test_prefill_attention_at_bench_size_sampled_rows():
    S = 2048
    wl = synth.C3.with_(B=16, T=S, name="prefill-llama-7b-B16-S2048")
    print("full-size case", wl.name, flush=True)
    with DecodeSession(wl, room=16) as sess:
        lens = np.full(wl.B, S, np.int32)
        lens[3], lens[7], lens[wl.B - 1] = 1500, 17, 2047               # ragged: the kernel masks per sequence
        dev_lens = torch.from_numpy(lens).cuda()
        warm = [l for l in range(wl.L) if sess.kv_slot[l][1]][0]
        cond = [l for l in range(wl.L) if not sess.kv_slot[l][1]][0]
        units = [(layer, b, h) for layer in (cond, warm) for b in (0, 3, 7, wl.B - 1) for h in (0, 13, wl.Hq - 1)]
        kv = sess.fill(units)                                           # rows [S][D] of the slot each unit reads
        q = synth._normal((wl.B, S, wl.Hq, wl.D), wl.sigma, wl.torch_dtype, wl.seed + 9, device="cuda")
        scale = 1.0 / np.sqrt(wl.D)
        for layer in (cond, warm):
            vis = sess.kv_slot[layer][1]
            out = torch.full_like(q, float("nan"))
            lk.lckv_prefill_attention(sess.h, layer, q, out, dev_lens, wl.B, S)
            torch.cuda.synchronize()
            got, want = [], []
            for (l, b, h) in units:
                if l != layer:
                    continue
                Ku, Vu = kv[(l, b, h)]
                n_b = int(lens[b])
                rows = sorted({0, 1, 15, 16, 17, 31, 32, 255, 1023, n_b - 1, min(n_b, S - 1), S - 1})
                for i in rows:
                    if i >= n_b:                                        # rows past the prompt are exact zeros
                        assert (out[b, i, h] == 0).all(), (layer, b, h, i)
                        continue
                    n = i + (1 if vis else 0)
                    want.append(orc.attend(to_f32_numpy(q[b, i, h]), Ku[:n], Vu[:n], scale))
                    got.append(out[b, i, h])
            err = check_close(torch.stack(got), np.stack(want), wl.dtype, "%s layer %d" % (wl.name, layer))
            print("  layer %d (self visible %d): %d rows, max-abs error %.3g" % (layer, vis, len(got), err), flush=True)
        assert lk.lckv_last_device_error(sess.h) == 0


@pytest.mark.parametrize("name,base,B,S,paged,tile", [
    ("long prompts, Llama-7B shape", "C3", 2, 16384, False, 0),
    ("long prompts, Llama-7B shape, paged", "C3", 2, 16384, True, 0),
    ("TinyLlama shape (D=64, 8 query heads per kv head)", "C2", 8, 2048, False, 0),
    ("TinyLlama shape, two query tiles per wave", "C2", 8, 2048, False, 4),
])
def test_prefill_attention_long_and_d64_sampled_rows(name, base, B, S, paged, tile):
    # the sizes the long-prompt and the D = 64 throughput figures are quoted at: rows sampled across the prompt,
    # at tile and workgroup edges, each compared with the oracle's definition on exactly the K/V rows it sees
    wl = getattr(synth, base).with_(B=B, T=S, paged=paged, name="prefill-%s-B%d-S%d" % (base, B, S))
    print("full-size case", name, wl.name, "tile", tile, flush=True)
    with DecodeSession(wl, room=16) as sess:
        if tile:
            lk.lckv_set_prefill_tile(sess.h, tile)
        lens = np.full(wl.B, S, np.int32)
        lens[1] = S - 4097 if S > 8192 else 1000                        # one shorter prompt
        dev_lens = torch.from_numpy(lens).cuda()
        warm = [l for l in range(wl.L) if sess.kv_slot[l][1]][0]
        cond = [l for l in range(wl.L) if not sess.kv_slot[l][1]][0]
        units = [(layer, b, h) for layer in (cond, warm) for b in (0, 1) for h in (0, 5, wl.Hq - 1)]
        kv = sess.fill(units)
        q = synth._normal((wl.B, S, wl.Hq, wl.D), wl.sigma, wl.torch_dtype, wl.seed + 9, device="cuda")
        scale = 1.0 / np.sqrt(wl.D)
        for layer in (cond, warm):
            vis = sess.kv_slot[layer][1]
            out = torch.full_like(q, float("nan"))
            lk.lckv_prefill_attention(sess.h, layer, q, out, dev_lens, wl.B, S)
            torch.cuda.synchronize()
            got, want = [], []
            for (l, b, h) in units:
                if l != layer:
                    continue
                Ku, Vu = kv[(l, b, h)]
                n_b = int(lens[b])
                rows = sorted({0, 1, 31, 32, 33, 127, 128, 129, 255, 256, 1023, S // 2 - 1, S // 2, n_b - 33, n_b - 32,
                               n_b - 1, min(n_b, S - 1), S - 1})
                for i in rows:
                    if i >= n_b:
                        assert (out[b, i, h] == 0).all(), (layer, b, h, i)
                        continue
                    n = i + (1 if vis else 0)
                    want.append(orc.attend(to_f32_numpy(q[b, i, h]), Ku[:n], Vu[:n], scale))
                    got.append(out[b, i, h])
            err = check_close(torch.stack(got), np.stack(want), wl.dtype, "%s layer %d" % (wl.name, layer))
            print("  layer %d (self visible %d): %d rows, max-abs error %.3g" % (layer, vis, len(got), err), flush=True)
        assert lk.lckv_last_device_error(sess.h) == 0


def test_projections_at_bench_size_sampled_outputs():
    hidden = 4096
    wl = synth.C3.with_(B=128, T=64, name="project-llama-7b-B128")
    print("full-size case", wl.name, flush=True)
    with DecodeSession(wl, room=8) as sess:
        producers = {lk.lckv_slot_producer(sess.h, s): s for s in range(sess.n_slots)}
        other = [l for l in range(wl.L) if l not in producers][0]
        sess.lens.copy_(torch.from_numpy(((np.arange(wl.B) * 5) % 64).astype(np.int32)))   # ragged positions
        lens = sess.lens.cpu().numpy()
        ws = torch.empty(lk.lckv_project_workspace_bytes(sess.h, wl.B, hidden), dtype=torch.uint8, device="cuda")
        rnd = lambda shape, sigma, seed: synth._normal(shape, sigma, torch.bfloat16, seed, device="cuda")
        for layer in [other] + sorted(producers):
            x = rnd((wl.B, hidden), 1.0, wl.seed + 300 + layer)
            W = [rnd((wl.Hq * wl.D, hidden), hidden ** -0.5, wl.seed + 400 + 3 * layer)]
            if layer in producers:
                W += [rnd((wl.Hkv * wl.D, hidden), hidden ** -0.5, wl.seed + 401 + 3 * layer + k) for k in (0, 1)]
            Wp = []
            for w in W:
                wp = torch.empty_like(w)
                lk.lckv_pack_projection_weight(sess.h, w, wp, w.shape[0], hidden)
                Wp.append(wp)
            Wp += [None] * (3 - len(Wp))
            q = torch.full((wl.B, wl.Hq, wl.D), float("nan"), dtype=torch.bfloat16, device="cuda")
            lk.lckv_project_qkv(sess.h, layer, x, hidden, Wp[0], Wp[1], Wp[2], q, sess.lens, wl.B, 10000.0, ws)
            torch.cuda.synchronize()
            got, want = [], []
            for b in (0, 1, 63, 64, wl.B - 1):
                xb = to_f32_numpy(x[b:b + 1])
                for h in (0, 17, wl.Hq - 1):
                    head = lambda w: to_f32_numpy(w[h * wl.D:(h + 1) * wl.D])
                    want.append(orc.project(xb, head(W[0]), 1, pos=lens[b:b + 1])[0, 0])
                    got.append(q[b, h].float().cpu())
                    if layer in producers:                              # the new token's K/V, read back from the cache
                        k = np.zeros((1, wl.Hkv, wl.D), np.uint16)
                        v = np.zeros_like(k)
                        lk.lckv_cache_read(sess.h, producers[layer], b, int(lens[b]), 1, k, v)
                        f32 = lambda a: torch.from_numpy((a.astype(np.uint32) << 16).view(np.float32)[0, h])
                        want.append(orc.project(xb, head(W[1]), 1, pos=lens[b:b + 1])[0, 0])
                        got.append(f32(k))
                        want.append(orc.project(xb, head(W[2]), 1)[0, 0])
                        got.append(f32(v))
            err = check_close(torch.stack(got), np.stack(want), wl.dtype, "%s layer %d" % (wl.name, layer))
            print("  layer %d: %d vectors, max-abs error %.3g" % (layer, len(got), err), flush=True)
        assert lk.lckv_last_device_error(sess.h) == 0
