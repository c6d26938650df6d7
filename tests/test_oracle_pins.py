"""Pins for the CPU oracle: what the paper and the mathematics fix, checked without any GPU.

Each test names the statement of the paper (section) or the closed form it rests on.  None of them
re-types the oracle's own loop; they use closed forms, a library attention routine as a black box,
invariants, and hand-derived pairing tables.
"""
import itertools
import math

import numpy as np
import pytest
import scipy.special
import torch

from oracle import lckv_oracle as orc

RULES = [orc.PAIR_TOP_OF_CONDENSED, orc.PAIR_LAST_LAYER]


def rnd(shape, seed, sigma=1.0):
    return (np.random.default_rng(seed).standard_normal(shape) * sigma).astype(np.float32)


def make_state(L, B, Hq, Hkv, D, T_cap, warm, rule, seed, lens=None):
    _, _, prod = orc.pairing(warm, rule)
    ns = len(prod)
    K = rnd((ns, B, T_cap, Hkv, D), seed + 1)
    V = rnd((ns, B, T_cap, Hkv, D), seed + 2)
    if lens is None:
        lens = np.random.default_rng(seed + 3).integers(0, T_cap - 1, size=B)
    lens = np.asarray(lens, np.int32).copy()
    q = rnd((L, B, Hq, D), seed + 4)
    kn = rnd((ns, B, Hkv, D), seed + 5)
    vn = rnd((ns, B, Hkv, D), seed + 6)
    return K, V, lens, q, kn, vn


# ---------------------------------------------------------------- pairing (Section 2.1)

def test_pairing_no_warmup_single_shared_slot():
    # Figure 1(b): queries of all layers pair with the top layer's KVs; one cached layer.
    for rule in RULES:
        slot, vis, prod = orc.pairing([0, 0, 0, 0, 0], rule)
        assert slot.tolist() == [0] * 5 and vis.tolist() == [0] * 5 and prod.tolist() == [4]


def test_pairing_all_warmup_is_standard_transformer():
    # Section 4.2 (warmup-layer figure caption): w = L is exactly the standard transformer.
    for rule in RULES:
        slot, vis, prod = orc.pairing([1] * 6, rule)
        assert slot.tolist() == list(range(6)) and vis.tolist() == [1] * 6 and prod.tolist() == list(range(6))


def test_pairing_tiny_config_layer0_warm():
    # L=4, layer 0 warmup, layers 1-3 read the top layer's cache (same under both rules).
    for rule in RULES:
        slot, vis, prod = orc.pairing([1, 0, 0, 0], rule)
        assert slot.tolist() == [0, 1, 1, 1] and vis.tolist() == [1, 0, 0, 0] and prod.tolist() == [0, 3]


def test_pairing_sandwich_rule1_and_rule2():
    # Sandwich w=2 on 4 layers: warm = {0, 3}.
    slot, vis, prod = orc.pairing([1, 0, 0, 1], orc.PAIR_TOP_OF_CONDENSED)
    assert prod.tolist() == [0, 2, 3]          # warm 0, topmost condensed layer 2, warm 3
    assert slot.tolist() == [0, 1, 1, 2] and vis.tolist() == [1, 0, 0, 1]
    slot, vis, prod = orc.pairing([1, 0, 0, 1], orc.PAIR_LAST_LAYER)
    assert prod.tolist() == [0, 3]             # the shared cache is layer L-1's
    assert slot.tolist() == [0, 1, 1, 1] and vis.tolist() == [1, 0, 0, 1]


def test_pairing_slot_count_depends_on_w_not_placement_rule1():
    # Section 4.1: inference efficiency is set by w, not by where the warmup layers sit.
    L = 6
    for w in range(1, L):
        counts = set()
        for warm_idx in itertools.combinations(range(L), w):
            warm = np.zeros(L, np.uint8)
            warm[list(warm_idx)] = 1
            _, _, prod = orc.pairing(warm, orc.PAIR_TOP_OF_CONDENSED)
            counts.add(len(prod))
        assert counts == {w + 1}


def test_pairing_every_mask_consistent():
    L = 5
    for bits in range(2 ** L):
        warm = np.array([(bits >> l) & 1 for l in range(L)], np.uint8)
        for rule in RULES:
            slot, vis, prod = orc.pairing(warm, rule)
            assert sorted(prod.tolist()) == prod.tolist()            # slots by ascending producer
            for l in range(L):
                assert vis[l] == warm[l]
                if warm[l]:
                    assert prod[slot[l]] == l                       # own cache
            cond = [l for l in range(L) if not warm[l]]
            if cond:
                shared = {int(slot[l]) for l in cond}
                assert len(shared) == 1                              # one shared cache
                want = max(cond) if rule == orc.PAIR_TOP_OF_CONDENSED else L - 1
                assert prod[shared.pop()] == want


# ---------------------------------------------------------------- single-query attention

def test_attend_one_key_returns_its_value():
    q, K, V = rnd(8, 1), rnd((1, 8), 2), rnd((1, 8), 3)
    np.testing.assert_array_equal(orc.attend(q, K, V, 0.37), V[0].astype(np.float64))


def test_attend_two_keys_is_a_sigmoid_mix():
    D = 16
    q, K, V = rnd(D, 4), rnd((2, D), 5), rnd((2, D), 6)
    scale = 1.0 / math.sqrt(D)
    s = [scale * float(np.dot(q.astype(np.float64), K[j].astype(np.float64))) for j in range(2)]
    sig = 1.0 / (1.0 + math.exp(-(s[0] - s[1])))
    want = sig * V[0].astype(np.float64) + (1.0 - sig) * V[1].astype(np.float64)
    np.testing.assert_allclose(orc.attend(q, K, V, scale), want, rtol=0, atol=1e-14)
    # the scale matters: a different one must give a different answer
    assert np.abs(orc.attend(q, K, V, 1.0) - want).max() > 1e-3


def test_attend_equal_keys_or_zero_query_gives_the_mean_value():
    D, n = 8, 7
    V = rnd((n, D), 7)
    K = np.repeat(rnd((1, D), 8), n, axis=0)
    np.testing.assert_allclose(orc.attend(rnd(D, 9), K, V, 0.5), V.astype(np.float64).mean(0), atol=1e-14)
    np.testing.assert_allclose(orc.attend(np.zeros(D, np.float32), rnd((n, D), 10), V, 0.5),
                               V.astype(np.float64).mean(0), atol=1e-14)


def test_attend_probabilities_sum_to_one_and_constant_value():
    D, n = 32, 300
    q, K = rnd(D, 11, 3.0), rnd((n, D), 12, 3.0)
    V = np.full((n, D), 0.625, np.float32)
    out, p = orc.attend(q, K, V, 1.0 / math.sqrt(D), want_probs=True)
    assert abs(p.sum() - 1.0) <= 1e-12 and (p >= 0).all()
    np.testing.assert_allclose(out, 0.625, atol=1e-13)


def test_attend_matches_library_softmax_and_matmul():
    # scipy's softmax and numpy's matmul as black boxes (float64)
    for n, D, seed in [(1, 4, 20), (5, 8, 21), (129, 64, 22), (1000, 128, 23)]:
        q, K, V = rnd(D, seed), rnd((n, D), seed + 100), rnd((n, D), seed + 200)
        scale = 1.0 / math.sqrt(D)
        p = scipy.special.softmax(scale * (K.astype(np.float64) @ q.astype(np.float64)))
        want = p @ V.astype(np.float64)
        out, probs = orc.attend(q, K, V, scale, want_probs=True)
        np.testing.assert_allclose(out, want, rtol=0, atol=1e-13)
        np.testing.assert_allclose(probs, p, rtol=0, atol=1e-15)


def test_attend_huge_scores_stay_finite_and_pick_the_needle():
    D, n = 64, 50
    q = rnd(D, 30)
    K, V = rnd((n, D), 31), rnd((n, D), 32)
    K[17] = 200.0 * math.sqrt(D) * q / np.linalg.norm(q)      # score ~ +1600: exp() of it overflows a double
    K[3] = -200.0 * math.sqrt(D) * q / np.linalg.norm(q)
    out, p = orc.attend(q, K, V, 1.0 / math.sqrt(D), want_probs=True)
    assert np.isfinite(out).all() and p[17] > 1 - 1e-12 and p[3] == 0.0
    np.testing.assert_allclose(out, V[17].astype(np.float64), atol=1e-10)


def test_attend_no_keys_is_the_zero_vector():
    # Section 2.1: the first token has nothing to attend to; zero dummy K/V give a zero output.
    out = orc.attend(rnd(8, 40), np.zeros((0, 8), np.float32), np.zeros((0, 8), np.float32), 1.0)
    assert (out == 0).all()


def test_attend_many_equals_attend():
    N, T, D = 9, 33, 16
    q, K, V = rnd((N, D), 50), rnd((N, T, D), 51), rnd((N, T, D), 52)
    n_keys = np.array([0, 1, 2, 5, 16, 17, 32, 33, 20])
    out, used = orc.attend_many(q, K, V, n_keys, 0.25, threads=3)
    assert used == 3
    for i in range(N):
        np.testing.assert_array_equal(out[i], orc.attend(q[i], K[i, : n_keys[i]], V[i, : n_keys[i]], 0.25))


# ---------------------------------------------------------------- the whole step

def sdpa64(q, K, V, scale):
    """torch's scaled_dot_product_attention in float64, used as a black box: q [H][D], K,V [H][n][D]."""
    qq = torch.from_numpy(q.astype(np.float64))[None, :, None, :]
    kk = torch.from_numpy(K.astype(np.float64))[None]
    vv = torch.from_numpy(V.astype(np.float64))[None]
    return torch.nn.functional.scaled_dot_product_attention(qq, kk, vv, scale=scale)[0, :, 0, :].numpy()


@pytest.mark.parametrize("rule", RULES)
@pytest.mark.parametrize("Hq,Hkv", [(4, 4), (8, 2)])
def test_all_warmup_step_is_standard_causal_attention(rule, Hq, Hkv):
    # Section 4.2: with every layer a warmup layer the model is the standard transformer:
    # layer l attends to its own cache, positions 0..t, the new token included.
    L, B, D, T_cap = 3, 3, 16, 12
    warm = [1] * L
    K, V, lens, q, kn, vn = make_state(L, B, Hq, Hkv, D, T_cap, warm, rule, 60, lens=[0, 5, 10])
    K0, V0, lens0 = K.copy(), V.copy(), lens.copy()
    scale = 1.0 / math.sqrt(D)
    out, _ = orc.step(warm, K, V, lens, q, kn, vn, scale, rule)
    G = Hq // Hkv
    for l in range(L):
        for b in range(B):
            t = lens0[b]
            Kfull = np.concatenate([K0[l, b, :t], kn[l, b][None]], 0)      # [t+1][Hkv][D]
            Vfull = np.concatenate([V0[l, b, :t], vn[l, b][None]], 0)
            Kh = np.repeat(Kfull.transpose(1, 0, 2), G, axis=0)           # query head h -> kv head h // G
            Vh = np.repeat(Vfull.transpose(1, 0, 2), G, axis=0)
            want = sdpa64(q[l, b], Kh, Vh, scale)
            np.testing.assert_allclose(out[l, b], want, rtol=0, atol=1e-13)
    assert (lens == lens0 + 1).all()


def expected_step_by_library(warm, rule_table, K0, V0, lens0, q, kn, vn, scale):
    """The step evaluated with library softmax/matmul from an explicit pairing table
    (slot, self_visible, producer) that the caller wrote down by hand."""
    slot, vis, prod = rule_table
    L, B, Hq, D = q.shape
    Hkv = K0.shape[3]
    G = Hq // Hkv
    out = np.zeros((L, B, Hq, D))
    for l in range(L):
        for b in range(B):
            t = int(lens0[b])
            s = slot[l]
            Ks, Vs = K0[s, b, :t].astype(np.float64), V0[s, b, :t].astype(np.float64)
            if vis[l]:
                assert prod[s] == l
                Ks = np.concatenate([Ks, kn[s, b][None].astype(np.float64)], 0)
                Vs = np.concatenate([Vs, vn[s, b][None].astype(np.float64)], 0)
            for h in range(Hq):
                g = h // G
                if Ks.shape[0] == 0:
                    continue
                p = scipy.special.softmax(scale * (Ks[:, g] @ q[l, b, h].astype(np.float64)))
                out[l, b, h] = p @ Vs[:, g]
    return out


HAND_TABLES = [
    # (warm, rule, (kv_slot, self_visible, producer)) written out from Section 2.1 by hand
    ([0, 0, 0], 0, ([0, 0, 0], [0, 0, 0], [2])),
    ([1, 0, 0, 0], 0, ([0, 1, 1, 1], [1, 0, 0, 0], [0, 3])),
    ([1, 0, 0, 1], 0, ([0, 1, 1, 2], [1, 0, 0, 1], [0, 2, 3])),
    ([1, 0, 0, 1], 1, ([0, 1, 1, 1], [1, 0, 0, 1], [0, 3])),
    ([0, 1, 0, 1, 1], 0, ([1, 0, 1, 2, 3], [0, 1, 0, 1, 1], [1, 2, 3, 4])),
    ([1, 1, 0, 0], 0, ([0, 1, 2, 2], [1, 1, 0, 0], [0, 1, 3])),
]


@pytest.mark.parametrize("warm,rule,table", HAND_TABLES)
def test_step_against_library_evaluation_with_hand_pairing(warm, rule, table):
    L, B, Hq, Hkv, D, T_cap = len(warm), 2, 4, 2, 8, 9
    K, V, lens, q, kn, vn = make_state(L, B, Hq, Hkv, D, T_cap, warm, rule, 70 + L, lens=[0, 6])
    K0, V0, lens0 = K.copy(), V.copy(), lens.copy()
    out, _ = orc.step(warm, K, V, lens, q, kn, vn, 0.3, rule)
    want = expected_step_by_library(warm, table, K0, V0, lens0, q, kn, vn, 0.3)
    np.testing.assert_allclose(out, want, rtol=0, atol=1e-13)


def test_step_first_token_condensed_layers_output_zero():
    # Section 2.1: t = 0, diagonal masked => nothing visible => zero output; warmup layers see only
    # the new token => output is exactly its value.
    warm = [1, 0, 0, 1]
    L, B, Hq, Hkv, D = 4, 2, 4, 2, 8
    K, V, lens, q, kn, vn = make_state(L, B, Hq, Hkv, D, 4, warm, 0, 80, lens=[0, 0])
    out, _ = orc.step(warm, K, V, lens, q, kn, vn, 0.5)
    assert np.isfinite(out).all()
    assert (out[1] == 0).all() and (out[2] == 0).all()
    for l, s in [(0, 0), (3, 2)]:
        for h in range(Hq):
            np.testing.assert_array_equal(out[l, :, h], vn[s, :, h // 2].astype(np.float64))


def test_step_visible_length_t_for_condensed_t_plus_1_for_warmup():
    # q = 0 makes the output the mean of the visible values: the count of visible keys shows directly.
    warm = [1, 0, 0]
    L, B, Hq, Hkv, D, T_cap = 3, 1, 2, 2, 4, 8
    K, V, lens, q, kn, vn = make_state(L, B, Hq, Hkv, D, T_cap, warm, 0, 90, lens=[5])
    q[:] = 0
    V0 = V.copy()
    out, _ = orc.step(warm, K, V, lens, q, kn, vn, 1.0)
    want_warm = (V0[0, 0, :5].astype(np.float64).sum(0) + vn[0, 0]) / 6.0
    want_cond = V0[1, 0, :5].astype(np.float64).mean(0)
    np.testing.assert_allclose(out[0, 0], want_warm, atol=1e-14)
    np.testing.assert_allclose(out[1, 0], want_cond, atol=1e-14)
    np.testing.assert_allclose(out[2, 0], want_cond, atol=1e-14)


def test_step_diagonal_is_masked_this_step_and_visible_next_step():
    # Section 2.1: a token does not attend to itself in condensed layers; its top-layer K/V first
    # become visible to the next token.
    warm = [1, 0, 0, 0]
    L, B, Hq, Hkv, D, T_cap = 4, 2, 2, 2, 8, 10
    base = make_state(L, B, Hq, Hkv, D, T_cap, warm, 0, 100, lens=[3, 7])

    def run(kn_scale):
        K, V, lens, q, kn, vn = [a.copy() for a in base]
        kn[1] *= kn_scale          # new K/V of the shared slot
        vn[1] *= kn_scale
        o1, _ = orc.step(warm, K, V, lens, q, kn, vn, 0.4)
        o2, _ = orc.step(warm, K, V, lens, q, kn, vn, 0.4)
        return o1, o2

    a1, a2 = run(1.0)
    b1, b2 = run(-3.0)
    np.testing.assert_array_equal(a1, b1)                       # invisible now
    assert np.abs(a2[1:] - b2[1:]).min(axis=-1).min() > 0       # every condensed output moves next step
    np.testing.assert_array_equal(a2[0], b2[0])                 # the warmup layer never sees that slot


def test_step_condensed_layers_share_one_cache_and_warmup_slots_are_private():
    warm = [1, 0, 0, 1]
    L, B, Hq, Hkv, D, T_cap = 4, 2, 4, 2, 8, 10
    K, V, lens, q, kn, vn = make_state(L, B, Hq, Hkv, D, T_cap, warm, 0, 110, lens=[4, 9])
    q[2] = q[1]
    o, _ = orc.step(warm, K.copy(), V.copy(), lens.copy(), q, kn, vn, 0.4)
    np.testing.assert_array_equal(o[1], o[2])                   # same q, same shared cache, same output
    K2 = K.copy()
    K2[2] += 1.0                                                # perturb the top warmup layer's slot
    o2, _ = orc.step(warm, K2, V.copy(), lens.copy(), q, kn, vn, 0.4)
    np.testing.assert_array_equal(o[:3], o2[:3])
    assert np.abs(o[3] - o2[3]).max() > 1e-6


def test_step_gqa_head_h_reads_kv_head_h_div_G():
    warm = [0, 0]
    L, B, Hq, Hkv, D, T_cap = 2, 1, 6, 3, 4, 6
    K, V, lens, q, kn, vn = make_state(L, B, Hq, Hkv, D, T_cap, warm, 0, 120, lens=[4])
    for g in range(Hkv):
        V[:, :, :, g, :] = 10.0 * (g + 1)          # a constant per kv head: the output names the head read
    out, _ = orc.step(warm, K, V, lens, q, kn, vn, 1.0)
    for h in range(Hq):
        np.testing.assert_allclose(out[:, 0, h], 10.0 * (h // 2 + 1), atol=1e-12)


def test_step_batch_permutation_invariance_is_bitwise():
    warm = [1, 0, 0, 1]
    L, B, Hq, Hkv, D, T_cap = 4, 5, 4, 2, 8, 12
    K, V, lens, q, kn, vn = make_state(L, B, Hq, Hkv, D, T_cap, warm, 0, 130)
    perm = np.array([3, 0, 4, 2, 1])
    o, _ = orc.step(warm, K.copy(), V.copy(), lens.copy(), q, kn, vn, 0.35)
    op, _ = orc.step(warm, np.ascontiguousarray(K[:, perm]), np.ascontiguousarray(V[:, perm]), lens[perm].copy(),
                     np.ascontiguousarray(q[:, perm]), np.ascontiguousarray(kn[:, perm]),
                     np.ascontiguousarray(vn[:, perm]), 0.35)
    np.testing.assert_array_equal(o[:, perm], op)


def test_step_append_copies_bits_at_position_t_and_nothing_else():
    warm = [1, 0, 0, 1]
    L, B, Hq, Hkv, D, T_cap = 4, 3, 2, 2, 4, 8
    K, V, lens, q, kn, vn = make_state(L, B, Hq, Hkv, D, T_cap, warm, 0, 140, lens=[0, 3, 6])
    kn[0, 0, 0, 0] = np.float32(-0.0)
    kn[1, 1, 1, 2] = np.float32(np.nan)            # bits, not values: a NaN payload must survive too
    q[:] = 0
    K0, V0, lens0 = K.copy(), V.copy(), lens.copy()
    orc.step(warm, K, V, lens, q, kn, vn, 1.0)
    for s in range(3):
        for b in range(B):
            t = lens0[b]
            assert K[s, b, t].tobytes() == kn[s, b].tobytes() and V[s, b, t].tobytes() == vn[s, b].tobytes()
            keep = np.ones(T_cap, bool)
            keep[t] = False
            assert K[s, b, keep].tobytes() == K0[s, b, keep].tobytes()
            assert V[s, b, keep].tobytes() == V0[s, b, keep].tobytes()
    assert (lens == lens0 + 1).all()


def test_step_needle_positions_including_the_boundary():
    # A key aligned with q and scaled up takes all the probability mass: the output names the position read.
    warm = [1, 0]
    L, B, Hq, Hkv, D, T_cap = 2, 1, 1, 1, 16, 40
    t = 33
    for pos in [0, 15, 16, 17, 31, 32, 33]:
        K, V, lens, q, kn, vn = make_state(L, B, Hq, Hkv, D, T_cap, warm, 0, 150, lens=[t])
        for l, s in [(0, 0), (1, 1)]:
            needle = 60.0 * q[l, 0, 0] / np.linalg.norm(q[l, 0, 0])
            if pos < t:
                K[s, 0, pos, 0] = needle
            else:
                kn[s, 0, 0] = needle
        Vall = [np.concatenate([V[s, 0, :t, 0], vn[s, 0]], 0) for s in range(2)]
        out, _ = orc.step(warm, K, V, lens, q, kn, vn, 1.0)
        np.testing.assert_allclose(out[0, 0, 0], Vall[0][pos], atol=1e-9)       # warmup sees 0..t
        if pos < t:
            np.testing.assert_allclose(out[1, 0, 0], Vall[1][pos], atol=1e-9)   # condensed sees 0..t-1
        else:
            assert np.abs(out[1, 0, 0] - Vall[1][pos]).max() > 1e-2


def test_step_rejects_a_full_sequence():
    warm = [0]
    K, V, lens, q, kn, vn = make_state(1, 1, 1, 1, 4, 4, warm, 0, 160, lens=[4])
    with pytest.raises(ValueError):
        orc.step(warm, K, V, lens, q, kn, vn, 1.0)


# ---------------------------------------------------------------- sink + window policy (Section 3.3)

def kept_positions(n, sink, window):
    """Written out by hand for the tests: first `sink` and last `window` of positions 0..n-1."""
    if window <= 0 or n <= sink + window:
        return list(range(n))
    return list(range(sink)) + list(range(n - window, n))


def test_streaming_kept_sets_by_hand():
    # StreamingLLM keeps the K/V of the first few tokens and of the recent tokens (Section 3.3).
    assert kept_positions(10, 2, 3) == [0, 1, 7, 8, 9]
    assert kept_positions(11, 2, 3) == [0, 1, 8, 9, 10]
    assert kept_positions(5, 2, 3) == [0, 1, 2, 3, 4]
    assert kept_positions(6, 4, 1) == [0, 1, 2, 3, 5]


def test_streaming_zero_query_gives_the_mean_over_the_kept_set():
    warm = [1, 0, 0]
    L, B, Hq, Hkv, D, T_cap = 3, 1, 2, 2, 4, 16
    K, V, lens, q, kn, vn = make_state(L, B, Hq, Hkv, D, T_cap, warm, 0, 200, lens=[10])
    q[:] = 0
    V0 = V.copy()
    out, _ = orc.step(warm, K, V, lens, q, kn, vn, 1.0, sink=2, window=3)
    # condensed layers: 10 candidates -> {0,1,7,8,9}; warmup layer: 11 candidates -> {0,1,8,9,new}
    want_cond = V0[1, 0, [0, 1, 7, 8, 9]].astype(np.float64).mean(0)
    want_warm = (V0[0, 0, [0, 1, 8, 9]].astype(np.float64).sum(0) + vn[0, 0]) / 5.0
    np.testing.assert_allclose(out[1, 0], want_cond, atol=1e-14)
    np.testing.assert_allclose(out[2, 0], want_cond, atol=1e-14)
    np.testing.assert_allclose(out[0, 0], want_warm, atol=1e-14)


def test_streaming_with_a_wide_window_equals_the_full_cache_bitwise():
    warm = [1, 0, 0, 1]
    L, B, Hq, Hkv, D, T_cap = 4, 3, 4, 2, 8, 20
    base = make_state(L, B, Hq, Hkv, D, T_cap, warm, 0, 210, lens=[0, 7, 15])
    a = [x.copy() for x in base]
    b = [x.copy() for x in base]
    oa, _ = orc.step(warm, *a, 0.3)
    ob, _ = orc.step(warm, *b, 0.3, sink=4, window=12)          # 4 + 12 >= 16 candidates: nothing dropped
    np.testing.assert_array_equal(oa, ob)


def test_streaming_matches_library_evaluation_on_the_hand_built_kept_set():
    warm = [0, 1, 0]
    L, B, Hq, Hkv, D, T_cap = 3, 2, 4, 2, 8, 40
    sink, window = 4, 6
    K, V, lens, q, kn, vn = make_state(L, B, Hq, Hkv, D, T_cap, warm, 0, 220, lens=[30, 9])
    K0, V0, lens0 = K.copy(), V.copy(), lens.copy()
    out, _ = orc.step(warm, K, V, lens, q, kn, vn, 0.4, sink=sink, window=window)
    slot, vis, prod = [1, 0, 1], [0, 1, 0], [1, 2]              # by hand: layer 1 warm, top condensed layer 2
    for l in range(L):
        s = slot[l]
        for b in range(B):
            t = int(lens0[b])
            Ks, Vs = K0[s, b, :t].astype(np.float64), V0[s, b, :t].astype(np.float64)
            if vis[l]:
                Ks = np.concatenate([Ks, kn[s, b][None]], 0)
                Vs = np.concatenate([Vs, vn[s, b][None]], 0)
            keep = kept_positions(Ks.shape[0], sink, window)
            for h in range(Hq):
                g = h // 2
                p = scipy.special.softmax(0.4 * (Ks[keep, g] @ q[l, b, h].astype(np.float64)))
                np.testing.assert_allclose(out[l, b, h], p @ Vs[keep, g], rtol=0, atol=1e-13)


def test_streaming_needles_evicted_sink_and_window_edges():
    warm = [0]
    L, B, Hq, Hkv, D, T_cap = 1, 1, 1, 1, 16, 64
    sink, window, t = 4, 8, 40                   # kept: 0..3 and 32..39
    for pos, visible in [(0, True), (3, True), (4, False), (20, False), (31, False), (32, True), (39, True)]:
        K, V, lens, q, kn, vn = make_state(L, B, Hq, Hkv, D, T_cap, warm, 0, 230, lens=[t])
        K[0, 0, pos, 0] = 60.0 * q[0, 0, 0] / np.linalg.norm(q[0, 0, 0])
        target = V[0, 0, pos, 0].astype(np.float64)
        out, _ = orc.step(warm, K, V, lens, q, kn, vn, 1.0, sink=sink, window=window)
        if visible:
            np.testing.assert_allclose(out[0, 0, 0], target, atol=1e-9)
        else:
            assert np.abs(out[0, 0, 0] - target).max() > 1e-2


def test_streaming_window_slides_one_position_per_step():
    warm = [0, 0]
    L, B, Hq, Hkv, D, T_cap = 2, 1, 1, 1, 4, 32
    K, V, lens, q, kn, vn = make_state(L, B, Hq, Hkv, D, T_cap, warm, 0, 240, lens=[12])
    q[:] = 0
    for step in range(4):
        t = 12 + step
        V_before = V.copy()
        out, _ = orc.step(warm, K, V, lens, q, kn, vn, 1.0, sink=1, window=5)
        keep = [0] + list(range(t - 5, t))
        np.testing.assert_allclose(out[0, 0, 0], V_before[0, 0, keep, 0].astype(np.float64).mean(0), atol=1e-14)
