"""Pins for the oracle's all-prompt-tokens attention (Sections 2.2 and 2.3), no GPU.

The strongest pin is the paper's own Lemma 1 (Appendix A): in the parallel computation graph, where every
iteration pairs the queries of all layers with the top-layer K/V of the previous iteration, the computation of the
i-th token is identical to sequential decoding from iteration i on, whatever the initial K/V.  A toy model (random
linear maps, residual stream, tanh) is run both ways: token by token with the oracle's single-query attention and
a hand-kept cache, and in parallel iterations with the oracle's prefill attention.  This ties the prefill mask
(strictly lower triangular for condensed layers, causal for warmup layers) to the decode semantics."""
import math

import numpy as np
import pytest
import scipy.special
import torch

from oracle import lckv_oracle as orc


def rnd(shape, seed, sigma=1.0):
    return (np.random.default_rng(seed).standard_normal(shape) * sigma).astype(np.float32)


# ---------------------------------------------------------------- closed forms and library evaluations

def test_prefill_zero_query_gives_prefix_means():
    B, S, Hkv, D = 1, 6, 1, 4
    K, V = rnd((B, S, Hkv, D), 1), rnd((B, S, Hkv, D), 2)
    q = np.zeros((B, S, 1, D), np.float32)
    cond, _ = orc.prefill_attention(K, V, [S], q, False, 1.0)
    warm, _ = orc.prefill_attention(K, V, [S], q, True, 1.0)
    assert (cond[0, 0] == 0).all()                               # first token: zero dummy K/V (Section 2.1)
    for i in range(S):
        if i > 0:
            np.testing.assert_allclose(cond[0, i, 0], V[0, :i, 0].astype(np.float64).mean(0), atol=1e-14)
        np.testing.assert_allclose(warm[0, i, 0], V[0, : i + 1, 0].astype(np.float64).mean(0), atol=1e-14)


def test_prefill_warmup_layer_is_library_causal_attention():
    B, S, Hq, Hkv, D = 2, 9, 4, 2, 8
    K, V, q = rnd((B, S, Hkv, D), 3), rnd((B, S, Hkv, D), 4), rnd((B, S, Hq, D), 5)
    scale = 1.0 / math.sqrt(D)
    out, _ = orc.prefill_attention(K, V, [S, S], q, True, scale)
    G = Hq // Hkv
    for b in range(B):
        qq = torch.from_numpy(q[b].astype(np.float64)).permute(1, 0, 2)[None]                 # [1][Hq][S][D]
        kk = torch.from_numpy(np.repeat(K[b].astype(np.float64), G, axis=1)).permute(1, 0, 2)[None]
        vv = torch.from_numpy(np.repeat(V[b].astype(np.float64), G, axis=1)).permute(1, 0, 2)[None]
        want = torch.nn.functional.scaled_dot_product_attention(qq, kk, vv, is_causal=True, scale=scale)
        np.testing.assert_allclose(out[b], want[0].permute(1, 0, 2).numpy(), rtol=0, atol=1e-13)


def test_prefill_condensed_layer_is_strictly_lower_triangular():
    # library softmax over an explicit mask matrix
    B, S, Hq, Hkv, D = 1, 7, 2, 1, 8
    K, V, q = rnd((B, S, Hkv, D), 6), rnd((B, S, Hkv, D), 7), rnd((B, S, Hq, D), 8)
    out, _ = orc.prefill_attention(K, V, [S], q, False, 0.35)
    for h in range(Hq):
        scores = 0.35 * (q[0, :, h].astype(np.float64) @ K[0, :, 0].astype(np.float64).T)    # [S][S]
        mask = np.tril(np.ones((S, S), bool), k=-1)
        for i in range(1, S):
            p = scipy.special.softmax(scores[i, mask[i]])
            np.testing.assert_allclose(out[0, i, h], p @ V[0, mask[i], 0].astype(np.float64), atol=1e-13)
        assert (out[0, 0, h] == 0).all()


def test_prefill_ragged_lengths_rows_past_the_prompt_are_zero_and_do_not_matter():
    B, S, Hq, Hkv, D = 3, 8, 2, 2, 4
    K, V, q = rnd((B, S, Hkv, D), 9), rnd((B, S, Hkv, D), 10), rnd((B, S, Hq, D), 11)
    lens = [8, 3, 0]
    out, _ = orc.prefill_attention(K, V, lens, q, True, 0.5)
    assert (out[1, 3:] == 0).all() and (out[2] == 0).all() and np.abs(out[1, :3]).min() > 0
    K2, V2 = K.copy(), V.copy()
    K2[1, 3:], V2[1, 3:] = 99.0, -99.0                            # beyond the prompt: must not be read
    out2, _ = orc.prefill_attention(K2, V2, lens, q, True, 0.5)
    np.testing.assert_array_equal(out, out2)


def test_prefill_row_i_equals_single_query_attention_over_the_prefix():
    B, S, Hq, Hkv, D = 1, 12, 4, 2, 8
    K, V, q = rnd((B, S, Hkv, D), 12), rnd((B, S, Hkv, D), 13), rnd((B, S, Hq, D), 14)
    for vis in (False, True):
        out, _ = orc.prefill_attention(K, V, [S], q, vis, 0.3)
        for i in (0, 1, 5, 11):
            n = i + (1 if vis else 0)
            for h in range(Hq):
                want = orc.attend(q[0, i, h], K[0, :n, h // 2], V[0, :n, h // 2], 0.3)
                np.testing.assert_array_equal(out[0, i, h], want)


# ---------------------------------------------------------------- Lemma 1 (Appendix A) on a toy model

class ToyModel:
    """L layers on a residual stream of width Hq*D; layer l: q = Wq h, (k, v) = (Wk h, Wv h) from the layer's
    input, h <- h + tanh(Wo attn).  Which K/V a layer reads follows the oracle's pairing table."""

    def __init__(self, L, Hq, Hkv, D, warm, seed):
        self.L, self.Hq, self.Hkv, self.D, self.warm = L, Hq, Hkv, D, list(warm)
        W = Hq * D
        r = np.random.default_rng(seed)
        self.Wq = r.standard_normal((L, W, W)).astype(np.float32) / math.sqrt(W)
        self.Wk = r.standard_normal((L, Hkv * D, W)).astype(np.float32) / math.sqrt(W)
        self.Wv = r.standard_normal((L, Hkv * D, W)).astype(np.float32) / math.sqrt(W)
        self.Wo = r.standard_normal((L, W, W)).astype(np.float32) / math.sqrt(W)
        self.slot, self.vis, self.prod = orc.pairing(warm)
        self.scale = 1.0 / math.sqrt(D)

    def f32(self, x):
        return np.asarray(x, np.float32)

    def sequential(self, X):
        """Token by token, bottom-up (Figure 2a): returns final hidden states [n][W] and the caches."""
        n = X.shape[0]
        ns = len(self.prod)
        Kc = np.zeros((ns, n, self.Hkv, self.D), np.float32)
        Vc = np.zeros_like(Kc)
        H = np.zeros((n, X.shape[1]), np.float32)
        for i in range(n):
            h = X[i].copy()
            pending = {}
            for l in range(self.L):
                k = self.f32(self.Wk[l] @ h).reshape(self.Hkv, self.D)
                v = self.f32(self.Wv[l] @ h).reshape(self.Hkv, self.D)
                s = int(self.slot[l])
                if self.vis[l]:                         # warmup layer: own cache, itself included
                    Kc[s, i], Vc[s, i] = k, v
                elif self.prod[s] == l:                 # top condensed layer: visible from the next token on
                    pending[s] = (k, v)
                q = self.f32(self.Wq[l] @ h).reshape(self.Hq, self.D)
                nkeys = i + (1 if self.vis[l] else 0)
                G = self.Hq // self.Hkv
                a = np.concatenate([orc.attend(q[hh], Kc[s, :nkeys, hh // G], Vc[s, :nkeys, hh // G], self.scale)
                                    for hh in range(self.Hq)])
                h = self.f32(h + np.tanh(self.Wo[l] @ self.f32(a)))
            for s, (k, v) in pending.items():
                Kc[s, i], Vc[s, i] = k, v
            H[i] = h
        return H, Kc, Vc

    def parallel(self, X, iterations, init_seed=None):
        """All tokens at once, `iterations` times (Figure 2b); iteration t pairs the condensed layers with the
        shared K/V of iteration t-1 (zeros, or anything, before the first).  Returns the hidden states of every
        iteration [iterations][n][W]."""
        n = X.shape[0]
        ns = len(self.prod)
        shape = (ns, 1, n, self.Hkv, self.D)
        if init_seed is None:
            Kprev, Vprev = np.zeros(shape, np.float32), np.zeros(shape, np.float32)
        else:
            Kprev, Vprev = rnd(shape, init_seed), rnd(shape, init_seed + 1)
        hist = []
        for _ in range(iterations):
            Hcur = X.copy()
            Knew, Vnew = Kprev.copy(), Vprev.copy()
            for l in range(self.L):
                k = self.f32(Hcur @ self.Wk[l].T).reshape(n, self.Hkv, self.D)
                v = self.f32(Hcur @ self.Wv[l].T).reshape(n, self.Hkv, self.D)
                s = int(self.slot[l])
                q = self.f32(Hcur @ self.Wq[l].T).reshape(1, n, self.Hq, self.D)
                if self.vis[l]:
                    a, _ = orc.prefill_attention(k[None], v[None], [n], q, True, self.scale)
                else:
                    a, _ = orc.prefill_attention(Kprev[s], Vprev[s], [n], q, False, self.scale)
                    if self.prod[s] == l:
                        Knew[s, 0], Vnew[s, 0] = k, v
                Hcur = self.f32(Hcur + np.tanh(self.f32(a.reshape(n, -1)) @ self.Wo[l].T))
            Kprev, Vprev = Knew, Vnew
            hist.append(Hcur)
        return np.stack(hist)


@pytest.mark.parametrize("warm", [[0, 0, 0], [1, 0, 0, 1], [0, 1, 0]])
def test_lemma_1_token_i_is_exact_from_iteration_i_on(warm):
    n = 6
    m = ToyModel(len(warm), Hq=2, Hkv=1, D=4, warm=warm, seed=77)
    X = rnd((n, 8), 78)
    H_seq, _, _ = m.sequential(X)
    H_par = m.parallel(X, n)
    for t in range(1, n + 1):                     # iteration t (1-based): tokens 1..t are exact
        np.testing.assert_allclose(H_par[t - 1][:t], H_seq[:t], rtol=0, atol=2e-6)
    if any(w == 0 for w in warm):                 # and the later tokens are in general not yet exact early on
        assert np.abs(H_par[0][n - 1] - H_seq[n - 1]).max() > 1e-4


def test_lemma_1_holds_for_any_initial_kv():
    warm = [1, 0, 0]
    n = 5
    m = ToyModel(3, Hq=2, Hkv=2, D=4, warm=warm, seed=79)
    X = rnd((n, 8), 80)
    H_seq, _, _ = m.sequential(X)
    H_par = m.parallel(X, n, init_seed=81)        # garbage instead of zero dummy K/V
    np.testing.assert_allclose(H_par[-1], H_seq, rtol=0, atol=2e-6)
