"""Pins for the oracle's windowed evidence with a per-query causal mask (Eq. window_logits, Eqs. selector_pt,
selector_mu, selector_f) — CPU only.

The window's W queries are handed in as W * G vectors per KV head; vector (b, g) sees rows [0, vis[b, g]).
Pins: the equations written out with numpy on the visible parts, and what the mask implies: a vector that sees
all of J is unmasked; one that sees nothing of J only rescales mu (f unchanged); positions no vector sees carry
f = 0 and rank last, lower index first.
"""
import numpy as np
import pytest

import sfi_synth as syn
from oracle.sfi_oracle import SelectorParams

EPS = 1e-8


def _softmax(x):
    e = np.exp(x - x.max())
    return e / e.sum()


@pytest.mark.parametrize("alpha", [1.0, 0.5])
def test_masked_window_matches_the_equations(oracle, alpha):
    rng = syn.rng_for(70, 1)
    B, Hkv, W, G, L, n_sink, R, K = 2, 2, 5, 2, 90, 4, 2, 13
    Hq = Hkv * W * G
    lg = rng.standard_normal((B, Hq, L)) * 2.0
    # window query tau sits at row L - W + tau and sees rows up to its own; R < W: the first queries miss the tail of J
    vis = np.zeros((B, Hq), np.int32)
    for h in range(Hkv):
        for t in range(W):
            vis[:, h * W * G + t * G:h * W * G + (t + 1) * G] = L - W + t + 1
    j_hi = L - R
    assert vis.min() < j_hi <= vis.max()
    sel, nsel, z, dbg = oracle.selector_from_logits(lg, [L] * B, Hkv, K, n_sink, R, sp=SelectorParams(alpha=alpha),
                                                    debug=True, vis=vis)
    for b in range(B):
        for h in range(Hkv):
            mu = np.zeros(j_hi - n_sink)
            for v in range(W * G):
                g = h * W * G + v
                end = min(j_hi, int(vis[b, g]))
                p = np.zeros(j_hi - n_sink)
                p[:end - n_sink] = _softmax(lg[b, g, n_sink:end])
                mu += p ** alpha / (W * G)
            f = mu ** (1.0 / alpha)
            f /= f.sum()
            np.testing.assert_allclose(dbg["f"][b, h, n_sink:j_hi], f, rtol=1e-11, atol=1e-300)
            zz = np.log(f + EPS)
            np.testing.assert_allclose(z[b, h, n_sink:j_hi], zz, rtol=1e-11)
            j = np.arange(n_sink, j_hi)
            assert list(sel[b, h]) == sorted(j[np.lexsort((j, -zz))[:K]])


def test_mask_special_cases(oracle):
    rng = syn.rng_for(71, 1)
    B, Hkv, V, L, n_sink, R, K = 1, 1, 6, 60, 3, 4, 50
    lg = rng.standard_normal((B, V, L)) * 2.0
    j_hi = L - R
    # every vector sees all of J (recent >= W): the mask changes nothing
    a = oracle.selector_from_logits(lg, [L], Hkv, K, n_sink, R, vis=np.full((B, V), j_hi))
    b = oracle.selector_from_logits(lg, [L], Hkv, K, n_sink, R)
    c = oracle.selector_from_logits(lg, [L], Hkv, K, n_sink, R, vis=np.full((B, V), L))
    for x in (a, c):
        np.testing.assert_array_equal(x[0], b[0])
        np.testing.assert_array_equal(x[2], b[2])
    # a vector that sees nothing of J only rescales mu: f, z and the selection are those of the other vectors alone
    vis = np.full((B, V), L, np.int32)
    vis[0, 2] = n_sink
    vis[0, 4] = 1
    d = oracle.selector_from_logits(lg, [L], Hkv, K, n_sink, R, vis=vis)
    e = oracle.selector_from_logits(lg[:, [0, 1, 3, 5]], [L], Hkv, K, n_sink, R)
    np.testing.assert_array_equal(d[0], e[0])
    np.testing.assert_allclose(d[2][0, 0, n_sink:j_hi], e[2][0, 0, n_sink:j_hi], rtol=1e-12)
    # positions beyond every vector's view: f = 0, z = log(eps) exactly, taken last and in index order
    vis = np.full((B, V), 30, np.int32)
    s, n, z, dbg = oracle.selector_from_logits(lg, [L], Hkv, K, n_sink, R, vis=vis, debug=True)
    assert (dbg["f"][0, 0, 30:j_hi] == 0).all() and (z[0, 0, 30:j_hi] == np.log(EPS)).all()
    assert abs(dbg["f"][0, 0, n_sink:30].sum() - 1.0) < 1e-12
    assert n[0, 0] == K
    seen = 30 - n_sink
    assert set(range(n_sink, 30)) <= set(s[0, 0, :K]) and sorted(set(s[0, 0, :K]) - set(range(n_sink, 30))) == list(range(30, 30 + K - seen))


def test_masked_window_from_q_and_k(oracle):
    """sfio_selector applies the same mask to logits it computes itself."""
    w = syn.make_tiny(L0=260, steps=1, budget=20, recent=4, n_support=4, B=1, Hq=8, Hkv=2)
    q = w.q(0)
    vis = np.array([[260, 259, 258, 200, 260, 257, 256, 3]], np.int32)
    lg = oracle.logits(q, w.K, w.ctx_len(0))
    a = oracle.selector(q, w.K, w.ctx_len(0), w.budget, w.n_sink, w.recent, vis=vis)
    b = oracle.selector_from_logits(lg, w.ctx_len(0), w.Hkv, w.budget, w.n_sink, w.recent, vis=vis)
    np.testing.assert_array_equal(a[0], b[0])
    np.testing.assert_array_equal(a[2], b[2])
    c = oracle.selector(q, w.K, w.ctx_len(0), w.budget, w.n_sink, w.recent)
    assert not np.array_equal(a[2], c[2])
