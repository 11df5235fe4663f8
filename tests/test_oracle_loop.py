"""Pins for the oracle's state update and its Algorithm 1 driver — CPU only.

The driver is pinned by a brute-force replay of Algorithm 1 in python floats on a tiny problem (sets as python
sets, softmax written out, Top-K by numpy.lexsort) and by what the paper's state machine fixes: I_sel frozen
between slow steps (Eq. freeze_sel), I_sel inside J of its refresh step (Eq. allowed_set), the recent window
sliding with t, an all-slow schedule giving dense attention at every length.
"""
import math

import numpy as np

import sfi_synth as syn


def test_advance_closed_form(oracle):
    """After t updates from length L0: L = L0 + t and the window is the last `recent` rows, never reaching into
    the sink."""
    n_sink, recent = 4, 16
    L = np.array([1, 3, 4, 5, 19, 20, 21, 100], np.int32)
    rs = np.maximum(n_sink, L - recent).astype(np.int32)
    L0 = L.copy()
    for t in range(1, 40):
        L, rs = oracle.advance(L, rs, n_sink, recent)
        assert (L == L0 + t).all()
        for b in range(len(L)):
            window = set(range(int(rs[b]), int(L[b])))
            want = set(range(int(L[b]))[-recent:]) - set(range(n_sink))
            assert window == want
            # sink, J and the window partition the prefix (Eq. allowed_set)
            J = set(range(n_sink, int(L[b]) - recent))
            assert not (J & window) and (set(range(min(n_sink, int(L[b])))) | J | window) == set(range(int(L[b])))


def _f(bits):
    return syn.bf16_bits_to_f32(bits).astype(np.float64)


def _attend(q, K, V, rows, scale):
    rows = sorted(rows)
    l = np.array([scale * float(np.dot(q, K[j])) for j in rows])
    w = np.exp(l - l.max())
    return (w[:, None] * V[rows]).sum(0) / w.sum()


def test_decode_loop_brute_force(oracle):
    """Tiny problem, every step replayed in python: B = 2 (different lengths and schedules), G = 2, d = 8."""
    B, Hq, Hkv, d, n_sink, recent, budget, T = 2, 4, 2, 8, 2, 3, 4, 9
    G = Hq // Hkv
    rng = syn.rng_for(90, 1)
    L0 = np.array([11, 7], np.int32)
    La = int(L0.max()) + T
    K = syn.f32_to_bf16_bits(rng.standard_normal((B, Hkv, La, d)).astype(np.float32) * 1.5)
    V = syn.f32_to_bf16_bits(rng.standard_normal((B, Hkv, La, d)).astype(np.float32))
    q = syn.f32_to_bf16_bits(rng.standard_normal((T, B, Hq, d)).astype(np.float32) * 1.5)
    g = np.zeros((T, B), np.uint8)
    g[[0, 4, 5], 0] = 1
    g[[0, 2, 7], 1] = 1
    scale = 1.0 / math.sqrt(d)
    res = oracle.decode_loop(q, K, V, L0, np.maximum(n_sink, L0 - recent), g, budget, n_sink, recent)
    Kf, Vf, qf = _f(K), _f(V), _f(q)
    sel = [[set() for _ in range(Hkv)] for _ in range(B)]
    for t in range(T):
        for b in range(B):
            L = int(L0[b]) + t
            assert res["ctx_hist"][t, b] == L and res["rs_hist"][t, b] == max(n_sink, L - recent)
            sink = set(range(min(n_sink, L)))
            window = set(range(max(n_sink, L - recent), L))
            J = list(range(n_sink, L - recent))
            for h in range(Hkv):
                rows = set(range(L)) if g[t, b] else sink | window | sel[b][h]
                for gg in range(G):
                    want = _attend(qf[t, b, h * G + gg], Kf[b, h], Vf[b, h], rows, scale)
                    np.testing.assert_allclose(res["out"][t, b, h * G + gg], want, rtol=1e-11, atol=1e-13)
                if g[t, b]:
                    f = np.zeros(len(J))
                    for gg in range(G):
                        l = np.array([scale * float(np.dot(qf[t, b, h * G + gg], Kf[b, h, j])) for j in J])
                        e = np.exp(l - l.max())
                        f += e / e.sum() / G
                    order = np.lexsort((np.array(J), -np.log(f + 1e-8)))[:budget]
                    sel[b][h] = set(int(J[i]) for i in order)
                k = int(res["nsel_hist"][t, b, h])
                assert set(int(x) for x in res["sel_hist"][t, b, h, :k]) == sel[b][h]
                assert (res["sel_hist"][t, b, h, k:] == -1).all()
    assert (res["ctx_len"] == L0 + T).all()


def test_decode_loop_state_machine_properties(oracle):
    w = syn.make_tiny(L0=300, steps=12, budget=16, recent=20, n_support=6, B=2, Hq=4, Hkv=2)
    w.L0 = np.array([300, 180], np.int32)
    T = 12
    q = np.stack([w.q(t) for t in range(T)])
    g = np.zeros((T, 2), np.uint8)
    g[[0, 5, 11], 0] = 1
    g[[0, 3], 1] = 1
    res = oracle.decode_loop(q, w.K, w.V, w.ctx_len(0), w.recent_start(0), g, w.budget, w.n_sink, w.recent)
    for b in range(2):
        last = None
        for t in range(T):
            L = int(w.L0[b]) + t
            cur = res["sel_hist"][t, b]
            if g[t, b]:
                # refreshed inside J of this step, equal to the Selector called on its own
                s, n, _ = oracle.selector(q[t][b:b + 1], w.K[b:b + 1], [L], w.budget, w.n_sink, w.recent)
                assert (cur == s[0]).all() and cur.min() >= w.n_sink and cur.max() < L - w.recent
                d1 = oracle.dense(q[t][b:b + 1], w.K[b:b + 1], w.V[b:b + 1], [L])
                np.testing.assert_array_equal(res["out"][t, b], d1[0])
            else:
                assert (cur == last).all()                     # Eq. freeze_sel
                sp = oracle.sparse(q[t][b:b + 1], w.K[b:b + 1], w.V[b:b + 1], last[None], res["nsel_hist"][t, b][None],
                                   [max(w.n_sink, L - w.recent)], [L], w.n_sink)
                np.testing.assert_array_equal(res["out"][t, b], sp[0])
            last = cur
    # all-slow schedule: dense attention at every length
    res2 = oracle.decode_loop(q[:3], w.K, w.V, w.ctx_len(0), w.recent_start(0), np.ones((3, 2), np.uint8), w.budget,
                              w.n_sink, w.recent)
    for t in range(3):
        np.testing.assert_array_equal(res2["out"][t], oracle.dense(q[t], w.K, w.V, w.ctx_len(t)))
    # a fast step before any refresh attends to sink and window only
    res3 = oracle.decode_loop(q[:1], w.K, w.V, w.ctx_len(0), w.recent_start(0), np.zeros((1, 2), np.uint8), w.budget,
                              w.n_sink, w.recent)
    empty = np.full((2, 2, w.budget), -1, np.int32)
    np.testing.assert_array_equal(res3["out"][0], oracle.sparse(q[0], w.K, w.V, empty, np.zeros((2, 2), np.int32),
                                                                w.recent_start(0), w.ctx_len(0), w.n_sink))
