"""Pins for the oracle's Selector (Algorithm 2) — CPU only.

Mode 0 (evidence only) is the hot path; mode 1 adds prior, fusion and the two
log-score refinements.  Pins: hand-computed small cases, closed forms and
properties the paper states (Sec. 3.2, Sec. 3.3), brute-force sorting.
"""
import math

import numpy as np
import pytest

import sfi_synth as syn
from oracle.sfi_oracle import SelectorParams

EPS = 1e-8


def softmax(x):
    x = np.asarray(x, np.float64)
    e = np.exp(x - x.max())
    return e / e.sum()


def run(oracle, lg, L, Hkv, budget, n_sink, recent, sp=None, knorm=None, debug=False):
    lg = np.asarray(lg, np.float64)
    return oracle.selector_from_logits(lg, [L] * lg.shape[0], Hkv, budget, n_sink, recent, sp=sp, knorm=knorm,
                                       debug=debug)


# ------------------------------------------------------------------ mode 0

def test_hand_case_power_mean(oracle):
    """J of 3 positions, G = 2 heads with p_1 = (1/4, 1/2, 1/4), p_2 = (1/2, 1/4, 1/4).
    alpha = 1:   f = (3/8, 3/8, 1/4).
    alpha = 1/2: mu = (sqrt(1/4)+sqrt(1/2), sqrt(1/2)+sqrt(1/4), 2 sqrt(1/4)) / 2, f ~ mu^2 normalised."""
    lg = np.log(np.array([[[9.0, 1, 2, 1, 9.0], [9.0, 2, 1, 1, 9.0]]]))   # positions 0 and 4 are sink / recent
    sel, nsel, z, dbg = run(oracle, lg, 5, 1, 2, 1, 1, debug=True)
    np.testing.assert_allclose(dbg["f"][0, 0, 1:4], [3 / 8, 3 / 8, 1 / 4], rtol=1e-14)
    np.testing.assert_allclose(z[0, 0, 1:4], np.log(np.array([3 / 8, 3 / 8, 1 / 4]) + EPS), rtol=1e-14)
    assert np.isneginf(z[0, 0, 0]) and np.isneginf(z[0, 0, 4])
    # equal scores at positions 1 and 2: both taken with K = 2; with K = 1 the lower index wins
    assert list(sel[0, 0]) == [1, 2] and nsel[0, 0] == 2
    sel1, _, _ = run(oracle, lg, 5, 1, 1, 1, 1)
    assert list(sel1[0, 0]) == [1]
    a, b = math.sqrt(0.25), math.sqrt(0.5)
    mu = np.array([(a + b) / 2, (b + a) / 2, a])
    f_half = mu ** 2 / (mu ** 2).sum()
    _, _, _, dbg2 = run(oracle, lg, 5, 1, 2, 1, 1, sp=SelectorParams(alpha=0.5), debug=True)
    np.testing.assert_allclose(dbg2["f"][0, 0, 1:4], f_half, rtol=1e-14)


def test_single_head_evidence_is_softmax_over_J(oracle):
    """G = 1 (W = 1): f = p_1 exactly, for any alpha; softmax runs over J only."""
    rng = syn.rng_for(40, 1)
    L, n_sink, R = 200, 4, 16
    lg = rng.standard_normal((2, 3, L)) * 3.0
    lg[:, :, :n_sink] += 50.0          # huge sink / recent logits must not leak into the evidence
    lg[:, :, L - R:] += 50.0
    for alpha in (1.0, 0.5, 0.3):
        sel, nsel, z, dbg = run(oracle, lg, L, 3, 10, n_sink, R, sp=SelectorParams(alpha=alpha), debug=True)
        for b in range(2):
            for h in range(3):
                p = softmax(lg[b, h, n_sink:L - R])
                np.testing.assert_allclose(dbg["f"][b, h, n_sink:L - R], p, rtol=1e-11)
                np.testing.assert_allclose(z[b, h, n_sink:L - R], np.log(p + EPS), rtol=1e-11)
                assert abs(dbg["f"][b, h].sum() - 1.0) < 1e-12
                assert sel[b, h].min() >= n_sink and sel[b, h].max() < L - R


def test_group_evidence_mean_of_softmaxes_and_topk_bruteforce(oracle):
    rng = syn.rng_for(41, 1)
    B, Hq, Hkv, L, n_sink, R, K = 2, 8, 2, 500, 4, 32, 37
    G = Hq // Hkv
    lg = rng.standard_normal((B, Hq, L)) * 2.0
    sel, nsel, z = run(oracle, lg, L, Hkv, K, n_sink, R)
    for b in range(B):
        for h in range(Hkv):
            f = np.mean([softmax(lg[b, h * G + g, n_sink:L - R]) for g in range(G)], axis=0)
            zz = np.log(f + EPS)
            np.testing.assert_allclose(z[b, h, n_sink:L - R], zz, rtol=1e-11)
            j = np.arange(n_sink, L - R)
            order = np.lexsort((j, -zz))[:K]
            assert nsel[b, h] == K
            assert list(sel[b, h]) == sorted(j[order])
    # evidence is invariant to a per-head shift of the logits
    shift = rng.standard_normal((B, Hq, 1)) * 5.0
    sel2, _, z2 = run(oracle, lg + shift, L, Hkv, K, n_sink, R)
    np.testing.assert_array_equal(sel2, sel)
    np.testing.assert_allclose(z2[:, :, n_sink:L - R], z[:, :, n_sink:L - R], rtol=1e-10)


def test_topk_ties_lower_index_wins(oracle):
    L, n_sink, R = 40, 2, 4
    lg = np.zeros((1, 2, L))
    lg[0, :, [7, 20, 30]] = 2.0        # three equal maxima; everything else equal too
    sel, nsel, _ = run(oracle, lg, L, 1, 5, n_sink, R)
    assert list(sel[0, 0]) == [2, 3, 7, 20, 30]
    sel, _, _ = run(oracle, lg, L, 1, 2, n_sink, R)
    assert list(sel[0, 0]) == [7, 20]


def test_budget_edge_cases(oracle):
    L, n_sink, R = 30, 4, 8
    lg = syn.rng_for(42, 1).standard_normal((1, 2, L))
    sel, nsel, _ = run(oracle, lg, L, 2, 64, n_sink, R)       # K >= |J| -> all of J, padded with -1
    nJ = L - R - n_sink
    for h in range(2):
        assert nsel[0, h] == nJ
        assert list(sel[0, h, :nJ]) == list(range(n_sink, L - R))
        assert (sel[0, h, nJ:] == -1).all()
    for Ls in (1, 4, 11, 12):                                   # J empty
        sel, nsel, _ = run(oracle, lg[:, :, :max(Ls, 1)], Ls, 2, 5, n_sink, R)
        assert (nsel == 0).all() and (sel == -1).all()
    sel, nsel, _ = run(oracle, lg[:, :, :13], 13, 2, 5, n_sink, R)  # |J| = 1
    assert (nsel == 1).all() and (sel[:, :, 0] == 4).all() and (sel[:, :, 1:] == -1).all()


def test_planted_support_rows_are_selected(oracle):
    """Tiny-config structure: support key rows aligned with the query (scale x4) must all be selected."""
    w = syn.make_tiny(L0=1024, steps=1, budget=64, recent=32, n_support=16)
    d = w.d
    qf = np.zeros((w.B, w.Hq, d), np.float32)
    Kf = syn.bf16_bits_to_f32(w.K).copy()
    dirs = syn.rng_for(43, 1).standard_normal((w.Hkv, d)).astype(np.float32)
    for h in range(w.Hkv):
        u = dirs[h] / np.linalg.norm(dirs[h])
        for g in range(w.G):
            qf[0, h * w.G + g] = u * 12.0
        for j in w.support[0, h]:
            Kf[0, h, j] = u * (4.0 * math.sqrt(d))     # norm of a x4 N(0,1) row, aligned with q
    q, K = syn.f32_to_bf16_bits(qf), syn.f32_to_bf16_bits(Kf)
    sel, nsel, _ = oracle.selector(q, K, w.ctx_len(0), w.budget, w.n_sink, w.recent)
    for h in range(w.Hkv):
        assert set(int(x) for x in w.support[0, h]) <= set(int(x) for x in sel[0, h])
        assert nsel[0, h] == w.budget


def test_selector_from_qk_equals_from_logits(oracle):
    w = syn.make_tiny(L0=300, steps=1, budget=20, recent=16, n_support=4)
    q = w.q(0)
    lg = oracle.logits(q, w.K, w.ctx_len(0))
    a = oracle.selector(q, w.K, w.ctx_len(0), w.budget, w.n_sink, w.recent)
    b = oracle.selector_from_logits(lg, w.ctx_len(0), w.Hkv, w.budget, w.n_sink, w.recent)
    np.testing.assert_array_equal(a[0], b[0])
    np.testing.assert_array_equal(a[2], b[2])


# ------------------------------------------------------------------ mode 1

def _mode1(**kw):
    base = dict(mode=1, gamma=0.5, beta=1.0, p=2.0, eta=0.5, lambda_clip=0.02, alpha_soft=0.5,
                alpha_cross=0.35, temp=1.0, nms_radius=2)
    base.update(kw)
    return SelectorParams(**base)


def _rand_problem(seed, B=1, Hq=4, Hkv=2, L=120):
    rng = syn.rng_for(seed, 1)
    lg = rng.standard_normal((B, Hq, L)) * 2.5
    kn = np.abs(rng.standard_normal((B, Hkv, L))) * 3.0 + 8.0
    return lg, kn


def test_prior_special_cases(oracle):
    L, n_sink, R = 60, 4, 6
    lg, kn = _rand_problem(50, L=L)
    J = slice(n_sink, L - R)
    nJ = L - R - n_sink
    # no factor active -> uniform prior
    _, _, _, d0 = run(oracle, lg, L, 2, 8, n_sink, R, sp=_mode1(gamma=0, beta=0, eta=0), knorm=kn, debug=True)
    np.testing.assert_allclose(d0["r"][0, 0, J], 1.0 / nJ, rtol=1e-12)
    # key-norm factor only, gamma = 1: r ~ 1 / (||k|| + eps)
    _, _, _, d1 = run(oracle, lg, L, 2, 8, n_sink, R, sp=_mode1(gamma=1, beta=0, eta=0), knorm=kn, debug=True)
    inv = 1.0 / (kn[0, 1, J] + EPS)
    np.testing.assert_allclose(d1["r"][0, 1, J], inv / inv.sum(), rtol=1e-12)
    # decay only (p = 1): consecutive ratio r(j+1)/r(j) = exp(-beta / (jmax - jmin + eps))
    _, _, _, d2 = run(oracle, lg, L, 2, 8, n_sink, R, sp=_mode1(gamma=0, beta=3.0, p=1.0, eta=0), knorm=kn,
                      debug=True)
    r = d2["r"][0, 0, J]
    np.testing.assert_allclose(r[1:] / r[:-1], math.exp(-3.0 / (nJ - 1 + EPS)), rtol=1e-10)
    # tail brake only (eta = 1): r(j) ~ 1 - u + eps, linear, hitting ~eps-level mass at the last position
    _, _, _, d3 = run(oracle, lg, L, 2, 8, n_sink, R, sp=_mode1(gamma=0, beta=0, eta=1.0), knorm=kn, debug=True)
    r = d3["r"][0, 0, J]
    np.testing.assert_allclose(r[0] - r[1], r[1] - r[2], rtol=1e-9)
    expect = (EPS / (nJ - 1 + EPS) + EPS) / (1.0 + EPS)       # (1 - u_max + eps) / (1 - 0 + eps)
    np.testing.assert_allclose(r[-1] / r[0], expect, rtol=1e-4)
    for dd in (d0, d1, d2, d3):
        assert abs(dd["r"][0, 0].sum() - 1) < 1e-12 and abs(dd["s"][0, 0].sum() - 1) < 1e-12


def test_fusion_closed_form_minimises_kl_objective(oracle):
    """s = (1 - lam) f + lam r minimises (1-lam) KL(f||s) + lam KL(r||s) on the simplex (Eq. selector_obj)."""
    from scipy.optimize import minimize

    L, n_sink, R = 9, 2, 3     # |J| = 4
    lg, kn = _rand_problem(51, Hq=2, Hkv=1, L=L)
    _, _, _, dbg = run(oracle, lg, L, 1, 2, n_sink, R, sp=_mode1(lambda_clip=0.4), knorm=kn, debug=True)
    J = slice(n_sink, L - R)
    f, r, s, lam = dbg["f"][0, 0, J], dbg["r"][0, 0, J], dbg["s"][0, 0, J], dbg["lambda"][0, 0]
    assert 0 < lam <= 0.4

    def obj(theta):
        sv = softmax(theta)
        return (1 - lam) * np.sum(f * np.log(f / sv)) + lam * np.sum(r * np.log(r / sv))

    best = min((minimize(obj, x0, method="Nelder-Mead", options=dict(xatol=1e-10, fatol=1e-14, maxiter=20000))
                for x0 in (np.zeros(4), np.log(f))), key=lambda o: o.fun)
    np.testing.assert_allclose(softmax(best.x), s, atol=2e-6)
    np.testing.assert_allclose(s, (1 - lam) * f + lam * r, rtol=1e-13)
    # arithmetic mixture dominates the geometric one pointwise (Eq. selector_amgm)
    assert (s >= f ** (1 - lam) * r ** lam - 1e-15).all()


@pytest.mark.parametrize("clip", [0.0, 0.02, 0.3, 1.0])
def test_lambda_star_is_clipped_minimiser_of_sharpness(oracle, clip):
    L, n_sink, R = 80, 4, 8
    lg, kn = _rand_problem(52, L=L)
    _, _, _, dbg = run(oracle, lg, L, 2, 8, n_sink, R, sp=_mode1(lambda_clip=clip), knorm=kn, debug=True)
    J = slice(n_sink, L - R)
    for h in range(2):
        f, r, lam = dbg["f"][0, h, J], dbg["r"][0, h, J], dbg["lambda"][0, h]
        grid = np.linspace(0.0, clip, 20001)
        sharp = [np.sum(((1 - t) * f + t * r) ** 2) for t in grid]
        assert abs(grid[int(np.argmin(sharp))] - lam) <= clip / 20000 + 1e-12
        if clip == 0.0:
            np.testing.assert_array_equal(dbg["s"][0, h, J], f)


def test_soft_nms_hand_case_and_local_maxima(oracle):
    """Single head (no cross-head effect), prior off (lambda_clip = 0): z_base = log(f + eps)."""
    L, n_sink, R = 12, 1, 1
    lg = np.zeros((1, 1, L))
    lg[0, 0, 1:11] = np.log([8.0, 4, 1, 1, 2, 16, 1, 1, 1, 4])
    kn = np.ones((1, 1, L))
    sp = _mode1(lambda_clip=0.0, alpha_soft=0.5, alpha_cross=0.0, nms_radius=1)
    _, _, z, dbg = run(oracle, lg, L, 1, 3, n_sink, R, sp=sp, knorm=kn, debug=True)
    zb = dbg["zbase"][0, 0, 1:11]
    f = np.array([8.0, 4, 1, 1, 2, 16, 1, 1, 1, 4]) / 39.0
    np.testing.assert_allclose(zb, np.log(f + EPS), rtol=1e-13)
    m = np.array([zb[0], zb[0], zb[1], zb[4], zb[5], zb[5], zb[5], zb[6], zb[9], zb[9]])
    np.testing.assert_allclose(dbg["znms"][0, 0, 1:11], zb - 0.5 * (m - zb), rtol=1e-13)
    # local maximisers keep their score
    for i in (0, 5, 9):
        assert dbg["znms"][0, 0, 1 + i] == zb[i]
    # a wider neighbourhood reaches the global maximum from further away
    sp3 = _mode1(lambda_clip=0.0, alpha_soft=1.0, alpha_cross=0.0, nms_radius=3)
    _, _, _, dbg3 = run(oracle, lg, L, 1, 3, n_sink, R, sp=sp3, knorm=kn, debug=True)
    np.testing.assert_allclose(dbg3["znms"][0, 0, 1 + 2], zb[2] - (zb[5] - zb[2]), rtol=1e-13)


def test_cross_head_properties(oracle):
    L, n_sink, R = 90, 4, 8
    lg, kn = _rand_problem(53, Hq=8, Hkv=4, L=L)
    J = slice(n_sink, L - R)
    # refinements off -> ranking of z_adj equals ranking of f
    sp_off = _mode1(lambda_clip=0.0, alpha_soft=0.0, alpha_cross=0.0)
    sel_off, _, z_off, d_off = run(oracle, lg, L, 4, 11, n_sink, R, sp=sp_off, knorm=kn, debug=True)
    sel0, _, z0 = run(oracle, lg, L, 4, 11, n_sink, R)
    np.testing.assert_array_equal(sel_off, sel0)
    np.testing.assert_allclose(z_off[:, :, J], z0[:, :, J], rtol=1e-13)
    # the adjustment is never positive and equals alpha_cross * log softmax_h(z_nms / T)
    sp = _mode1(alpha_cross=0.35, temp=0.7)
    _, _, z, dbg = run(oracle, lg, L, 4, 11, n_sink, R, sp=sp, knorm=kn, debug=True)
    zn = dbg["znms"][0][:, J]
    adj = z[0][:, J] - zn
    assert (adj <= 1e-15).all()
    resp = np.exp(zn / 0.7 - (zn / 0.7).max(axis=0)) / np.exp(zn / 0.7 - (zn / 0.7).max(axis=0)).sum(axis=0)
    np.testing.assert_allclose(adj, 0.35 * np.log(np.maximum(resp, EPS)), rtol=1e-9, atol=1e-12)
    # a dominant head is almost untouched
    lg2 = lg.copy()
    lg2[0, 0:2, 40] += 30.0
    _, _, z2, dbg2 = run(oracle, lg2, L, 4, 11, n_sink, R, sp=_mode1(alpha_soft=0.0), knorm=kn, debug=True)
    assert abs(z2[0, 0, 40] - dbg2["znms"][0, 0, 40]) < 0.02          # responsibility ~ 1
    for h in (1, 2, 3):                                                # the others pay ~ alpha_cross * gap
        assert z2[0, h, 40] - dbg2["znms"][0, h, 40] < -1.0
    # one KV head: responsibility is 1, nothing changes
    lg1, kn1 = _rand_problem(54, Hq=2, Hkv=1, L=L)
    _, _, z1, dbg1 = run(oracle, lg1, L, 1, 11, n_sink, R, sp=_mode1(), knorm=kn1, debug=True)
    np.testing.assert_allclose(z1[0, 0, J], dbg1["znms"][0, 0, J], rtol=0, atol=1e-15)
    # identical heads: uniform shift alpha_cross * log(1/H), ranking unchanged
    lgi = np.tile(lg[:, :2, :], (1, 4, 1))
    kni = np.tile(kn[:, :1, :], (1, 4, 1))
    seli, _, zi, dbgi = run(oracle, lgi, L, 4, 11, n_sink, R, sp=_mode1(), knorm=kni, debug=True)
    np.testing.assert_allclose(zi[0][:, J] - dbgi["znms"][0][:, J], 0.35 * math.log(0.25), rtol=1e-12)
    for h in range(1, 4):
        np.testing.assert_array_equal(seli[0, h], seli[0, 0])


@pytest.mark.parametrize("p", [2.0, 3.0, 1.5])
def test_position_decay_exponent(oracle, p):
    """Decay factor alone (gamma = eta = 0): r(j) ~ exp(-beta u(j)^p) with u = (j - j_min) / (j_max - j_min + eps)
    (Eqs. selector_u, selector_prior_pos), so for ANY two positions
    log r(j) - log r(j') = -beta (u(j)^p - u(j')^p).  Checked on pairs far apart, where u^p and u differ most."""
    L, n_sink, R, beta = 75, 4, 7, 2.5
    lg, kn = _rand_problem(55, L=L)
    nJ = L - R - n_sink
    _, _, _, dbg = run(oracle, lg, L, 2, 8, n_sink, R, sp=_mode1(gamma=0, beta=beta, p=p, eta=0), knorm=kn, debug=True)
    r = dbg["r"][0, 1, n_sink:L - R]
    u = np.arange(nJ) / (nJ - 1 + EPS)
    for a, b in [(0, nJ - 1), (3, 40), (17, 60), (nJ // 2, nJ - 2), (1, 2)]:
        np.testing.assert_allclose(math.log(r[a]) - math.log(r[b]), -beta * (u[a] ** p - u[b] ** p), rtol=1e-11, atol=1e-13)
    # the first position has u = 0 whatever p is; the last has u^p = 1 up to eps: r(last) / r(first) = exp(-beta)
    np.testing.assert_allclose(r[-1] / r[0], math.exp(-beta * (1.0 / (1.0 + EPS / (nJ - 1))) ** p), rtol=1e-12)
    assert abs(r.sum() - 1.0) < 1e-12


def test_position_prior_both_factors_closed_form(oracle):
    """Both position factors and the key-norm factor at once against the equations written out with numpy
    (Eqs. selector_prior_kn, selector_prior_pos, selector_r)."""
    L, n_sink, R = 64, 3, 5
    lg, kn = _rand_problem(56, L=L)
    nJ = L - R - n_sink
    g, beta, p, eta = 0.7, 1.3, 3.0, 0.4
    _, _, _, dbg = run(oracle, lg, L, 2, 8, n_sink, R, sp=_mode1(gamma=g, beta=beta, p=p, eta=eta), knorm=kn, debug=True)
    u = np.arange(nJ) / (nJ - 1 + EPS)
    for h in range(2):
        w = (kn[0, h, n_sink:L - R] + EPS) ** (-g) * np.exp(-beta * u ** p) * (1.0 - u + EPS) ** eta
        np.testing.assert_allclose(dbg["r"][0, h, n_sink:L - R], w / w.sum(), rtol=1e-12)


def test_cross_head_responsibility_floor(oracle):
    """Eq. head_mutex: z_adj = z_nms + alpha_cross log max(r_h, eps).  Two KV heads, G = 1, prior and Soft-NMS off,
    so z_nms = log(p_h + eps) with p_h the head's softmax over J.  At one position head 0 carries almost all of
    its mass and head 1 almost none, so that (z_0 - z_1) / T exceeds ln(1 / eps): head 1's responsibility
    e^{-(z_0 - z_1)/T} / (1 + ...) is below eps and its adjustment must equal alpha_cross * ln(eps) exactly.
    At a second position the gap stays just inside ln(1 / eps): no floor, adjustment = alpha_cross * log r_h."""
    L, n_sink, R, T, ac = 40, 2, 3, 0.5, 0.35
    nJ = L - R - n_sink
    J = slice(n_sink, L - R)
    lg = np.zeros((1, 2, L))
    lg[0, 0, 10] = 18.0     # head 0: p(10) ~ 1
    lg[0, 1, 10] = -18.0    # head 1: p(10) ~ e^-18 / nJ, far below eps -> z_1 = log(eps-ish)
    lg[0, 0, 20] = 12.0     # p_0(20) = e^-6: a mild gap to head 1's 1 / |J| there
    kn = np.ones((1, 2, L))
    sp = _mode1(lambda_clip=0.0, alpha_soft=0.0, alpha_cross=ac, temp=T, nms_radius=0)
    _, _, z, dbg = run(oracle, lg, L, 2, 4, n_sink, R, sp=sp, knorm=kn, debug=True)
    p0, p1 = softmax(lg[0, 0, J]), softmax(lg[0, 1, J])
    z0, z1 = np.log(p0 + EPS), np.log(p1 + EPS)
    np.testing.assert_allclose(dbg["znms"][0, 0, J], z0, rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(dbg["znms"][0, 1, J], z1, rtol=1e-13, atol=1e-14)
    i = 10 - n_sink
    gap = (z0[i] - z1[i]) / T
    assert gap > math.log(1.0 / EPS) + 5.0                       # the floor is what decides here
    np.testing.assert_allclose(z[0, 1, 10] - z1[i], ac * math.log(EPS), rtol=1e-13)
    np.testing.assert_allclose(z[0, 0, 10] - z0[i], ac * math.log(1.0 / (1.0 + math.exp(-gap))), rtol=1e-9, atol=1e-14)
    # without the floor the adjustment would have been alpha_cross * (-gap - log(1 + e^-gap)): far lower
    assert ac * (-gap) < ac * math.log(EPS) - 1.0
    k = 20 - n_sink                                              # a position where no head drops below the floor
    gap2 = (z1[k] - z0[k]) / T                                   # here head 1 leads
    assert 0 < gap2 < math.log(1.0 / EPS) - 5.0
    np.testing.assert_allclose(z[0, 0, 20] - z0[k], ac * (-gap2 - math.log1p(math.exp(-gap2))), rtol=1e-12)
    np.testing.assert_allclose(z[0, 1, 20] - z1[k], -ac * math.log1p(math.exp(-gap2)), rtol=1e-9)
    # Either side of the floor, planted exactly.  Head 0 uniform over J (z_0 = log(1 / |J| + eps) everywhere); head 1
    # uniform except one low logit x at position 12, chosen so that its responsibility there,
    # 1 / (1 + e^{(z_0 - z_1) / T}), is 2 eps (untouched by the floor) or eps / 2 (lifted to eps).
    for resp, want in [(2.0 * EPS, 2.0 * EPS), (0.5 * EPS, EPS)]:
        g2 = math.log((1.0 - resp) / resp) * T                   # the z_0 - z_1 that gives head 1 this responsibility
        target = (1.0 / nJ + EPS) * math.exp(-g2) - EPS          # p_1(12) with log(p_1 + eps) = z_0 - g2
        assert target > 0
        x = math.log(target * (nJ - 1) / (1.0 - target))         # p_1(12) = e^x / (|J| - 1 + e^x)
        lg2 = np.zeros((1, 2, L))
        lg2[0, 1, 12] = x
        _, _, zz, dd = run(oracle, lg2, L, 2, 4, n_sink, R, sp=sp, knorm=kn, debug=True)
        adj = zz[0, 1, 12] - dd["znms"][0, 1, 12]
        np.testing.assert_allclose(adj, ac * math.log(want), rtol=1e-7)


def test_degenerate_prior_and_fusion_cases(oracle):
    """Where the epsilons and guards of Sec. 3.2 decide: |J| = 1 (u = 0 / eps, Eq. selector_u), f = r (the
    denominator of Eq. selector_lambda_closed vanishes: lambda* = 0) and an unclipped lambda* below 0."""
    kn1 = np.full((1, 1, 20), 3.0)
    # |J| = 1: the only position has u = 0, r = s = f = 1, z = log(1 + eps); nothing is NaN
    lg = syn.rng_for(57, 1).standard_normal((1, 2, 20))
    sel, nsel, z, dbg = run(oracle, lg[:, :, :9], 9, 1, 3, 4, 4, sp=_mode1(), knorm=kn1[:, :, :9], debug=True)
    assert nsel[0, 0] == 1 and sel[0, 0, 0] == 4
    assert dbg["r"][0, 0, 4] == 1.0 and dbg["f"][0, 0, 4] == 1.0 and dbg["s"][0, 0, 4] == 1.0
    np.testing.assert_allclose(z[0, 0, 4], math.log(1.0 + EPS), rtol=1e-12)
    # f = r = uniform: denominator 0 -> lambda* = 0, s = f, everything finite
    lgu = np.zeros((1, 2, 20))
    _, _, zu, du = run(oracle, lgu, 20, 1, 3, 4, 4, sp=_mode1(gamma=0, beta=0, eta=0, lambda_clip=1.0), knorm=kn1, debug=True)
    assert du["lambda"][0, 0] == 0.0 and np.isfinite(zu[0, 0, 4:16]).all()
    np.testing.assert_allclose(du["s"][0, 0, 4:16], 1.0 / 12, rtol=1e-14)
    # f mildly peaked, r sharply peaked at the same position: |f|^2 < f.r, so the unclipped minimiser is negative
    # and lambda* = 0 (Eq. selector_lambda_closed clips to [0, lambda_clip])
    lgp = np.zeros((1, 2, 20))
    lgp[0, :, 8] = 0.3
    knp = np.full((1, 1, 20), 50.0)
    knp[0, 0, 8] = 0.5
    _, _, _, dp = run(oracle, lgp, 20, 1, 3, 4, 4, sp=_mode1(gamma=2.0, beta=0, eta=0, lambda_clip=1.0), knorm=knp, debug=True)
    f, r = dp["f"][0, 0, 4:16], dp["r"][0, 0, 4:16]
    assert (f * f).sum() < (f * r).sum()
    assert dp["lambda"][0, 0] == 0.0
    np.testing.assert_array_equal(dp["s"][0, 0, 4:16], f)


def test_mode1_from_qk_uses_key_norms(oracle):
    """sfio_selector computes ||k||_2 from K: scaling one key row changes its prior mass as (norm)^-gamma."""
    w = syn.make_tiny(L0=200, steps=1, budget=8, recent=16, n_support=2)
    q = w.q(0)
    sp = _mode1(gamma=1.0, beta=0.0, eta=0.0, lambda_clip=1.0, alpha_soft=0.0, alpha_cross=0.0)
    kn = np.sqrt((syn.bf16_bits_to_f32(w.K).astype(np.float64) ** 2).sum(-1))[:, :, :200]
    lg = oracle.logits(q, w.K, w.ctx_len(0))
    a = oracle.selector(q, w.K, w.ctx_len(0), w.budget, w.n_sink, w.recent, sp=sp)
    b = oracle.selector_from_logits(lg, w.ctx_len(0), w.Hkv, w.budget, w.n_sink, w.recent, sp=sp, knorm=kn)
    np.testing.assert_array_equal(a[0], b[0])
    np.testing.assert_allclose(a[2], b[2], rtol=1e-12)
