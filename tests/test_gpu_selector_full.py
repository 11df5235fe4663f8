"""GPU parity of the full Selector (mode 1: prior, lambda*, fusion, Soft-NMS, cross-head exclusivity)
against the fp64 oracle's Algorithm 2, on the selected index sets.

The GPU ranks in fp32, the oracle in fp64, so the two may differ on positions whose final ranking
scores z_adj lie within FULL_BAND of the cut; outside that band the sets must be identical.  The band
is the one of the evidence-only mode.
"""
import dataclasses

import numpy as np
import pytest

import sfi_synth as syn
from helpers import Runner, check_out, check_selection
from oracle.sfi_oracle import SelectorParams

pytestmark = pytest.mark.gpu

FULL_BAND = 1e-5


def _step(msg):
    print(f"[gpu-selector-full] {msg}", flush=True)


def _params(**kw):
    sp = dataclasses.replace(SelectorParams(mode=1), **kw)
    d = {k: getattr(sp, k) for k in ("gamma", "beta", "p", "eta", "lambda_clip", "alpha_soft", "alpha_cross", "temp",
                                      "eps", "nms_radius")}
    return sp, d


def _run(oracle, w, sp, d, ctx=None, budget=None, band=FULL_BAND):
    r = Runner(w, selector=d, alpha=sp.alpha)
    try:
        q = w.q(0)
        ctx = w.ctx_len(0) if ctx is None else np.asarray(ctx, np.int32)
        budget = w.budget if budget is None else budget
        out, sel, nsel = r.slow(q, ctx, budget)
        check_out(out, oracle.dense(q, w.K, w.V, ctx))
        sel_ref, nsel_ref, z = oracle.selector(q, w.K, ctx, budget, w.n_sink, w.recent, sp=sp)
        n_exact = check_selection(sel, nsel, sel_ref, nsel_ref, z, ctx, w.n_sink, w.recent, budget, band=band)
        return n_exact, sel, sel_ref
    finally:
        r.close()


@pytest.mark.parametrize("kw", [
    {},                                                      # the defaults
    {"lambda_clip": 0.5, "gamma": 1.0},                      # strong prior
    {"lambda_clip": 1.0, "beta": 3.0, "p": 1.0, "eta": 2.0},  # lambda* unclipped; other prior shape
    {"nms_radius": 0},                                       # Soft-NMS window of one: no change
    {"nms_radius": 7, "alpha_soft": 1.0},
    {"nms_radius": 64, "alpha_soft": 0.25},                  # widest window the library takes
    {"temp": 0.5, "alpha_cross": 1.0},
    {"temp": 4.0, "alpha_cross": 0.1, "alpha_soft": 0.0},
])
def test_full_selector_matches_oracle(oracle, kw):
    sp, d = _params(**kw)
    w = syn.make_tiny(L0=4700, steps=1, budget=160, recent=48, n_support=24, B=2, Hq=8, Hkv=2)
    w.L0 = np.array([4700, 2300], np.int32)
    _step(f"mode 1 {kw}")
    n_exact, _, _ = _run(oracle, w, sp, d)
    assert n_exact >= 2  # most cuts are wider than the band


@pytest.mark.parametrize("Hq,Hkv", [(4, 1), (8, 8), (16, 2), (20, 4), (16, 1)])
def test_full_selector_head_layouts(oracle, Hq, Hkv):
    """One KV head (the head softmax is the constant 1), eight KV heads, G = 1, 5, 8, 16."""
    sp, d = _params()
    w = syn.make_tiny(L0=2500, steps=1, budget=64, recent=32, n_support=12, B=1, Hq=Hq, Hkv=Hkv)
    _step(f"mode 1 Hq={Hq} Hkv={Hkv}")
    _run(oracle, w, sp, d)


def test_full_selector_without_refinements_is_mode0(oracle):
    """lambda_clip = 0 and both refinement strengths 0: Alg. 2 reduces to Top-K of f (same sets as mode 0)."""
    sp, d = _params(lambda_clip=0.0, alpha_soft=0.0, alpha_cross=0.0)
    w = syn.make_tiny(L0=3000, steps=1, budget=100, recent=64, n_support=16, B=1, Hq=8, Hkv=2)
    _step("mode 1 reduced to mode 0")
    _, sel1, _ = _run(oracle, w, sp, d)
    r0 = Runner(w)
    try:
        _, sel0, _ = r0.slow(w.q(0), w.ctx_len(0), w.budget)
    finally:
        r0.close()
    assert (sel0 == sel1).all()


@pytest.mark.parametrize("L,budget", [(4 + 32 + 1, 8), (4 + 32 + 5, 8), (4 + 32 + 5, 3), (30, 8), (2048 + 36, 50),
                                      (2048 + 37, 50), (4096 + 36 + 2, 4096)])
def test_full_selector_edges(oracle, L, budget):
    """|J| = 1, |J| < budget, J empty, |J| a whole segment, one past it, budget >= |J| over two segments."""
    sp, d = _params()
    w = syn.make_tiny(L0=4200, steps=1, budget=4096, recent=32, n_support=8, B=1, Hq=8, Hkv=2)
    _step(f"mode 1 edge L={L} budget={budget}")
    _run(oracle, w, sp, d, ctx=[L], budget=budget)


def test_full_selector_at_llama8b_size(oracle):
    """Config 2's slow step (B4, 32/8 heads, ctx 32768, K = 2048, recent 128) with the full Selector."""
    sp, d = _params()
    w = syn.make_llama8b(steps=2)
    _step("mode 1 at config-2 size")
    n_exact, _, _ = _run(oracle, w, sp, d)
    _step(f"  index sets identical to the oracle's: {n_exact}/{w.B * w.Hkv}")
    assert n_exact >= (w.B * w.Hkv) // 2


def test_full_selector_at_long_context(oracle):
    """Config 3's slow step (B1, 32/8 heads, ctx 131072, K = 4096, recent 256) with the full Selector: the evidence
    of a typical position, ~1 / |J|, sits three decades above eps here, the prior's position terms span 64 segments."""
    sp, d = _params()
    w = syn.make_long(steps=2)
    _step("mode 1 at config-3 size")
    n_exact, _, _ = _run(oracle, w, sp, d)
    _step(f"  index sets identical to the oracle's: {n_exact}/{w.B * w.Hkv}")
    assert n_exact >= (w.B * w.Hkv) // 2


def test_full_selector_at_serving_shape(oracle):
    """Config 5's head layout (64/8 heads, G = 8, eight KV heads under the cross-head term), four ragged sequences."""
    sp, d = _params()
    w = syn.make_serving(steps=2, B=4)
    _step(f"mode 1 at config-5 shape, ctx {w.L0.tolist()}")
    n_exact, _, _ = _run(oracle, w, sp, d)
    _step(f"  index sets identical to the oracle's: {n_exact}/{w.B * w.Hkv}")
    assert n_exact >= (w.B * w.Hkv) // 2


@pytest.mark.parametrize("alpha", [0.5, 0.25, 0.9])
@pytest.mark.parametrize("mode", [0, 1])
def test_power_mean_evidence(oracle, mode, alpha):
    """Eq. selector_mu with alpha < 1 (the G heads of a KV head are the window), in both Selector modes."""
    sp, d = _params(alpha=alpha)
    if mode == 0:
        sp, d = dataclasses.replace(sp, mode=0), None
    w = syn.make_tiny(L0=3900, steps=1, budget=128, recent=48, n_support=24, B=2, Hq=8, Hkv=2)
    _step(f"power mean alpha={alpha} mode={mode}")
    _run(oracle, w, sp, d)


def test_power_mean_single_head_is_alpha_free(oracle):
    """G = 1: f = p_1 whatever alpha is (Eq. selector_f), so the selection equals the alpha = 1 one."""
    w = syn.make_tiny(L0=2100, steps=1, budget=64, recent=32, n_support=12, B=1, Hq=2, Hkv=2)
    _step("power mean with G = 1")
    sels = []
    for alpha in (1.0, 0.4):
        r = Runner(w, alpha=alpha)
        try:
            _, sel, _ = r.slow(w.q(0), w.ctx_len(0), w.budget)
            sels.append(sel)
        finally:
            r.close()
    sel_ref, nsel_ref, z = oracle.selector(w.q(0), w.K, w.ctx_len(0), w.budget, w.n_sink, w.recent,
                                           sp=SelectorParams(alpha=0.4))
    assert (sels[0] == sels[1]).all() and (sels[1] == sel_ref).all()


@pytest.mark.parametrize("with_out", [True, False])
@pytest.mark.parametrize("mode,alpha,W", [(0, 1.0, 5), (0, 0.5, 3), (1, 1.0, 4), (1, 0.5, 2), (0, 1.0, 1),
                                          (0, 0.5, 16), (1, 0.5, 16)])  # W = 16, alpha < 1: the paper's prefill setting
def test_windowed_evidence(oracle, mode, alpha, W, with_out):
    """Evidence accumulated over W window queries (Eq. selector_mu with a window): W calls of
    sfi_evidence_add and one sfi_evidence_select against the oracle's Selector on the W * G query vectors
    of each KV head.  Each call's `out` is that query's dense attention; without `out` (and without V) the
    call is the evidence-only pass and the selection must come out the same."""
    import torch
    import paper_2603_12038_amd as sfi
    from helpers import i32_dev, to_dev

    sp, d = _params(alpha=alpha)
    if mode == 0:
        sp, d = dataclasses.replace(sp, mode=0), None
    w = syn.make_tiny(L0=3100, steps=max(8, W), budget=96, recent=40, n_support=16, B=2, Hq=8, Hkv=2)
    w.L0 = np.array([3100, 1500], np.int32)
    G = w.Hq // w.Hkv
    r = Runner(w, selector=d, alpha=alpha)
    try:
        _step(f"windowed evidence mode={mode} alpha={alpha} W={W} with_out={with_out}")
        ctx = w.ctx_len(0)
        ctx_d = i32_dev(ctx)
        qs = [w.q(t) for t in range(W)]
        sel = torch.full((w.B, w.Hkv, w.budget), -7, dtype=torch.int32, device="cuda")
        nsel = torch.full((w.B, w.Hkv), -7, dtype=torch.int32, device="cuda")
        for t, q in enumerate(qs):
            r.out.fill_(float("nan"))
            if with_out:
                sfi.sfi_evidence_add(r.ctx.handle, to_dev(q), r.K, r.V, ctx_d, 0, r.out, t == 0)
                torch.cuda.synchronize()
                check_out(r.out.cpu().numpy(), oracle.dense(q, w.K, w.V, ctx))
            else:
                sfi.sfi_evidence_add(r.ctx.handle, to_dev(q), r.K, None, ctx_d, 0, None, t == 0)
                torch.cuda.synchronize()
                assert torch.isnan(r.out).all()  # nothing wrote an output
        sfi.sfi_evidence_select(r.ctx.handle, W, ctx_d, 0, w.budget, sel, nsel)
        torch.cuda.synchronize()
        # the oracle's window: per KV head the W * G vectors (query tau, head g)
        q_cat = np.empty((w.B, w.Hkv * W * G, w.d), np.uint16)
        for h in range(w.Hkv):
            for t in range(W):
                q_cat[:, h * W * G + t * G:h * W * G + (t + 1) * G] = qs[t][:, h * G:(h + 1) * G]
        sel_ref, nsel_ref, z = oracle.selector(q_cat, w.K, ctx, w.budget, w.n_sink, w.recent, sp=sp)
        check_selection(sel.cpu().numpy(), nsel.cpu().numpy(), sel_ref, nsel_ref, z, ctx, w.n_sink, w.recent, w.budget)
    finally:
        r.close()


@pytest.mark.parametrize("mode,alpha,W,recent", [(0, 0.5, 16, 4), (1, 0.5, 16, 4), (0, 1.0, 6, 0), (1, 1.0, 5, 2),
                                                 (0, 0.5, 16, 40), (1, 0.7, 3, 1)])
def test_windowed_evidence_under_the_causal_mask(oracle, mode, alpha, W, recent):
    """The tail of a prefill block as the observation window (Eq. window_logits with masked logits): window query
    tau sits at row L - W + tau and sees rows up to its own.  With recent < W the earlier queries miss the end of J:
    their softmax runs over the part of J they see.  sfi_evidence_add_causal per query (its `out` is its attention
    over the rows it sees) and one sfi_evidence_select, against the oracle's Selector on the W * G vectors with
    their visible lengths.  recent >= W: every query sees all of J (the unmasked case)."""
    import torch
    import paper_2603_12038_amd as sfi
    from helpers import i32_dev, to_dev

    sp, d = _params(alpha=alpha)
    if mode == 0:
        sp, d = dataclasses.replace(sp, mode=0), None
    w = syn.make_tiny(L0=3100, steps=max(8, W), budget=96, recent=recent, n_support=16, B=2, Hq=8, Hkv=2)
    w.L0 = np.array([3100, 1500], np.int32)
    G = w.Hq // w.Hkv
    # high-norm key rows in the stretch of J that only the later window queries see, so that the mask decides what is picked
    for b in range(w.B):
        lo, hi = int(w.L0[b]) - W, int(w.L0[b]) - recent
        if hi > lo:
            w.K[b, :, lo:hi] = syn.f32_to_bf16_bits(syn.bf16_bits_to_f32(w.K[b, :, lo:hi]) * np.float32(5.0))
    r = Runner(w, selector=d, alpha=alpha)
    try:
        _step(f"causal window mode={mode} alpha={alpha} W={W} recent={recent}")
        ctx = w.ctx_len(0)
        ctx_d = i32_dev(ctx)
        qs = [w.q(t) for t in range(W)]
        sel = torch.full((w.B, w.Hkv, w.budget), -7, dtype=torch.int32, device="cuda")
        nsel = torch.full((w.B, w.Hkv), -7, dtype=torch.int32, device="cuda")
        vis = np.zeros((w.B, w.Hkv * W * G), np.int32)
        q_cat = np.empty((w.B, w.Hkv * W * G, w.d), np.uint16)
        for t, q in enumerate(qs):
            q_len = (ctx - W + t + 1).astype(np.int32)
            r.out.fill_(float("nan"))
            sfi.sfi_evidence_add_causal(r.ctx.handle, to_dev(q), r.K, r.V, ctx_d, i32_dev(q_len), 0, r.out, t == 0)
            torch.cuda.synchronize()
            check_out(r.out.cpu().numpy(), oracle.dense(q, w.K, w.V, q_len))
            for h in range(w.Hkv):
                q_cat[:, h * W * G + t * G:h * W * G + (t + 1) * G] = q[:, h * G:(h + 1) * G]
                vis[:, h * W * G + t * G:h * W * G + (t + 1) * G] = q_len[:, None]
        sfi.sfi_evidence_select(r.ctx.handle, W, ctx_d, 0, w.budget, sel, nsel)
        torch.cuda.synchronize()
        sel_ref, nsel_ref, z = oracle.selector(q_cat, w.K, ctx, w.budget, w.n_sink, w.recent, sp=sp, vis=vis)
        n_exact = check_selection(sel.cpu().numpy(), nsel.cpu().numpy(), sel_ref, nsel_ref, z, ctx, w.n_sink, w.recent,
                                  w.budget)
        if recent < W - 1:  # the mask matters: without it the oracle ranks differently somewhere
            sel_nomask, _, _ = oracle.selector(q_cat, w.K, ctx, w.budget, w.n_sink, w.recent, sp=sp)
            _step(f"  sets identical {n_exact}/{w.B * w.Hkv}")
            assert not np.array_equal(sel_nomask, sel_ref), "the case is meant to be one where the mask changes the selection"
        assert r.sfi.sfi_device_status(r.ctx.handle) == 0
    finally:
        r.close()


@pytest.mark.parametrize("paged,mode,alpha", [(False, 1, 1.0), (True, 1, 1.0), (False, 1, 0.5), (False, 0, 0.5)])
def test_full_selector_in_the_ragged_step(oracle, paged, mode, alpha):
    """Mode 1 (and the power mean with alpha < 1 in either mode) inside sfi_mixed_step (Sec. 4.2's ragged step: per-sequence modes known only on the device): ragged
    sequences from empty to the whole cache; for each mix of slow and fast sequences, with the dense launch planned on
    the device and with one workgroup per cell, the slow sequences' outputs and index sets against the oracle's dense
    attention and Algorithm 2 (within the band), the fast sequences' outputs against the oracle's sparse attention on
    the sets they came in with, and their sets untouched."""
    import torch
    import paper_2603_12038_amd as sfi
    from helpers import i32_dev, to_dev

    sp, d = _params(alpha=alpha)
    if mode == 0:  # the power mean alone (Eq. selector_mu with alpha < 1), ranked without the refinements
        sp, d = dataclasses.replace(sp, mode=0), None
    w = syn.make_serving(steps=2, B=7, Hq=16, Hkv=2, len_lo=300, len_hi=6000, budget=96, recent=32)
    w.L0 = np.array([int(w.L_alloc) - 4, 0, 33, 4100, 1500, 5, 2800], np.int32)
    r = Runner(w, selector=d, alpha=sp.alpha, page_size=16 if paged else 0)
    try:
        B, h = w.B, r.ctx.handle
        ctx0, rs0, q0 = w.ctx_len(0), w.recent_start(0), w.q(0)
        ctx_d, rs_d = i32_dev(ctx0), i32_dev(rs0)
        ref_dense = oracle.dense(q0, w.K, w.V, ctx0)
        sel_ref, nsel_ref, z = oracle.selector(q0, w.K, ctx0, w.budget, w.n_sink, w.recent, sp=sp)
        ref_sparse = oracle.sparse(q0, w.K, w.V, sel_ref, nsel_ref, rs0, ctx0, w.n_sink)
        sel_d = torch.empty((B, w.Hkv, w.budget), dtype=torch.int32, device="cuda")
        nsel_d = torch.empty((B, w.Hkv), dtype=torch.int32, device="cuda")
        for plan in (1, 0):
            sfi.sfi_set_mixed_plan(h, plan)
            for mix in ([], [0], [1], [3, 5], [0, 2, 4, 6], list(range(B))):
                _step(f"mode {mode}, alpha {alpha} in the ragged step (paged={paged}, planned={plan}): slow {mix}")
                fl = np.zeros(B, np.uint8)
                fl[mix] = 1
                sel_d.copy_(torch.from_numpy(sel_ref)); nsel_d.copy_(torch.from_numpy(nsel_ref))  # what the fast ones read
                r.out.fill_(float("nan"))
                sfi.sfi_mixed_step(h, to_dev(q0), r.K, r.V, torch.from_numpy(fl).cuda(), ctx_d, rs_d, 0, w.budget, r.out, sel_d, nsel_d)
                torch.cuda.synchronize()
                out, sel, nsel = r.out.float().cpu().numpy(), sel_d.cpu().numpy(), nsel_d.cpu().numpy()
                for b in range(B):
                    check_out(out[b], ref_dense[b] if fl[b] else ref_sparse[b])
                    if not fl[b]:
                        assert (sel[b] == sel_ref[b]).all() and (nsel[b] == nsel_ref[b]).all()
                if mix:
                    check_selection(sel[mix], nsel[mix], sel_ref[mix], nsel_ref[mix], z[mix], ctx0[mix], w.n_sink, w.recent,
                                    w.budget, band=FULL_BAND)
        assert sfi.sfi_device_status(h) == 0
    finally:
        sfi.sfi_set_mixed_plan(r.ctx.handle, 1)
        r.close()
