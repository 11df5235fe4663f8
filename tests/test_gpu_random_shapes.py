"""GPU parity on seeded random shapes: every entry point of the hot path against the fp64 oracle on shapes
nobody picked by hand (heads, group sizes, ragged batches, contexts from one row to 14K, sinks longer than
a context or a tile, budgets above |J|, flat and paged caches, every launch knob).  The same bars as the
hand-written cases: outputs within 2e-3 row-relative, index sets identical outside the 1e-5 band."""
import dataclasses

import numpy as np
import pytest

import sfi_synth as syn
from helpers import Runner, check_out, check_selection, i32_dev, to_dev
from oracle.sfi_oracle import SelectorParams

pytestmark = pytest.mark.gpu


def _workload(rng, seed, B, Hkv, G, L0, recent, n_sink, budget):
    w = syn.make_tiny(L0=max(L0, recent + 16), steps=3, budget=budget, recent=recent, n_support=4, B=B, Hq=G * Hkv,
                      Hkv=Hkv, seed=seed)
    w.n_sink = n_sink
    w.L0 = np.array([max(1, L0 - int(rng.integers(0, max(1, L0 // 2)))) if b else L0 for b in range(B)], np.int32)
    return w


@pytest.mark.parametrize("seed", [11, 12, 13, 14])
def test_slow_fast_and_compact_steps_on_random_shapes(oracle, seed):
    rng = np.random.default_rng(seed)
    for it in range(12):
        Hkv, G, B = int(rng.choice([1, 2, 4, 8])), int(rng.choice([1, 2, 3, 4, 5, 8, 16])), int(rng.choice([1, 2, 3, 5]))
        L0 = int(rng.choice([rng.integers(1, 200), rng.integers(200, 3000), rng.integers(3000, 14000)]))
        recent, n_sink = int(rng.choice([1, 16, 64, 128, 333, 700])), int(rng.choice([0, 1, 4, 4, 4, 33, 70]))
        budget = int(rng.choice([1, 7, 64, 256, 777, 1500]))
        page, layout = int(rng.choice([0, 0, 16, 64, 256])), str(rng.choice(["thd", "htd"]))
        tpw, dwg, merge = int(rng.choice([0, 0, 0, 1, 2, 5, 33])), int(rng.choice([0, 0, 0, 1, 7, 100, 2000])), int(rng.choice([1, 1, 2]))
        print(f"[gpu-random] seed {seed} case {it}: B={B} Hkv={Hkv} G={G} L0={L0} recent={recent} n_sink={n_sink} "
              f"budget={budget} page={page}/{layout} tpw={tpw} dense_wgs={dwg} merge={merge}", flush=True)
        w = _workload(rng, seed * 1000 + it, B, Hkv, G, L0, recent, n_sink, budget)
        r = Runner(w, page_size=page, page_layout=layout)
        try:
            r.sfi.sfi_set_tuning(r.ctx.handle, dwg if dwg else -1, tpw if tpw else -1, merge)
            q0, c0 = w.q(0), w.ctx_len(0)
            out, sel, nsel = r.slow(q0, c0, budget)
            check_out(out, oracle.dense(q0, w.K, w.V, c0))
            sel_ref, nsel_ref, z = oracle.selector(q0, w.K, c0, budget, w.n_sink, w.recent)
            check_selection(sel, nsel, sel_ref, nsel_ref, z, c0, w.n_sink, w.recent, budget)
            check_out(r.dense(q0, c0), oracle.dense(q0, w.K, w.V, c0))
            for t in (1, 2):
                q, ct, rt = w.q(t), w.ctx_len(t), w.recent_start(t)
                check_out(r.fast(q, sel, nsel, rt, ct), oracle.sparse(q, w.K, w.V, sel, nsel, rt, ct, w.n_sink))
            r.reorg(sel, nsel, c0)
            q, ct, rt = w.q(1), w.ctx_len(1), w.recent_start(1)
            if ((c0 >= w.n_sink) | (ct <= w.n_sink)).all():  # the compact path's precondition on a sink still filling up
                check_out(r.fast_compact(q, nsel, sel.shape[2], rt, ct),
                          oracle.sparse(q, w.K, w.V, sel, nsel, rt, ct, w.n_sink))
        finally:
            r.close()


@pytest.mark.parametrize("seed", [21, 22])
def test_mixed_step_and_full_selector_on_random_shapes(oracle, seed):
    import torch
    rng = np.random.default_rng(seed)
    for it in range(10):
        Hkv, G, B = int(rng.choice([1, 2, 4, 8])), int(rng.choice([1, 2, 3, 4, 8, 16])), int(rng.choice([1, 2, 3, 6]))
        L0 = int(rng.choice([rng.integers(1, 300), rng.integers(300, 3000), rng.integers(3000, 11000)]))
        recent, n_sink, budget = int(rng.choice([1, 16, 64, 200])), int(rng.choice([0, 4, 4, 33])), int(rng.choice([1, 7, 64, 300, 900]))
        mode, alpha = int(rng.choice([0, 1])), float(rng.choice([1.0, 1.0, 0.5, 0.25]))
        page, merge = int(rng.choice([0, 0, 64])), int(rng.choice([1, 1, 2]))
        kw = {}
        if mode == 1:
            kw = dict(nms_radius=int(rng.choice([0, 2, 7, 64])), alpha_soft=float(rng.choice([0.0, 0.5, 1.0])),
                      temp=float(rng.choice([0.5, 1.0, 4.0])), alpha_cross=float(rng.choice([0.1, 0.35, 1.0])),
                      lambda_clip=float(rng.choice([0.02, 0.5, 1.0])), gamma=float(rng.choice([0.5, 1.0])))
        print(f"[gpu-random] seed {seed} case {it}: B={B} Hkv={Hkv} G={G} L0={L0} recent={recent} n_sink={n_sink} "
              f"budget={budget} mode={mode} alpha={alpha} page={page} merge={merge} {kw}", flush=True)
        w = _workload(rng, seed * 1000 + it, B, Hkv, G, L0, recent, n_sink, budget)
        sp = dataclasses.replace(SelectorParams(mode=mode), alpha=alpha, **kw)
        d = None
        if mode == 1:
            d = {k: getattr(sp, k) for k in ("gamma", "beta", "p", "eta", "lambda_clip", "alpha_soft", "alpha_cross", "temp",
                                              "eps", "nms_radius")}
        r = Runner(w, selector=d, alpha=alpha, page_size=page)
        try:
            sfi, h = r.sfi, r.ctx.handle
            sfi.sfi_set_tuning(h, 0, 0, merge)
            ctx_d, rs_d = i32_dev(w.ctx_len(0)), i32_dev(w.recent_start(0))
            sel_d = torch.full((B, Hkv, max(budget, 1)), -7, dtype=torch.int32, device="cuda")
            nsel_d = torch.full((B, Hkv), -7, dtype=torch.int32, device="cuda")
            q0, c0 = w.q(0), w.ctx_len(0)
            sfi.sfi_mixed_step(h, to_dev(q0), r.K, r.V, torch.ones(B, dtype=torch.uint8, device="cuda"), ctx_d, rs_d, 0,
                               budget, r.out, sel_d, nsel_d)
            torch.cuda.synchronize()
            check_out(r.out.cpu().numpy(), oracle.dense(q0, w.K, w.V, c0))
            sel_ref, nsel_ref, z = oracle.selector(q0, w.K, c0, budget, n_sink, recent, sp=sp)
            sel0, nsel0 = sel_d.cpu().numpy(), nsel_d.cpu().numpy()
            check_selection(sel0, nsel0, sel_ref, nsel_ref, z, c0, n_sink, recent, budget)
            _, sel_s, nsel_s = r.slow(q0, c0, budget)
            assert np.array_equal(sel_s, sel0) and np.array_equal(nsel_s, nsel0), "slow step and mixed step disagree"
            sfi.sfi_advance(h, ctx_d, rs_d)
            slow1 = (rng.random(B) < 0.4).astype(np.uint8)
            q1, c1, r1 = w.q(1), w.ctx_len(1), w.recent_start(1)
            sfi.sfi_mixed_step(h, to_dev(q1), r.K, r.V, torch.from_numpy(slow1).cuda(), ctx_d, rs_d, 0, budget, r.out,
                               sel_d, nsel_d)
            torch.cuda.synchronize()
            got = r.out.cpu().numpy()
            ref_dense = oracle.dense(q1, w.K, w.V, c1)
            ref_sparse = oracle.sparse(q1, w.K, w.V, sel0, nsel0, r1, c1, n_sink)
            sel1, nsel1 = sel_d.cpu().numpy(), nsel_d.cpu().numpy()
            sel_ref1, nsel_ref1, z1 = oracle.selector(q1, w.K, c1, budget, n_sink, recent, sp=sp)
            for b in range(B):
                if slow1[b]:  # (the cross-head term of the full Selector couples the heads of one sequence only)
                    check_out(got[b], ref_dense[b])
                    check_selection(sel1[b:b + 1], nsel1[b:b + 1], sel_ref1[b:b + 1], nsel_ref1[b:b + 1], z1[b:b + 1],
                                    c1[b:b + 1], n_sink, recent, budget)
                else:
                    check_out(got[b], ref_sparse[b])
                    assert (sel1[b] == sel0[b]).all() and (nsel1[b] == nsel0[b]).all()
        finally:
            r.close()
