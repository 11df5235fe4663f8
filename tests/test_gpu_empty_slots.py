"""Empty batch slots: sequences with ctx_len = 0 between live ones (a serving batch padded to its shape).  The
empty softmax gives a zero output and nothing is selected -- the oracle's convention for an empty index set --
and the neighbours are computed as if the slot were not there.  Through every entry point of the hot path, flat
and paged cache, both Selector modes."""
import dataclasses

import numpy as np
import pytest

import sfi_synth as syn
from helpers import Runner, check_out, check_selection, i32_dev, to_dev
from oracle.sfi_oracle import SelectorParams

pytestmark = pytest.mark.gpu


def _step(msg):
    print(f"[gpu-empty] {msg}", flush=True)


def _full():
    sp = dataclasses.replace(SelectorParams(mode=1))
    d = {k: getattr(sp, k) for k in ("gamma", "beta", "p", "eta", "lambda_clip", "alpha_soft", "alpha_cross", "temp",
                                      "eps", "nms_radius")}
    return sp, d


@pytest.mark.parametrize("variant", ["flat", "paged", "full-selector"])
def test_empty_slots_through_every_entry_point(oracle, variant):
    import torch
    w = syn.make_tiny(L0=1500, steps=3, budget=64, recent=48, n_support=8, B=4)
    ctx0 = np.array([1500, 0, 700, 0], np.int32)
    sp, d = _full() if variant == "full-selector" else (None, None)
    kw = dict(selector=d, alpha=sp.alpha) if sp is not None else {}
    # paged: the table of an empty slot holds no valid entry at all
    r = Runner(w, page_size=16 if variant == "paged" else 0,
               ctx_max=np.where(ctx0 > 0, ctx0 + 3, 0) if variant == "paged" else None, **kw)
    band = {}
    try:
        sfi, h = r.sfi, r.ctx.handle
        q0 = w.q(0)
        _step(f"{variant}: dense attention and slow step")
        check_out(r.dense(q0, ctx0), oracle.dense(q0, w.K, w.V, ctx0))
        out, sel, nsel = r.slow(q0, ctx0, w.budget)
        check_out(out, oracle.dense(q0, w.K, w.V, ctx0))
        assert not out[1].any() and not out[3].any()
        sel_ref, nsel_ref, z = oracle.selector(q0, w.K, ctx0, w.budget, w.n_sink, w.recent, **({"sp": sp} if sp else {}))
        check_selection(sel, nsel, sel_ref, nsel_ref, z, ctx0, w.n_sink, w.recent, w.budget, **band)
        assert (nsel[1] == 0).all() and (sel[3] == -1).all()

        live = (ctx0 > 0).astype(np.int32)
        ctx1 = ctx0 + live  # the live sequences grow, the empty slots stay empty
        rs1 = np.where(live > 0, np.maximum(w.n_sink, ctx1 - w.recent), 0).astype(np.int32)
        q1 = w.q(1)
        ref_sparse = oracle.sparse(q1, w.K, w.V, sel, nsel, rs1, ctx1, w.n_sink)
        for tpw in (1, 3):
            _step(f"{variant}: fast step, {tpw} tiles per wave")
            sfi.sfi_set_tuning(h, 0, tpw)
            got = r.fast(q1, sel, nsel, rs1, ctx1)
            check_out(got, ref_sparse)
            assert not got[1].any() and not got[3].any()
        sfi.sfi_set_tuning(h, 0, -1)
        _step(f"{variant}: a recent_start left at n_sink by sfi_advance reads as an empty window")
        check_out(r.fast(q1, sel, nsel, np.maximum(rs1, w.n_sink).astype(np.int32), ctx1), ref_sparse)

        _step(f"{variant}: reorg + compact fast step")
        Kc, Vc = r.reorg(sel, nsel, ctx1)
        assert (Kc[1] == 0x7FC1).all() and (Vc[3] == 0x7FC1).all()  # nothing copied for an empty slot
        check_out(r.fast_compact(q1, nsel, sel.shape[2], rs1, ctx1), ref_sparse)

        _step(f"{variant}: mixed step, an empty slot on either side")
        slow = np.array([0, 1, 1, 0], np.uint8)
        sel_d, nsel_d = i32_dev(sel), i32_dev(nsel)
        r.out.fill_(float("nan"))
        sfi.sfi_mixed_step(h, to_dev(q1), r.K, r.V, torch.from_numpy(slow).cuda(), i32_dev(ctx1), i32_dev(rs1), 0,
                           w.budget, r.out, sel_d, nsel_d)
        torch.cuda.synchronize()
        got = r.out.cpu().numpy()
        ref_dense = oracle.dense(q1, w.K, w.V, ctx1)
        sel1, nsel1 = sel_d.cpu().numpy(), nsel_d.cpu().numpy()
        sel_ref1, nsel_ref1, z1 = oracle.selector(q1, w.K, ctx1, w.budget, w.n_sink, w.recent, **({"sp": sp} if sp else {}))
        for b in range(w.B):
            check_out(got[b], ref_dense[b] if slow[b] else ref_sparse[b])
            if slow[b]:
                check_selection(sel1[b:b + 1], nsel1[b:b + 1], sel_ref1[b:b + 1], nsel_ref1[b:b + 1], z1[b:b + 1],
                                ctx1[b:b + 1], w.n_sink, w.recent, w.budget, **band)
            else:
                assert (sel1[b] == sel[b]).all() and (nsel1[b] == nsel[b]).all()

        _step(f"{variant}: windowed evidence over two queries")
        ctx_d = i32_dev(ctx0)
        r.out.fill_(float("nan"))
        sfi.sfi_evidence_add(h, to_dev(q0), r.K, r.V, ctx_d, 0, r.out, True)
        sfi.sfi_evidence_add(h, to_dev(q1), r.K, r.V, ctx_d, 0, None, False)
        sel_w = torch.full((w.B, w.Hkv, w.budget), -7, dtype=torch.int32, device="cuda")
        nsel_w = torch.full((w.B, w.Hkv), -7, dtype=torch.int32, device="cuda")
        sfi.sfi_evidence_select(h, 2, ctx_d, 0, w.budget, sel_w, nsel_w)
        torch.cuda.synchronize()
        check_out(r.out.cpu().numpy(), oracle.dense(q0, w.K, w.V, ctx0))
        nsel_w = nsel_w.cpu().numpy()
        assert (nsel_w[1] == 0).all() and (nsel_w[3] == 0).all() and (nsel_w[0] == w.budget).all()
        assert (sel_w.cpu().numpy()[1] == -1).all()

        assert sfi.sfi_device_status(h) == 0  # an empty slot is a legal input
    finally:
        r.close()


def test_all_slots_empty(oracle):
    """Nothing live at all: every call returns zeros and empty index sets."""
    w = syn.make_tiny(L0=600, steps=1, budget=32, recent=32, n_support=4, B=2)
    ctx = np.zeros(2, np.int32)
    r = Runner(w)
    try:
        _step("all slots empty")
        q = w.q(0)
        out, sel, nsel = r.slow(q, ctx, w.budget)
        assert not out.any() and not nsel.any() and (sel == -1).all()
        assert not r.dense(q, ctx).any()
        assert not r.fast(q, sel, nsel, ctx, ctx).any()
        r.reorg(sel, nsel, ctx)
        assert not r.fast_compact(q, nsel, sel.shape[2], ctx, ctx).any()
        assert r.sfi.sfi_device_status(r.ctx.handle) == 0
    finally:
        r.close()
