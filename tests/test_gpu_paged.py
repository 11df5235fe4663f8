"""GPU parity with a paged cache: K and V handed over as block pools plus a per-sequence block table, the
expected values from the oracle on the flat cache the pools were scattered from.  Blocks no valid table
entry points to hold a NaN pattern, so a wrong translation shows up as a wrong (non-finite) result."""
import numpy as np
import pytest

import sfi_synth as syn
from helpers import Runner, check_out, check_selection, i32_dev, to_dev

pytestmark = pytest.mark.gpu


def _step(msg):
    print(f"[gpu-paged] {msg}", flush=True)


@pytest.mark.parametrize("page,layout", [(16, "thd"), (64, "thd"), (512, "thd"), (16, "htd"), (128, "htd")])
def test_paged_slow_and_fast_steps(oracle, page, layout):
    """Slow step (dense output + Selector) and fast steps (one tile per wave and the pipelined walk) through
    the block table, ragged contexts, table entries past each context pointing at a poison block."""
    w = syn.make_tiny(L0=2500, steps=4, budget=96, recent=64, n_support=16, B=2)
    w.L0 = np.array([2500, 1203], np.int32)
    r = Runner(w, page_size=page, ctx_max=w.L0 + 4, page_layout=layout)
    try:
        _step(f"page {page} {layout}: slow step")
        q0, ctx = w.q(0), w.ctx_len(0)
        out, sel, nsel = r.slow(q0, ctx, w.budget)
        check_out(out, oracle.dense(q0, w.K, w.V, ctx))
        sel_ref, nsel_ref, z = oracle.selector(q0, w.K, ctx, w.budget, w.n_sink, w.recent)
        check_selection(sel, nsel, sel_ref, nsel_ref, z, ctx, w.n_sink, w.recent, w.budget)
        check_out(r.dense(q0, ctx), oracle.dense(q0, w.K, w.V, ctx))
        for tpw in (1, 3, 40):
            _step(f"page {page}: fast steps, {tpw} tiles per wave")
            r.sfi.sfi_set_tuning(r.ctx.handle, 0, tpw)
            for t in range(1, 3):
                q, ctx_t, rs = w.q(t), w.ctx_len(t), w.recent_start(t)
                got = r.fast(q, sel, nsel, rs, ctx_t)
                check_out(got, oracle.sparse(q, w.K, w.V, sel, nsel, rs, ctx_t, w.n_sink))
        _step(f"page {page}: reorg + compact fast step")
        Kc, Vc = r.reorg(sel, nsel, ctx)
        Kc_ref, Vc_ref = np.full_like(Kc, 0x7FC1), np.full_like(Vc, 0x7FC1)
        oracle.reorg(w.K, w.V, sel, nsel, ctx, w.n_sink, Kc_ref, Vc_ref)
        assert (Kc == Kc_ref).all() and (Vc == Vc_ref).all()
        q, ctx_t, rs = w.q(1), w.ctx_len(1), w.recent_start(1)
        check_out(r.fast_compact(q, nsel, sel.shape[2], rs, ctx_t), oracle.sparse(q, w.K, w.V, sel, nsel, rs, ctx_t, w.n_sink))
    finally:
        r.close()


@pytest.mark.parametrize("L", [1, 3, 5, 37, 69, 70, 200])
def test_paged_short_contexts(oracle, L):
    """Contexts of a single row up to a few pages: sink / recent only, J empty or tiny."""
    w = syn.make_tiny(L0=400, steps=1, budget=32, recent=32, n_support=4, B=2, Hq=16, Hkv=2)
    ctx = np.array([L, max(1, L - 1)], np.int32)
    r = Runner(w, page_size=16, ctx_max=ctx)
    try:
        _step(f"paged short context L={L}")
        q = w.q(0)
        out, sel, nsel = r.slow(q, ctx, w.budget)
        check_out(out, oracle.dense(q, w.K, w.V, ctx))
        sel_ref, nsel_ref, z = oracle.selector(q, w.K, ctx, w.budget, w.n_sink, w.recent)
        check_selection(sel, nsel, sel_ref, nsel_ref, z, ctx, w.n_sink, w.recent, w.budget)
        rs = np.maximum(np.minimum(w.n_sink, ctx), ctx - w.recent).astype(np.int32)
        got = r.fast(q, sel, nsel, rs, ctx)
        check_out(got, oracle.sparse(q, w.K, w.V, sel, nsel, rs, ctx, w.n_sink))
    finally:
        r.close()


def test_paged_few_splits_and_group_sizes(oracle):
    """G = 8 with one split per pair (stash written out on the way), and the full Selector, over pages of 32."""
    w = syn.make_tiny(L0=5000, steps=1, budget=96, recent=40, n_support=8, B=1, Hq=16, Hkv=2)
    r = Runner(w, page_size=32)
    try:
        _step("paged, one split per pair")
        r.sfi.sfi_set_tuning(r.ctx.handle, 1, 1)
        q, ctx = w.q(0), w.ctx_len(0)
        out, sel, nsel = r.slow(q, ctx, w.budget)
        check_out(out, oracle.dense(q, w.K, w.V, ctx))
        sel_ref, nsel_ref, z = oracle.selector(q, w.K, ctx, w.budget, w.n_sink, w.recent)
        check_selection(sel, nsel, sel_ref, nsel_ref, z, ctx, w.n_sink, w.recent, w.budget)
    finally:
        r.close()


def test_paged_mixed_step(oracle):
    """Per-sequence modes over a paged cache."""
    import torch
    import paper_2603_12038_amd as sfi

    w = syn.make_serving(steps=4, B=5, Hq=16, Hkv=2, len_lo=300, len_hi=1400, budget=64, recent=32)
    r = Runner(w, page_size=64)
    try:
        _step("paged mixed step")
        B = w.B
        ctx_d, rs_d = i32_dev(w.ctx_len(0)), i32_dev(w.recent_start(0))
        sel_d = torch.full((B, w.Hkv, w.budget), -7, dtype=torch.int32, device="cuda")
        nsel_d = torch.full((B, w.Hkv), -7, dtype=torch.int32, device="cuda")
        q0 = w.q(0)
        sfi.sfi_mixed_step(r.ctx.handle, to_dev(q0), r.K, r.V, torch.ones(B, dtype=torch.uint8, device="cuda"), ctx_d, rs_d,
                           0, w.budget, r.out, sel_d, nsel_d)
        torch.cuda.synchronize()
        ctx0 = w.ctx_len(0)
        check_out(r.out.cpu().numpy(), oracle.dense(q0, w.K, w.V, ctx0))
        sel0, nsel0 = sel_d.cpu().numpy(), nsel_d.cpu().numpy()
        sfi.sfi_advance(r.ctx.handle, ctx_d, rs_d)
        slow1 = np.array([0, 1, 0, 0, 1], np.uint8)
        q1, ctx1, rs1 = w.q(1), w.ctx_len(1), w.recent_start(1)
        sfi.sfi_mixed_step(r.ctx.handle, to_dev(q1), r.K, r.V, torch.from_numpy(slow1).cuda(), ctx_d, rs_d, 0, w.budget,
                           r.out, sel_d, nsel_d)
        torch.cuda.synchronize()
        got = r.out.cpu().numpy()
        ref_dense = oracle.dense(q1, w.K, w.V, ctx1)
        ref_sparse = oracle.sparse(q1, w.K, w.V, sel0, nsel0, rs1, ctx1, w.n_sink)
        for b in range(B):
            check_out(got[b], ref_dense[b] if slow1[b] else ref_sparse[b])
    finally:
        r.close()


def test_paged_calls_need_a_table(oracle):
    """A context created for a paged cache refuses hot calls until a block table is attached."""
    import paper_2603_12038_amd as sfi

    w = syn.make_tiny(L0=300, steps=1, budget=16, recent=16, n_support=2, B=1)
    r = Runner(w, page_size=16)
    try:
        sfi.sfi_set_block_table(r.ctx.handle, None, 0)
        with pytest.raises(sfi.SfiError):
            r.dense(w.q(0), w.ctx_len(0))
        with pytest.raises(sfi.SfiError):
            short = r.torch.zeros(w.B, 2, dtype=r.torch.int32, device="cuda")  # 2 pages per sequence < max_ctx / 16
            sfi.sfi_set_block_table(r.ctx.handle, short.repeat(2, 1), r.K.shape[0])
        sfi.sfi_set_block_table(r.ctx.handle, r.table, r.K.shape[0])
        check_out(r.dense(w.q(0), w.ctx_len(0)), oracle.dense(w.q(0), w.K, w.V, w.ctx_len(0)))
    finally:
        r.close()


@pytest.mark.parametrize("mode", [0, 1])
def test_paged_evidence_only_pass(oracle, mode):
    """The evidence-only pass (sfi_evidence_add without V and out) over a paged cache: the windowed selection
    equals the one of the flat cache, bit for bit, in both Selector modes."""
    import dataclasses
    import torch
    from oracle.sfi_oracle import SelectorParams
    sp = SelectorParams(mode=1)
    d = None
    if mode == 1:
        d = {k: getattr(sp, k) for k in ("gamma", "beta", "p", "eta", "lambda_clip", "alpha_soft", "alpha_cross", "temp",
                                          "eps", "nms_radius")}
    w = syn.make_tiny(L0=3300, steps=4, budget=120, recent=40, n_support=16, B=2, Hq=8, Hkv=2)
    w.L0 = np.array([3300, 2111], np.int32)
    got = []
    for page in (0, 64):
        r = Runner(w, selector=d, page_size=page)
        try:
            _step(f"evidence-only pass, mode {mode}, page size {page}")
            ctx_d = i32_dev(w.ctx_len(0))
            sel = torch.full((w.B, w.Hkv, w.budget), -7, dtype=torch.int32, device="cuda")
            nsel = torch.full((w.B, w.Hkv), -7, dtype=torch.int32, device="cuda")
            for t in range(3):
                r.sfi.sfi_evidence_add(r.ctx.handle, to_dev(w.q(t)), r.K, None, ctx_d, 0, None, t == 0)
            r.sfi.sfi_evidence_select(r.ctx.handle, 3, ctx_d, 0, w.budget, sel, nsel)
            torch.cuda.synchronize()
            got.append((sel.cpu().numpy(), nsel.cpu().numpy()))
        finally:
            r.close()
    assert np.array_equal(got[0][0], got[1][0]) and np.array_equal(got[0][1], got[1][1])
    assert (got[0][1] == w.budget).all()
