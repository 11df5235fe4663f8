"""Outputs stored as bf16 (cfg.out_bf16 = 1): the fp32 result of every path rounded to nearest even as it is
written -- direct output of a single workgroup, in-kernel merge, merge launch, merge inside the Selector's
first launch.  The index sets do not depend on the output type."""
import numpy as np
import pytest

import sfi_synth as syn
from helpers import Runner, check_out_bf16, check_selection, i32_dev, to_dev

pytestmark = pytest.mark.gpu


def _step(msg):
    print(f"[gpu-bf16-out] {msg}", flush=True)


@pytest.mark.parametrize("page", [0, 32])
def test_bf16_outputs_through_every_entry_point(oracle, page):
    import torch
    w = syn.make_tiny(L0=3000, steps=3, budget=96, recent=64, n_support=16, B=3)
    w.L0 = np.array([3000, 1100, 0], np.int32)
    r = Runner(w, out_bf16=True, page_size=page)
    f32 = Runner(w, page_size=page)
    try:
        sfi, h = r.sfi, r.ctx.handle
        q0, ctx0 = w.q(0), w.ctx_len(0)
        _step(f"page {page}: slow step and dense attention")
        out, sel, nsel = r.slow(q0, ctx0, w.budget)
        ref = oracle.dense(q0, w.K, w.V, ctx0)
        check_out_bf16(out, ref)
        out32, sel32, nsel32 = f32.slow(q0, ctx0, w.budget)
        assert np.array_equal(sel, sel32) and np.array_equal(nsel, nsel32)
        # the bf16 output is the fp32 output rounded to nearest even, bit for bit
        rounded = torch.from_numpy(out32).to(torch.bfloat16).float().numpy()
        assert np.array_equal(out, rounded)
        check_out_bf16(r.dense(q0, ctx0), ref)
        q1, ctx1, rs1 = w.q(1), w.ctx_len(1), w.recent_start(1)
        ctx1[2], rs1[2] = 0, 0
        ref1 = oracle.sparse(q1, w.K, w.V, sel, nsel, rs1, ctx1, w.n_sink)
        for tpw, merge in ((1, 1), (3, 1), (1, 2), (40, 1)):
            _step(f"page {page}: fast step, {tpw} tiles per wave, merge mode {merge}")
            sfi.sfi_set_tuning(h, 0, tpw, merge)
            f32.sfi.sfi_set_tuning(f32.ctx.handle, 0, tpw, merge)
            got = r.fast(q1, sel, nsel, rs1, ctx1)
            check_out_bf16(got, ref1)
            got32 = f32.fast(q1, sel, nsel, rs1, ctx1)
            assert np.array_equal(got, torch.from_numpy(got32).to(torch.bfloat16).float().numpy())
        sfi.sfi_set_tuning(h, 0, -1, 1)
        _step(f"page {page}: reorg + compact fast step")
        r.reorg(sel, nsel, ctx0)
        check_out_bf16(r.fast_compact(q1, nsel, sel.shape[2], rs1, ctx1), ref1)
        _step(f"page {page}: mixed step")
        slow = np.array([1, 0, 1], np.uint8)
        sel_d, nsel_d = i32_dev(sel), i32_dev(nsel)
        r.out.fill_(float("nan"))
        sfi.sfi_mixed_step(h, to_dev(q1), r.K, r.V, torch.from_numpy(slow).cuda(), i32_dev(ctx1), i32_dev(rs1), 0,
                           w.budget, r.out, sel_d, nsel_d)
        torch.cuda.synchronize()
        got = r.out.float().cpu().numpy()
        ref_dense = oracle.dense(q1, w.K, w.V, ctx1)
        for b in range(w.B):
            check_out_bf16(got[b], ref_dense[b] if slow[b] else ref1[b])
        _step(f"page {page}: slow step in two halves, windowed evidence")
        ctx_d = i32_dev(ctx0)
        r.out.fill_(float("nan"))
        sfi.sfi_slow_attn(h, to_dev(q0), r.K, r.V, ctx_d, 0, r.out)
        torch.cuda.synchronize()
        check_out_bf16(r.out.float().cpu().numpy(), ref)
        r.out.fill_(float("nan"))
        sfi.sfi_evidence_add(h, to_dev(q0), r.K, r.V, ctx_d, 0, r.out, True)
        torch.cuda.synchronize()
        check_out_bf16(r.out.float().cpu().numpy(), ref)
        assert sfi.sfi_device_status(h) == 0
    finally:
        r.close()
        f32.close()


def test_bf16_outputs_full_selector(oracle):
    import dataclasses
    from oracle.sfi_oracle import SelectorParams
    sp = SelectorParams(mode=1)
    d = {k: getattr(sp, k) for k in ("gamma", "beta", "p", "eta", "lambda_clip", "alpha_soft", "alpha_cross", "temp",
                                      "eps", "nms_radius")}
    w = syn.make_tiny(L0=2600, steps=1, budget=96, recent=48, n_support=12, B=2, Hq=8, Hkv=2)
    r = Runner(w, selector=d, alpha=sp.alpha, out_bf16=True)
    try:
        _step("full Selector with bf16 outputs")
        q, ctx = w.q(0), w.ctx_len(0)
        out, sel, nsel = r.slow(q, ctx, w.budget)
        check_out_bf16(out, oracle.dense(q, w.K, w.V, ctx))
        sel_ref, nsel_ref, z = oracle.selector(q, w.K, ctx, w.budget, w.n_sink, w.recent, sp=sp)
        check_selection(sel, nsel, sel_ref, nsel_ref, z, ctx, w.n_sink, w.recent, w.budget)
    finally:
        r.close()
