"""GPU parity at the baseline configurations' full sizes, in the launch configuration bench.py times.

The oracle finishes most of these sizes in about a second per step on the GPU machine's host cores, so every
output element and every index set is compared; the full serving batch (32 ragged sequences of up to 65536
rows) is the exception: the GPU computes all of it, the oracle checks every sequence's fast steps and a sample
of the dense ones, named in the test."""
import numpy as np
import pytest

import sfi_synth as syn
from helpers import Runner, check_out, check_selection, i32_dev, to_dev

pytestmark = pytest.mark.gpu


def _step(msg):
    print(f"[gpu-full] {msg}", flush=True)


def _slow_then_fast(oracle, w, n_fast=2):
    r = Runner(w)
    try:
        q0, c0 = w.q(0), w.ctx_len(0)
        _step(f"{w.name}: slow step B={w.B} Hq={w.Hq} Hkv={w.Hkv} ctx={int(c0.max())} K={w.budget}")
        out, sel, nsel = r.slow(q0, c0, w.budget)
        e = check_out(out, oracle.dense(q0, w.K, w.V, c0))
        sel_ref, nsel_ref, z = oracle.selector(q0, w.K, c0, w.budget, w.n_sink, w.recent)
        n_exact = check_selection(sel, nsel, sel_ref, nsel_ref, z, c0, w.n_sink, w.recent, w.budget)
        _step(f"  slow out err {e:.2e}; index sets identical to the oracle's: {n_exact}/{w.B * w.Hkv}")
        assert n_exact >= (w.B * w.Hkv) // 2
        for t in range(1, 1 + n_fast):
            q, ct, rt = w.q(t), w.ctx_len(t), w.recent_start(t)
            got = r.fast(q, sel, nsel, rt, ct)
            e = check_out(got, oracle.sparse(q, w.K, w.V, sel, nsel, rt, ct, w.n_sink))
            _step(f"  fast step {t} out err {e:.2e}")
        return r
    except Exception:
        r.close()
        raise


def test_llama8b_shaped_layer(oracle):
    """Config 2: B4, 32/8 heads, ctx 32768, K = 2048, recent 128 — the workload bench.py times."""
    w = syn.make_llama8b(steps=8)
    r = _slow_then_fast(oracle, w)
    try:
        # support drift: 10 % of the planted rows move, then the next slow step must follow them
        patches = syn.drift_support(w, epoch=1)
        Kd = to_dev(w.K)
        r.K.copy_(Kd)
        q, c = w.q(3), w.ctx_len(3)
        out, sel, nsel = r.slow(q, c, w.budget)
        check_out(out, oracle.dense(q, w.K, w.V, c))
        sel_ref, nsel_ref, z = oracle.selector(q, w.K, c, w.budget, w.n_sink, w.recent)
        check_selection(sel, nsel, sel_ref, nsel_ref, z, c, w.n_sink, w.recent, w.budget)
        assert len(patches) == w.B * w.Hkv
    finally:
        r.close()


def test_in_kernel_merge_never_reads_a_stale_record(oracle):
    """Config 2 shape, several split workgroups per pair: 600 fast steps in a row alternating
    between two queries and two index sets.  Every output must be bit-identical to the first output of its
    query (checked against the oracle): a record left over from the launch before, read in place of a fresh
    one, would belong to the other query."""
    import torch
    w = syn.make_llama8b(steps=4)
    r = Runner(w)
    try:
        ctx, rs = w.ctx_len(1), w.recent_start(1)
        ctx_d, rs_d = i32_dev(ctx), i32_dev(rs)
        cases = []
        for k in range(2):
            q = w.q(1 + k)
            nsel = np.full((w.B, w.Hkv), w.budget - 5 * k, np.int32)
            sel = syn.random_sel(900 + k, w.B, w.Hkv, w.budget, nsel, w.n_sink, rs)
            ref = r.fast(q, sel, nsel, rs, ctx)
            check_out(ref, oracle.sparse(q, w.K, w.V, sel, nsel, rs, ctx, w.n_sink))
            cases.append((to_dev(q), i32_dev(sel), i32_dev(nsel), torch.from_numpy(ref).cuda()))
        assert r.sfi.sfi_query_splits(r.ctx.handle)[1] >= 4
        _step("600 alternating fast steps, in-kernel merge")
        outs = [torch.empty_like(cases[0][3]) for _ in range(600)]
        for i, o in enumerate(outs):
            qd, sd, nd, _ = cases[i & 1]
            r.sfi.sfi_fast_step(r.ctx.handle, qd, r.K, r.V, sd, nd, w.budget, rs_d, ctx_d, o)
        torch.cuda.synchronize()
        for i, o in enumerate(outs):
            assert torch.equal(o, cases[i & 1][3]), f"launch {i} differs from the first output of its query"
    finally:
        r.close()


def test_long_single_stream(oracle):
    """Config 3: B1, 32/8 heads, ctx 131072, clustered support, K = 4096, recent 256."""
    w = syn.make_long(steps=4)
    _slow_then_fast(oracle, w).close()


@pytest.mark.parametrize("L0", [8192, 24576, 38912])
def test_long_cot_window(oracle, L0):
    """Config 4 at its three sample points (start of the windows at 8K, 24K and 40K): B8, 40/8 heads (G = 5),
    K = 1024, recent 128."""
    w = syn.make_cot(L0=L0, steps=4)
    _slow_then_fast(oracle, w).close()


def test_serving_mix_ragged(oracle):
    """Config 5 shape at a quarter of the batch: B8, 64/8 heads (G = 8), ragged ctx in [16384, 65536],
    K = 2048: first step all slow, then a mixed step with per-sequence modes."""
    import torch
    import paper_2603_12038_amd as sfi

    w = syn.make_serving(steps=4, B=8)
    r = Runner(w)
    try:
        B = w.B
        ctx_d, rs_d = i32_dev(w.ctx_len(0)), i32_dev(w.recent_start(0))
        sel_d = torch.full((B, w.Hkv, w.budget), -7, dtype=torch.int32, device="cuda")
        nsel_d = torch.full((B, w.Hkv), -7, dtype=torch.int32, device="cuda")
        q0, c0 = w.q(0), w.ctx_len(0)
        _step(f"serving mix: all-slow mixed step, ctx {c0.tolist()}")
        sfi.sfi_mixed_step(r.ctx.handle, to_dev(q0), r.K, r.V, torch.ones(B, dtype=torch.uint8, device="cuda"), ctx_d,
                           rs_d, 0, w.budget, r.out, sel_d, nsel_d)
        torch.cuda.synchronize()
        check_out(r.out.cpu().numpy(), oracle.dense(q0, w.K, w.V, c0))
        sel_ref, nsel_ref, z = oracle.selector(q0, w.K, c0, w.budget, w.n_sink, w.recent)
        sel0, nsel0 = sel_d.cpu().numpy(), nsel_d.cpu().numpy()
        check_selection(sel0, nsel0, sel_ref, nsel_ref, z, c0, w.n_sink, w.recent, w.budget)
        sfi.sfi_advance(r.ctx.handle, ctx_d, rs_d)
        slow1 = np.zeros(B, np.uint8)
        slow1[[2, 5]] = 1
        q1, c1, rs1 = w.q(1), w.ctx_len(1), w.recent_start(1)
        _step("serving mix: 2 slow + 6 fast sequences in one call")
        sfi.sfi_mixed_step(r.ctx.handle, to_dev(q1), r.K, r.V, torch.from_numpy(slow1).cuda(), ctx_d, rs_d, 0,
                           w.budget, r.out, sel_d, nsel_d)
        torch.cuda.synchronize()
        got = r.out.cpu().numpy()
        ref_d = oracle.dense(q1, w.K, w.V, c1)
        ref_s = oracle.sparse(q1, w.K, w.V, sel0, nsel0, rs1, c1, w.n_sink)
        sel1, nsel1 = sel_d.cpu().numpy(), nsel_d.cpu().numpy()
        sel_ref1, nsel_ref1, z1 = oracle.selector(q1, w.K, c1, w.budget, w.n_sink, w.recent)
        for b in range(B):
            if slow1[b]:
                check_out(got[b], ref_d[b])
                check_selection(sel1[b:b + 1], nsel1[b:b + 1], sel_ref1[b:b + 1], nsel_ref1[b:b + 1], z1[b:b + 1],
                                c1[b:b + 1], w.n_sink, w.recent, w.budget)
            else:
                check_out(got[b], ref_s[b])
                assert (sel1[b] == sel0[b]).all()
    finally:
        r.close()


def test_serving_mix_full_batch(oracle):
    """Config 5 at its full batch: B32, 64/8 heads (G = 8), ragged ctx in [16384, 65536], K = 2048 -- the launch
    plan bench.py's serving workload times (256 pairs: one workgroup per pair in the fast part, output written
    directly).  An all-slow step, a mixed step and an all-fast step.  The GPU computes all 32 sequences every time;
    the oracle checks every sequence on the fast side (cheap) and, on the dense side, the longest, the shortest
    and four more (a dense sequence costs it seconds)."""
    import torch
    import paper_2603_12038_amd as sfi

    w = syn.make_serving(steps=4)
    assert w.B == 32
    _step(f"serving mix at full batch: generated, ctx {int(w.L0.min())}..{int(w.L0.max())}")
    r = Runner(w)
    try:
        B = w.B
        one = lambda x, b: x[b:b + 1]
        ctx_d, rs_d = i32_dev(w.ctx_len(0)), i32_dev(w.recent_start(0))
        sel_d = torch.full((B, w.Hkv, w.budget), -7, dtype=torch.int32, device="cuda")
        nsel_d = torch.full((B, w.Hkv), -7, dtype=torch.int32, device="cuda")
        order = np.argsort(w.L0)
        sample = sorted({int(order[0]), int(order[-1]), 3, 11, 19, 27})
        # ---- all slow
        q0, c0 = w.q(0), w.ctx_len(0)
        sfi.sfi_mixed_step(r.ctx.handle, to_dev(q0), r.K, r.V, torch.ones(B, dtype=torch.uint8, device="cuda"), ctx_d,
                           rs_d, 0, w.budget, r.out, sel_d, nsel_d)
        torch.cuda.synchronize()
        got0, sel0, nsel0 = r.out.cpu().numpy(), sel_d.cpu().numpy(), nsel_d.cpu().numpy()
        assert np.isfinite(got0).all()
        for b in sample:
            e = check_out(got0[b:b + 1], oracle.dense(one(q0, b), one(w.K, b), one(w.V, b), one(c0, b)))
            sr, nr, z = oracle.selector(one(q0, b), one(w.K, b), one(c0, b), w.budget, w.n_sink, w.recent)
            n_exact = check_selection(one(sel0, b), one(nsel0, b), sr, nr, z, one(c0, b), w.n_sink, w.recent, w.budget)
            _step(f"  all-slow step, sequence {b} (ctx {int(c0[b])}): out err {e:.2e}, sets identical {n_exact}/{w.Hkv}")
        for b in range(B):  # structure of every sequence's sets
            for h in range(w.Hkv):
                k = int(nsel0[b, h])
                assert k == min(w.budget, int(c0[b]) - w.recent - w.n_sink) and (np.diff(sel0[b, h, :k]) > 0).all()
                assert sel0[b, h, 0] >= w.n_sink and sel0[b, h, k - 1] < int(c0[b]) - w.recent
        # ---- mixed: three slow sequences, one of them checked densely by the oracle
        sfi.sfi_advance(r.ctx.handle, ctx_d, rs_d)
        slow1 = np.zeros(B, np.uint8)
        slow1[[sample[1], 17, 30]] = 1
        q1, c1, rs1 = w.q(1), w.ctx_len(1), w.recent_start(1)
        sfi.sfi_mixed_step(r.ctx.handle, to_dev(q1), r.K, r.V, torch.from_numpy(slow1).cuda(), ctx_d, rs_d, 0,
                           w.budget, r.out, sel_d, nsel_d)
        torch.cuda.synchronize()
        got1, sel1, nsel1 = r.out.cpu().numpy(), sel_d.cpu().numpy(), nsel_d.cpu().numpy()
        ref_s = oracle.sparse(q1, w.K, w.V, sel0, nsel0, rs1, c1, w.n_sink)
        for b in range(B):
            if slow1[b]:
                if b in (sample[1], 17):
                    check_out(got1[b:b + 1], oracle.dense(one(q1, b), one(w.K, b), one(w.V, b), one(c1, b)))
                    sr, nr, z = oracle.selector(one(q1, b), one(w.K, b), one(c1, b), w.budget, w.n_sink, w.recent)
                    check_selection(one(sel1, b), one(nsel1, b), sr, nr, z, one(c1, b), w.n_sink, w.recent, w.budget)
            else:
                check_out(got1[b], ref_s[b])
                assert (sel1[b] == sel0[b]).all()
        _step("  mixed step (3 slow + 29 fast sequences) ok")
        # ---- all fast
        sfi.sfi_advance(r.ctx.handle, ctx_d, rs_d)
        q2, c2, rs2 = w.q(2), w.ctx_len(2), w.recent_start(2)
        sfi.sfi_mixed_step(r.ctx.handle, to_dev(q2), r.K, r.V, torch.zeros(B, dtype=torch.uint8, device="cuda"), ctx_d,
                           rs_d, 0, w.budget, r.out, sel_d, nsel_d)
        torch.cuda.synchronize()
        e = check_out(r.out.cpu().numpy(), oracle.sparse(q2, w.K, w.V, sel1, nsel1, rs2, c2, w.n_sink))
        assert (sel_d.cpu().numpy() == sel1).all()
        assert sfi.sfi_query_splits(r.ctx.handle)[1] == 1, "256 pairs: one workgroup per pair, output written directly"
        got = r.fast(q2, sel1, nsel1, rs2, c2)     # the same step through sfi_fast_step
        check_out(got, oracle.sparse(q2, w.K, w.V, sel1, nsel1, rs2, c2, w.n_sink))
        _step(f"  all-fast step ok, out err {e:.2e}")
        assert sfi.sfi_device_status(r.ctx.handle) == 0
    finally:
        r.close()


def test_retention_sweep_shape(oracle):
    """Shape of the paper's kernel-speedup table: KV length 16K, batch 16, retention 25 %."""
    w = syn.make_retention_sweep(0.25)
    r = Runner(w)
    try:
        _step("retention sweep shape, 25 %")
        q, c = w.q(0), w.ctx_len(0)
        out, sel, nsel = r.slow(q, c, w.budget)
        check_out(out, oracle.dense(q, w.K, w.V, c))
        got = r.fast(q, sel, nsel, w.recent_start(0), c)
        check_out(got, oracle.sparse(q, w.K, w.V, sel, nsel, w.recent_start(0), c, w.n_sink))
    finally:
        r.close()


def test_million_token_context(oracle):
    """One sequence of 2^20 cached rows (B1, 4/1 heads, K = 4096, recent 512): 512 Selector segments, the
    finest dense split, 32-bit row offsets close to their limit for this row stride."""
    w = syn.make_long(L0=(1 << 20) - 2, steps=2, B=1, Hq=4, Hkv=1, budget=4096, recent=512, n_clusters=256)
    _slow_then_fast(oracle, w, n_fast=1).close()
