"""GPU parity: libsfi (through its C-ABI binding) against the fp64 oracle, element by element.

Sizes are small enough for the oracle to finish in seconds yet span several 32-row tiles, several
split workgroups and a ragged tail.  Output bar: row-relative error <= 2e-3.  Index sets: identical
to the oracle's wherever the ranking-score gap at the cut exceeds 1e-5, valid inside that band.
"""
import numpy as np
import pytest

import sfi_synth as syn
from helpers import Runner, check_out, check_selection, i32_dev, to_dev

pytestmark = pytest.mark.gpu


def _step(msg):
    print(f"[gpu-parity] {msg}", flush=True)


@pytest.fixture(scope="module")
def tiny():
    w = syn.make_tiny(L0=1500, steps=4, budget=96, recent=64, n_support=16, B=2)
    w.L0 = np.array([1500, 1003], np.int32)
    r = Runner(w)
    yield w, r
    r.close()


def test_dense_matches_oracle(oracle, tiny):
    w, r = tiny
    _step("dense B=2 Hq=8 Hkv=2 L=(1500,1003)")
    q = w.q(0)
    ctx = w.ctx_len(0)
    got = r.dense(q, ctx)
    check_out(got, oracle.dense(q, w.K, w.V, ctx))


@pytest.mark.parametrize("L", [1, 3, 4, 5, 31, 32, 33, 68, 69, 100, 257])
def test_dense_short_contexts(oracle, tiny, L):
    """ctx_len around n_sink, n_sink + recent and tile boundaries; J may be empty."""
    w, r = tiny
    _step(f"dense short L={L}")
    q = w.q(1)
    ctx = np.array([L, max(1, L - 1)], np.int32)
    got = r.dense(q, ctx)
    check_out(got, oracle.dense(q, w.K, w.V, ctx))


def test_slow_step_matches_oracle(oracle, tiny):
    w, r = tiny
    _step("slow step")
    q = w.q(2)
    ctx = w.ctx_len(0)
    out, sel, nsel = r.slow(q, ctx, w.budget)
    check_out(out, oracle.dense(q, w.K, w.V, ctx))
    sel_ref, nsel_ref, z = oracle.selector(q, w.K, ctx, w.budget, w.n_sink, w.recent)
    n_exact = check_selection(sel, nsel, sel_ref, nsel_ref, z, ctx, w.n_sink, w.recent, w.budget)
    assert n_exact >= 1


@pytest.mark.parametrize("budget", [0, 1, 7, 96])
@pytest.mark.parametrize("L", [1, 4, 68, 69, 70, 100, 165, 700])
def test_slow_step_edges(oracle, tiny, L, budget):
    """|J| = 0, 1, 2, < budget, == budget + 1; budget 0 and 1."""
    w, r = tiny
    _step(f"slow edges L={L} budget={budget}")
    q = w.q(3)
    ctx = np.array([L, L + 1], np.int32)
    out, sel, nsel = r.slow(q, ctx, budget)
    check_out(out, oracle.dense(q, w.K, w.V, ctx))
    sel_ref, nsel_ref, z = oracle.selector(q, w.K, ctx, budget, w.n_sink, w.recent)
    if budget == 0:
        assert (nsel == 0).all()
    else:
        check_selection(sel, nsel, sel_ref, nsel_ref, z, ctx, w.n_sink, w.recent, budget)


def test_fast_step_matches_oracle(oracle, tiny):
    w, r = tiny
    _step("fast step with the slow step's own selection, then three more steps")
    q0 = w.q(0)
    ctx = w.ctx_len(0)
    _, sel, nsel = r.slow(q0, ctx, w.budget)
    for t in range(1, 4):
        q = w.q(t)
        ctx_t, rs = w.ctx_len(t), w.recent_start(t)
        got = r.fast(q, sel, nsel, rs, ctx_t)
        check_out(got, oracle.sparse(q, w.K, w.V, sel, nsel, rs, ctx_t, w.n_sink))


def test_fast_step_random_sets_and_edges(oracle, tiny):
    """Arbitrary valid index sets (not the Selector's), ragged n_sel, contexts down to a single row."""
    w, r = tiny
    q = w.q(5)
    for case, (L, ns) in enumerate([(1500, 96), (1500, 0), (1500, 1), (300, 33), (70, 2), (68, 0), (5, 0), (3, 0), (1, 0)]):
        _step(f"fast random sets L={L} n_sel={ns}")
        ctx = np.array([L, max(1, L - 2)], np.int32)
        rs = np.maximum(np.minimum(w.n_sink, ctx), ctx - w.recent).astype(np.int32)
        room = np.maximum(0, rs - w.n_sink)
        nsel = np.minimum(ns, room)[:, None].repeat(w.Hkv, axis=1).astype(np.int32)
        nsel[1, 0] = max(0, nsel[1, 0] - 1)
        sel = syn.random_sel(100 + case, w.B, w.Hkv, w.budget, nsel, w.n_sink, rs)
        got = r.fast(q, sel, nsel, rs, ctx)
        check_out(got, oracle.sparse(q, w.K, w.V, sel, nsel, rs, ctx, w.n_sink))


def test_fast_with_full_index_set_equals_dense(oracle, tiny):
    """sel = all of J  =>  the fast step reproduces dense attention (checked against the oracle's dense)."""
    w, _ = tiny
    L = 900
    w2 = syn.make_tiny(L0=L, steps=1, budget=L, recent=64, n_support=4, B=1)
    r2 = Runner(w2)
    try:
        _step("fast with sel = J")
        q = w2.q(0)
        ctx = np.array([L], np.int32)
        rs = ctx - w2.recent
        nJ = L - w2.recent - w2.n_sink
        sel = np.full((1, w2.Hkv, L), -1, np.int32)
        sel[0, :, :nJ] = np.arange(w2.n_sink, w2.n_sink + nJ)
        nsel = np.full((1, w2.Hkv), nJ, np.int32)
        got = r2.fast(q, sel, nsel, rs, ctx)
        check_out(got, oracle.dense(q, w2.K, w2.V, ctx))
        # and the slow step with budget >= |J| returns exactly J
        _, s, n = r2.slow(q, ctx, L)
        assert (n == nJ).all() and (s[0, :, :nJ] == sel[0, :, :nJ]).all() and (s[0, :, nJ:] == -1).all()
    finally:
        r2.close()


@pytest.mark.parametrize("Hq,Hkv", [(2, 2), (10, 2), (14, 2), (16, 2), (18, 2), (12, 1), (16, 1), (32, 2)])
def test_group_sizes(oracle, Hq, Hkv):
    """G = 1, 5, 7, 8, 9, 12, 16 (and 16 again with more KV heads): the fast-step kernels change their K-row
    layout between groups of 8 and 9 heads."""
    w = syn.make_tiny(L0=777, steps=2, budget=50, recent=32, n_support=8, B=1, Hq=Hq, Hkv=Hkv)
    r = Runner(w)
    try:
        _step(f"group size G={Hq // Hkv}")
        q = w.q(0)
        ctx = w.ctx_len(0)
        out, sel, nsel = r.slow(q, ctx, w.budget)
        check_out(out, oracle.dense(q, w.K, w.V, ctx))
        sel_ref, nsel_ref, z = oracle.selector(q, w.K, ctx, w.budget, w.n_sink, w.recent)
        check_selection(sel, nsel, sel_ref, nsel_ref, z, ctx, w.n_sink, w.recent, w.budget)
        q1 = w.q(1)
        got = r.fast(q1, sel, nsel, w.recent_start(1), w.ctx_len(1))
        check_out(got, oracle.sparse(q1, w.K, w.V, sel, nsel, w.recent_start(1), w.ctx_len(1), w.n_sink))
    finally:
        r.close()


def test_exact_ties_take_lower_index(oracle):
    """Duplicated key rows give bit-identical scores on both sides: the lower position must win."""
    w = syn.make_tiny(L0=600, steps=1, budget=40, recent=32, n_support=1, B=1)
    base = w.K[0, :, 100].copy()
    for j in range(100, 400):            # 300 identical rows -> one huge tie class
        w.K[0, :, j] = base
    r = Runner(w)
    try:
        _step("exact ties")
        q = w.q(0)
        ctx = w.ctx_len(0)
        _, sel, nsel = r.slow(q, ctx, w.budget)
        sel_ref, nsel_ref, z = oracle.selector(q, w.K, ctx, w.budget, w.n_sink, w.recent)
        for h in range(w.Hkv):
            got = sel[0, h, :nsel[0, h]]
            tied = got[(got >= 100) & (got < 400)]
            if len(tied):                # whichever of the tie class is taken, it is its lowest positions
                assert tied.tolist() == list(range(100, 100 + len(tied)))
            assert (z[0, h, 100:400] == z[0, h, 100]).all()
    finally:
        r.close()


def test_all_equal_scores(oracle):
    """K == 0: every score equals 1/|J|; the selected set is the first `budget` positions of J."""
    w = syn.make_tiny(L0=5000, steps=1, budget=300, recent=64, n_support=1, B=1)
    w.K[:] = 0
    r = Runner(w)
    try:
        _step("all-equal scores")
        q = w.q(0)
        out, sel, nsel = r.slow(q, w.ctx_len(0), w.budget)
        assert (nsel == 300).all()
        for h in range(w.Hkv):
            assert sel[0, h].tolist() == list(range(w.n_sink, w.n_sink + 300))
        check_out(out, oracle.dense(q, w.K, w.V, w.ctx_len(0)))
    finally:
        r.close()


def test_mixed_step_and_advance(oracle):
    import torch
    import paper_2603_12038_amd as sfi

    w = syn.make_serving(steps=4, B=5, Hq=16, Hkv=2, len_lo=300, len_hi=1400, budget=64, recent=32)
    r = Runner(w)
    try:
        _step("mixed step: all slow, then a mix")
        B = w.B
        ctx_d, rs_d = i32_dev(w.ctx_len(0)), i32_dev(w.recent_start(0))
        sel_d = torch.full((B, w.Hkv, w.budget), -7, dtype=torch.int32, device="cuda")
        nsel_d = torch.full((B, w.Hkv), -7, dtype=torch.int32, device="cuda")
        slow0 = torch.ones(B, dtype=torch.uint8, device="cuda")
        q0 = w.q(0)
        sfi.sfi_mixed_step(r.ctx.handle, to_dev(q0), r.K, r.V, slow0, ctx_d, rs_d, 0, w.budget, r.out, sel_d, nsel_d)
        torch.cuda.synchronize()
        ctx0 = w.ctx_len(0)
        check_out(r.out.cpu().numpy(), oracle.dense(q0, w.K, w.V, ctx0))
        sel_ref, nsel_ref, z = oracle.selector(q0, w.K, ctx0, w.budget, w.n_sink, w.recent)
        sel0, nsel0 = sel_d.cpu().numpy(), nsel_d.cpu().numpy()
        check_selection(sel0, nsel0, sel_ref, nsel_ref, z, ctx0, w.n_sink, w.recent, w.budget)

        sfi.sfi_advance(r.ctx.handle, ctx_d, rs_d)
        torch.cuda.synchronize()
        ctx_o, rs_o = oracle.advance(ctx0, w.recent_start(0), w.n_sink, w.recent)   # the oracle's state update
        assert (ctx_d.cpu().numpy() == ctx_o).all() and (rs_d.cpu().numpy() == rs_o).all()

        slow1 = np.array([0, 1, 0, 0, 1], np.uint8)
        q1 = w.q(1)
        ctx1, rs1 = w.ctx_len(1), w.recent_start(1)
        sfi.sfi_mixed_step(r.ctx.handle, to_dev(q1), r.K, r.V, torch.from_numpy(slow1).cuda(), ctx_d, rs_d, 0,
                           w.budget, r.out, sel_d, nsel_d)
        torch.cuda.synchronize()
        got = r.out.cpu().numpy()
        ref_dense = oracle.dense(q1, w.K, w.V, ctx1)
        ref_sparse = oracle.sparse(q1, w.K, w.V, sel0, nsel0, rs1, ctx1, w.n_sink)
        sel1, nsel1 = sel_d.cpu().numpy(), nsel_d.cpu().numpy()
        sel_ref1, nsel_ref1, z1 = oracle.selector(q1, w.K, ctx1, w.budget, w.n_sink, w.recent)
        for b in range(B):
            if slow1[b]:
                check_out(got[b], ref_dense[b])
                check_selection(sel1[b:b + 1], nsel1[b:b + 1], sel_ref1[b:b + 1], nsel_ref1[b:b + 1], z1[b:b + 1],
                                ctx1[b:b + 1], w.n_sink, w.recent, w.budget)
            else:
                check_out(got[b], ref_sparse[b])
                assert (sel1[b] == sel0[b]).all() and (nsel1[b] == nsel0[b]).all()   # frozen on fast steps
    finally:
        r.close()


def test_tiny_config_all_steps(oracle):
    """Config 1 as stated: 16 steps, slow at t = 0 and 8, the state carried on the device from step to step
    (sfi_advance), every step checked against the oracle's Algorithm 1 driver: outputs, the state each step ran
    on and the index sets after it."""
    import torch
    import paper_2603_12038_amd as sfi

    w = syn.make_tiny()
    qs = np.stack([w.q(t) for t in range(w.steps)])
    ref = oracle.decode_loop(qs, w.K, w.V, w.ctx_len(0), w.recent_start(0), w.slow.astype(np.uint8), w.budget, w.n_sink,
                             w.recent)
    r = Runner(w)
    try:
        ctx_d, rs_d = i32_dev(w.ctx_len(0)), i32_dev(w.recent_start(0))
        sel_d = torch.full((w.B, w.Hkv, w.budget), -7, dtype=torch.int32, device="cuda")
        nsel_d = torch.zeros((w.B, w.Hkv), dtype=torch.int32, device="cuda")
        for t in range(w.steps):
            _step(f"tiny config step {t} ({'slow' if w.slow[t, 0] else 'fast'})")
            q = qs[t]
            assert (ctx_d.cpu().numpy() == ref["ctx_hist"][t]).all() and (rs_d.cpu().numpy() == ref["rs_hist"][t]).all()
            if w.slow[t, 0]:
                sfi.sfi_slow_step(r.ctx.handle, to_dev(q), r.K, r.V, ctx_d, 0, w.budget, r.out, sel_d, nsel_d)
                torch.cuda.synchronize()
                ctx = ref["ctx_hist"][t]
                _, _, z = oracle.selector(q, w.K, ctx, w.budget, w.n_sink, w.recent)
                check_selection(sel_d.cpu().numpy(), nsel_d.cpu().numpy(), ref["sel_hist"][t], ref["nsel_hist"][t], z, ctx,
                                w.n_sink, w.recent, w.budget)
                # the fast steps that follow are compared on the oracle's set: the two must carry the same one
                assert (sel_d.cpu().numpy() == ref["sel_hist"][t]).all(), "a near-tie at the cut: pick another seed"
            else:
                sfi.sfi_fast_step(r.ctx.handle, to_dev(q), r.K, r.V, sel_d, nsel_d, w.budget, rs_d, ctx_d, r.out)
                torch.cuda.synchronize()
                assert (sel_d.cpu().numpy() == ref["sel_hist"][t]).all()     # Eq. freeze_sel
            check_out(r.out.cpu().numpy(), ref["out"][t])
            sfi.sfi_advance(r.ctx.handle, ctx_d, rs_d)
        torch.cuda.synchronize()
        assert (ctx_d.cpu().numpy() == ref["ctx_len"]).all() and (rs_d.cpu().numpy() == ref["recent_start"]).all()
    finally:
        r.close()


def test_results_are_deterministic(tiny):
    w, r = tiny
    _step("determinism")
    q = w.q(0)
    a = r.slow(q, w.ctx_len(0), w.budget)
    b = r.slow(q, w.ctx_len(0), w.budget)
    for x, y in zip(a, b):
        assert (x.view(np.uint32) == y.view(np.uint32)).all() if x.dtype == np.float32 else (x == y).all()


@pytest.mark.parametrize("recent", [20, 700])
def test_fast_step_without_selected_rows(oracle, recent):
    """Index lists of width 0 (sink + recent window only, sel_idx = NULL): the one-tile kernel and, with a long
    window, the pipelined one, which reads its indices ahead of the list length."""
    import torch
    w = syn.make_tiny(L0=2500, steps=2, budget=8, recent=recent, n_support=4, B=2)
    w.L0 = np.array([2500, 1300], np.int32)
    r = Runner(w)
    try:
        _step(f"fast step with sel_stride 0, recent {recent}")
        q, ctx, rs = w.q(1), w.ctx_len(1), w.recent_start(1)
        nsel = np.zeros((w.B, w.Hkv), np.int32)
        sel = np.zeros((w.B, w.Hkv, 0), np.int32)
        ref = oracle.sparse(q, w.K, w.V, sel, nsel, rs, ctx, w.n_sink)
        for tpw in (0, 1, 3):
            r.sfi.sfi_set_tuning(r.ctx.handle, 0, tpw if tpw else -1)
            r.out.fill_(float("nan"))
            r.sfi.sfi_fast_step(r.ctx.handle, to_dev(q), r.K, r.V, None, i32_dev(nsel), 0, i32_dev(rs), i32_dev(ctx), r.out)
            torch.cuda.synchronize()
            check_out(r.out.cpu().numpy(), ref)
        assert r.sfi.sfi_device_status(r.ctx.handle) == 0
    finally:
        r.close()


def test_interleaved_kv_layout(oracle):
    """K and V in one tensor [B, Hkv, L, 2, d] (row t: k_t then v_t), handed over as two base pointers 256 bytes
    apart with a row stride of 2 d: slow step, both fast-step launch shapes, reorg + compact fast step."""
    import torch

    w = syn.make_tiny(L0=3000, steps=2, budget=96, recent=48, n_support=8, B=2)
    w.L0 = np.array([3000, 1777], np.int32)
    r = Runner(w)
    try:
        _step("interleaved K/V layout")
        kv = torch.empty(w.B, w.Hkv, w.L_alloc, 2, w.d, dtype=torch.bfloat16, device="cuda")
        kv[:, :, :, 0], kv[:, :, :, 1] = r.K, r.V
        r.ctx.close()
        r.K, r.V = kv[:, :, :, 0], kv[:, :, :, 1]
        r.ctx = r.sfi.SfiContext(w.B, w.Hq, w.Hkv, r.max_ctx, w.budget, w.n_sink, w.recent, r.K, r.V)
        q0, ctx0 = w.q(0), w.ctx_len(0)
        out, sel, nsel = r.slow(q0, ctx0, w.budget)
        check_out(out, oracle.dense(q0, w.K, w.V, ctx0))
        sel_ref, nsel_ref, z = oracle.selector(q0, w.K, ctx0, w.budget, w.n_sink, w.recent)
        check_selection(sel, nsel, sel_ref, nsel_ref, z, ctx0, w.n_sink, w.recent, w.budget)
        q1, ctx1, rs1 = w.q(1), w.ctx_len(1), w.recent_start(1)
        ref = oracle.sparse(q1, w.K, w.V, sel, nsel, rs1, ctx1, w.n_sink)
        for tpw in (1, 3):
            r.sfi.sfi_set_tuning(r.ctx.handle, 0, tpw)
            check_out(r.fast(q1, sel, nsel, rs1, ctx1), ref)
        r.reorg(sel, nsel, ctx0)
        check_out(r.fast_compact(q1, nsel, sel.shape[2], rs1, ctx1), ref)
    finally:
        r.close()


def test_strided_kv_layout(oracle):
    """Token-major K/V storage ([B, L, Hkv, d]) through the stride fields."""
    import torch
    import paper_2603_12038_amd as sfi

    w = syn.make_tiny(L0=400, steps=1, budget=32, recent=16, n_support=4, B=2)
    _step("strided layout")
    Kt = to_dev(np.ascontiguousarray(w.K.transpose(0, 2, 1, 3))).permute(0, 2, 1, 3)
    Vt = to_dev(np.ascontiguousarray(w.V.transpose(0, 2, 1, 3))).permute(0, 2, 1, 3)
    ctx = sfi.SfiContext(w.B, w.Hq, w.Hkv, w.L_alloc, w.budget, w.n_sink, w.recent, Kt, Vt)
    try:
        out = torch.zeros(w.B, w.Hq, w.d, dtype=torch.float32, device="cuda")
        q = w.q(0)
        sfi.sfi_dense_attn(ctx.handle, to_dev(q), Kt, Vt, i32_dev(w.ctx_len(0)), 0, out)
        torch.cuda.synchronize()
        check_out(out.cpu().numpy(), oracle.dense(q, w.K, w.V, w.ctx_len(0)))
    finally:
        ctx.close()


@pytest.mark.parametrize("Hq,Hkv,L0", [(16, 2, 5000), (16, 1, 3000), (8, 2, 9000)])
def test_slow_step_with_few_splits(oracle, Hq, Hkv, L0):
    """One split per (sequence, KV head): a wave owns far more tiles than its logits stash holds
    (G = 8: 16 tiles, G = 16: 8, G = 4: 32), so the stash is written out several times on the way."""
    w = syn.make_tiny(L0=L0, steps=1, budget=96, recent=40, n_support=8, B=1, Hq=Hq, Hkv=Hkv)
    r = Runner(w)
    try:
        _step(f"few splits G={Hq // Hkv} L={L0}")
        r.sfi.sfi_set_tuning(r.ctx.handle, 1, 1)
        q, ctx = w.q(0), w.ctx_len(0)
        out, sel, nsel = r.slow(q, ctx, w.budget)
        assert r.sfi.sfi_query_splits(r.ctx.handle)[0] == 1
        check_out(out, oracle.dense(q, w.K, w.V, ctx))
        sel_ref, nsel_ref, z = oracle.selector(q, w.K, ctx, w.budget, w.n_sink, w.recent)
        check_selection(sel, nsel, sel_ref, nsel_ref, z, ctx, w.n_sink, w.recent, w.budget)
    finally:
        r.close()


def test_reorg_and_compact_fast_step(oracle, tiny):
    """Reorg is a byte copy: compact buffers bit-exact against the oracle's, untouched rows keep their
    poison (a NaN pattern, which the compact kernel must mask).  The two-segment fast step then matches
    the oracle's sparse attention on the original cache, over several steps of a sliding recent window."""
    w, r = tiny
    _step("reorg + compact fast step, Selector's own selection")
    q0, ctx = w.q(0), w.ctx_len(0)
    _, sel, nsel = r.slow(q0, ctx, w.budget)
    Kc, Vc = r.reorg(sel, nsel, ctx)
    Kc_ref, Vc_ref = np.full_like(Kc, 0x7FC1), np.full_like(Vc, 0x7FC1)
    oracle.reorg(w.K, w.V, sel, nsel, ctx, w.n_sink, Kc_ref, Vc_ref)
    assert (Kc == Kc_ref).all() and (Vc == Vc_ref).all()
    for t in range(1, 4):
        q = w.q(t)
        ctx_t, rs = w.ctx_len(t), w.recent_start(t)
        got = r.fast_compact(q, nsel, sel.shape[2], rs, ctx_t)
        check_out(got, oracle.sparse(q, w.K, w.V, sel, nsel, rs, ctx_t, w.n_sink))


def test_compact_random_sets_and_edges(oracle, tiny):
    """Arbitrary valid index sets, ragged n_sel (full budget, tile multiples, 0, 1), contexts down to one row,
    compact buffers larger than needed."""
    w, r = tiny
    q = w.q(5)
    cases = [(1500, 96), (1500, 0), (1500, 1), (1500, 28), (1500, 60), (300, 33), (70, 2), (68, 0), (5, 0), (3, 0), (1, 0)]
    for case, (L, ns) in enumerate(cases):
        _step(f"compact random sets L={L} n_sel={ns}")
        ctx = np.array([L, max(1, L - 2)], np.int32)
        rs = np.maximum(np.minimum(w.n_sink, ctx), ctx - w.recent).astype(np.int32)
        room = np.maximum(0, rs - w.n_sink)
        nsel = np.minimum(ns, room)[:, None].repeat(w.Hkv, axis=1).astype(np.int32)
        nsel[1, 0] = max(0, nsel[1, 0] - 1)
        sel = syn.random_sel(200 + case, w.B, w.Hkv, w.budget, nsel, w.n_sink, rs)
        Kc, Vc = r.reorg(sel, nsel, ctx, c_rows=w.n_sink + w.budget + (case % 3) * 7)
        Kc_ref, Vc_ref = np.full_like(Kc, 0x7FC1), np.full_like(Vc, 0x7FC1)
        oracle.reorg(w.K, w.V, sel, nsel, ctx, w.n_sink, Kc_ref, Vc_ref)
        assert (Kc == Kc_ref).all() and (Vc == Vc_ref).all()
        got = r.fast_compact(q, nsel, w.budget, rs, ctx)
        check_out(got, oracle.sparse(q, w.K, w.V, sel, nsel, rs, ctx, w.n_sink))


def test_compact_long_recent_window_and_groups(oracle):
    """G = 8 and a caller-chosen recent window longer than cfg.recent (extra trips of the tile loop)."""
    w = syn.make_tiny(L0=900, steps=2, budget=64, recent=32, n_support=8, B=1, Hq=16, Hkv=2)
    r = Runner(w)
    try:
        _step("compact: long recent window, G=8")
        q, ctx = w.q(0), w.ctx_len(0)
        _, sel, nsel = r.slow(q, ctx, w.budget)
        r.reorg(sel, nsel, ctx)
        q1, ctx1 = w.q(1), w.ctx_len(1)
        for rs in (w.recent_start(1), ctx1 - 700, ctx1 - 1, ctx1):
            rs = np.asarray(rs, np.int32).reshape(1)
            keep = [sel[0, h, :nsel[0, h]][sel[0, h, :nsel[0, h]] < rs[0]] for h in range(w.Hkv)]
            n2 = np.array([[len(k) for k in keep]], np.int32)
            s2 = np.full_like(sel, -1)
            for h, k in enumerate(keep):
                s2[0, h, :len(k)] = k
            r.reorg(s2, n2, ctx1)
            got = r.fast_compact(q1, n2, sel.shape[2], rs, ctx1)
            check_out(got, oracle.sparse(q1, w.K, w.V, s2, n2, rs, ctx1, w.n_sink))
    finally:
        r.close()


def test_reorg_only_slow_sequences(oracle, tiny):
    """With is_slow given, sequences whose flag is 0 keep their compact rows."""
    w, r = tiny
    _step("reorg predicate")
    ctx = w.ctx_len(0)
    rs = w.recent_start(0)
    nsel = np.full((w.B, w.Hkv), 40, np.int32)
    sel = syn.random_sel(77, w.B, w.Hkv, w.budget, nsel, w.n_sink, rs)
    Kc, Vc = r.reorg(sel, nsel, ctx, is_slow=[0, 1])
    Kc_ref, Vc_ref = np.full_like(Kc, 0x7FC1), np.full_like(Vc, 0x7FC1)
    oracle.reorg(w.K, w.V, sel, nsel, ctx, w.n_sink, Kc_ref, Vc_ref)
    assert (Kc[0] == 0x7FC1).all() and (Vc[0] == 0x7FC1).all()
    assert (Kc[1] == Kc_ref[1]).all() and (Vc[1] == Vc_ref[1]).all()


def test_slow_step_halves_on_two_streams(oracle, tiny):
    """sfi_slow_attn on one stream and sfi_slow_select on another, a ring of two contexts over four
    'layers' (different queries), ordered by events only: same bits as sfi_slow_step layer by layer."""
    import torch
    import paper_2603_12038_amd as sfi

    w, r = tiny
    _step("slow step halves on two streams")
    ctx = w.ctx_len(0)
    ctx_d = i32_dev(ctx)
    qs = [w.q(t) for t in range(4)]
    ref = [r.slow(q, ctx, w.budget) for q in qs]
    ring = [sfi.SfiContext(w.B, w.Hq, w.Hkv, r.max_ctx, w.budget, w.n_sink, w.recent, r.K, r.V) for _ in range(2)]
    try:
        main, aux = torch.cuda.Stream(), torch.cuda.Stream()
        outs = [torch.zeros(w.B, w.Hq, w.d, dtype=torch.float32, device="cuda") for _ in qs]
        sels = [torch.full((w.B, w.Hkv, w.budget), -7, dtype=torch.int32, device="cuda") for _ in qs]
        nsels = [torch.full((w.B, w.Hkv), -7, dtype=torch.int32, device="cuda") for _ in qs]
        q_d = [to_dev(q) for q in qs]
        torch.cuda.synchronize()
        free = [None, None]
        for l in range(4):
            slot = l % 2
            if free[slot] is not None:
                main.wait_event(free[slot])
            sfi.sfi_slow_attn(ring[slot].handle, q_d[l], r.K, r.V, ctx_d, 0, outs[l], stream=main)
            done = torch.cuda.Event()
            done.record(main)
            aux.wait_event(done)
            sfi.sfi_slow_select(ring[slot].handle, ctx_d, 0, w.budget, sels[l], nsels[l], stream=aux)
            free[slot] = torch.cuda.Event()
            free[slot].record(aux)
        torch.cuda.synchronize()
        for l in range(4):
            o, s, n = ref[l]
            assert (outs[l].cpu().numpy().view(np.uint32) == o.view(np.uint32)).all()
            assert (sels[l].cpu().numpy() == s).all() and (nsels[l].cpu().numpy() == n).all()
    finally:
        for c in ring:
            c.close()


@pytest.mark.parametrize("tpw", [2, 3, 7, 40])
def test_fast_step_pipelined_gather(oracle, tiny, tpw):
    """The pipelined gather kernel (several tiles per wave, forced through the tuning knob): the Selector's
    own sets, arbitrary sets, ragged n_sel, and lists shorter than one tile."""
    w, r = tiny
    _step(f"pipelined gather, {tpw} tiles per wave")
    r.sfi.sfi_set_tuning(r.ctx.handle, 0, tpw)
    try:
        q0, ctx = w.q(0), w.ctx_len(0)
        _, sel, nsel = r.slow(q0, ctx, w.budget)
        for t in range(1, 3):
            q, ctx_t, rs = w.q(t), w.ctx_len(t), w.recent_start(t)
            got = r.fast(q, sel, nsel, rs, ctx_t)
            check_out(got, oracle.sparse(q, w.K, w.V, sel, nsel, rs, ctx_t, w.n_sink))
        q = w.q(5)
        for case, (L, ns) in enumerate([(1500, 96), (1500, 0), (1500, 1), (300, 33), (70, 2), (5, 0), (1, 0)]):
            ctx = np.array([L, max(1, L - 2)], np.int32)
            rs = np.maximum(np.minimum(w.n_sink, ctx), ctx - w.recent).astype(np.int32)
            room = np.maximum(0, rs - w.n_sink)
            nsel2 = np.minimum(ns, room)[:, None].repeat(w.Hkv, axis=1).astype(np.int32)
            nsel2[1, 0] = max(0, nsel2[1, 0] - 1)
            sel2 = syn.random_sel(300 + case, w.B, w.Hkv, w.budget, nsel2, w.n_sink, rs)
            got = r.fast(q, sel2, nsel2, rs, ctx)
            check_out(got, oracle.sparse(q, w.K, w.V, sel2, nsel2, rs, ctx, w.n_sink))
    finally:
        r.sfi.sfi_set_tuning(r.ctx.handle, 0, -1)


def test_trigger_policy_on_device(oracle, tiny):
    """sfi_trigger step by step against the oracle's schedule, one request per batch row (different
    token streams), tokens outside the vocabulary included."""
    import torch

    w, r = tiny
    _step("trigger policy")
    vocab, t_max, n = 1000, 9, 120
    trig = [3, 64, 65, 999]
    bitmap = np.zeros((vocab + 31) // 32, np.uint32)
    for i in trig:
        bitmap[i >> 5] |= np.uint32(1 << (i & 31))
    rng = syn.rng_for(11, 555)
    toks = rng.integers(-2, vocab + 40, size=(n, w.B)).astype(np.int32)
    toks[rng.random((n, w.B)) < 0.08] = 64
    ref = np.stack([oracle.trigger_schedule(toks[:, b], trig, t_max) for b in range(w.B)], axis=1)
    bm_d = torch.from_numpy(bitmap.view(np.int32)).cuda()
    since = torch.full((w.B,), t_max, dtype=torch.int32, device="cuda")
    flag = torch.zeros(w.B, dtype=torch.uint8, device="cuda")
    got = np.zeros((n, w.B), np.uint8)
    last = torch.zeros(w.B, dtype=torch.int32, device="cuda")  # step 0 is slow through since_slow = t_max
    for t in range(n):
        r.sfi.sfi_trigger(r.ctx.handle, last, bm_d, vocab, t_max, since, flag)
        got[t] = flag.cpu().numpy()
        last = torch.from_numpy(toks[t]).cuda()
    assert (got == ref).all()


@pytest.mark.parametrize("recent,n_sink,splits", [(1500, 4, 1), (1500, 70, 0), (700, 33, 1), (2900, 4, 0)])
def test_long_recent_window_and_sink(oracle, recent, n_sink, splits):
    """Sink + recent rows spanning many tiles (several such tiles per wave when the split is forced to one
    workgroup per pair), a sink longer than a tile, and a recent window that leaves almost no J."""
    w = syn.make_tiny(L0=3000, steps=2, budget=80, recent=recent, n_support=8, B=2, Hq=8, Hkv=2)
    w.n_sink = n_sink
    w.L0 = np.array([3000, 1777], np.int32)
    r = Runner(w)
    try:
        _step(f"long recent window R={recent} sink={n_sink} splits={'forced 1' if splits else 'default'}")
        if splits:
            r.sfi.sfi_set_tuning(r.ctx.handle, 1, 1)
        q, ctx = w.q(0), w.ctx_len(0)
        out, sel, nsel = r.slow(q, ctx, w.budget)
        check_out(out, oracle.dense(q, w.K, w.V, ctx))
        sel_ref, nsel_ref, z = oracle.selector(q, w.K, ctx, w.budget, w.n_sink, w.recent)
        check_selection(sel, nsel, sel_ref, nsel_ref, z, ctx, w.n_sink, w.recent, w.budget)
        q1, ctx1, rs1 = w.q(1), w.ctx_len(1), w.recent_start(1)
        got = r.fast(q1, sel, nsel, rs1, ctx1)
        check_out(got, oracle.sparse(q1, w.K, w.V, sel, nsel, rs1, ctx1, w.n_sink))
        Kc, Vc = r.reorg(sel, nsel, ctx)
        got = r.fast_compact(q1, nsel, sel.shape[2], rs1, ctx1)
        check_out(got, oracle.sparse(q1, w.K, w.V, sel, nsel, rs1, ctx1, w.n_sink))
    finally:
        r.close()


@pytest.mark.parametrize("scale", [1.0, 0.35, 0.004])
def test_logit_scales_far_from_default(oracle, scale):
    """The config's logit scale: 1.0 makes the softmax nearly one-hot (logits of several hundred in the log2
    domain, most weights underflow to 0), 0.004 makes it nearly uniform."""
    w = syn.make_tiny(L0=2200, steps=2, budget=64, recent=48, n_support=12, B=2, Hq=8, Hkv=2)
    r = Runner(w, scale=scale)
    try:
        _step(f"logit scale {scale}")
        q, ctx = w.q(0), w.ctx_len(0)
        out, sel, nsel = r.slow(q, ctx, w.budget)
        check_out(out, oracle.dense(q, w.K, w.V, ctx, scale=scale))
        sel_ref, nsel_ref, z = oracle.selector(q, w.K, ctx, w.budget, w.n_sink, w.recent, scale=scale)
        check_selection(sel, nsel, sel_ref, nsel_ref, z, ctx, w.n_sink, w.recent, w.budget)
        q1, ctx1, rs1 = w.q(1), w.ctx_len(1), w.recent_start(1)
        got = r.fast(q1, sel, nsel, rs1, ctx1)
        check_out(got, oracle.sparse(q1, w.K, w.V, sel, nsel, rs1, ctx1, w.n_sink, scale=scale))
    finally:
        r.close()


@pytest.mark.parametrize("merge", [1, 2])
def test_fast_step_merge_in_kernel_and_in_its_own_launch(oracle, tiny, merge):
    """Both ways of merging a fast step's split records, on calls in a row whose lists differ in length
    (the number of workgroups per pair changes from call to call; the arrival counters of the in-kernel
    merge must come back to zero every time)."""
    w, r = tiny
    r.sfi.sfi_set_tuning(r.ctx.handle, 0, 0, merge)
    try:
        q = w.q(6)
        for case, (L, ns) in enumerate([(1500, 96), (1500, 3), (700, 40), (1500, 96), (69, 1), (1200, 64)]):
            _step(f"fast merge mode {merge}: L={L} n_sel={ns}")
            ctx = np.array([L, max(1, L - 5)], np.int32)
            rs = np.maximum(np.minimum(w.n_sink, ctx), ctx - w.recent).astype(np.int32)
            room = np.maximum(0, rs - w.n_sink)
            nsel = np.minimum(ns, room)[:, None].repeat(w.Hkv, axis=1).astype(np.int32)
            sel = syn.random_sel(500 + case, w.B, w.Hkv, max(ns, 1), nsel, w.n_sink, rs)
            got = r.fast(q, sel, nsel, rs, ctx)
            check_out(got, oracle.sparse(q, w.K, w.V, sel, nsel, rs, ctx, w.n_sink))
            assert r.sfi.sfi_query_splits(r.ctx.handle)[1] >= 1
        # the compact path shares the merge
        q0, ctx0 = w.q(0), w.ctx_len(0)
        _, sel, nsel = r.slow(q0, ctx0, w.budget)
        r.reorg(sel, nsel, ctx0)
        for t in range(1, 3):
            qt, ctx_t, rs = w.q(t), w.ctx_len(t), w.recent_start(t)
            got = r.fast_compact(qt, nsel, sel.shape[2], rs, ctx_t)
            check_out(got, oracle.sparse(qt, w.K, w.V, sel, nsel, rs, ctx_t, w.n_sink))
    finally:
        r.sfi.sfi_set_tuning(r.ctx.handle, 0, 0, 1)


@pytest.mark.parametrize("Hq,Hkv", [(4, 1), (6, 2), (16, 1)])
def test_fast_step_many_split_workgroups(oracle, Hq, Hkv):
    """Long index lists over one or two (b, h) pairs: 10, 24, 32 and 63 (the cap) split workgroups per pair, so
    the in-kernel merge walks its records in several groups of eight, the last one ragged; G = 4, 3 and 16
    (two rounds of output threads).  The last list is shorter again: the arrival counters must be back at zero."""
    w = syn.make_tiny(L0=9000, steps=1, budget=8100, recent=64, n_support=8, B=1, Hq=Hq, Hkv=Hkv)
    r = Runner(w)
    try:
        r.sfi.sfi_set_tuning(r.ctx.handle, 0, 1)  # one tile per wave: as many workgroups as the list has tiles for
        q, ctx, rs = w.q(0), w.ctx_len(0), w.recent_start(0)
        for case, (ns, want) in enumerate([(1100, 10), (3000, 24), (4000, 32), (8100, 63), (300, 3)]):
            _step(f"fast step with {want} split workgroups per pair, G={Hq // Hkv}")
            nsel = np.full((w.B, w.Hkv), ns, np.int32)
            nsel[0, -1] = ns - 7
            sel = syn.random_sel(700 + case, w.B, w.Hkv, ns, nsel, w.n_sink, rs)
            got = r.fast(q, sel, nsel, rs, ctx)
            assert r.sfi.sfi_query_splits(r.ctx.handle)[1] == want
            check_out(got, oracle.sparse(q, w.K, w.V, sel, nsel, rs, ctx, w.n_sink))
    finally:
        r.close()


def test_graph_replays_match_eager_runs(oracle):
    """One refresh segment (slow step, state update, three fast steps with state updates) captured into
    a HIP graph and replayed three times, with eager work of the library and synchronisations between the
    replays: every replay must leave the bits the eager run left (outputs of all four steps, index sets,
    state), and the eager run matches the oracle.  Sizes give split launches, so the in-kernel merge and
    its arrival counters are part of what is replayed."""
    import torch
    w = syn.make_tiny(L0=6000, steps=4, budget=700, recent=64, n_support=16, B=2)
    w.L0 = np.array([6000, 4321], np.int32)
    r = Runner(w)
    try:
        sfi, h, t = r.sfi, r.ctx.handle, torch
        qs = [to_dev(w.q(i)) for i in range(4)]
        outs = [t.zeros(w.B, w.Hq, w.d, dtype=t.float32, device="cuda") for _ in range(4)]
        sel = t.full((w.B, w.Hkv, w.budget), -7, dtype=t.int32, device="cuda")
        nsel = t.full((w.B, w.Hkv), -7, dtype=t.int32, device="cuda")
        ctx0, rs0 = i32_dev(w.ctx_len(0)), i32_dev(w.recent_start(0))
        ctx_d, rs_d = ctx0.clone(), rs0.clone()

        def segment():
            sfi.sfi_slow_step(h, qs[0], r.K, r.V, ctx_d, r.max_ctx, w.budget, outs[0], sel, nsel)
            sfi.sfi_advance(h, ctx_d, rs_d)
            for i in range(1, 4):
                sfi.sfi_fast_step(h, qs[i], r.K, r.V, sel, nsel, w.budget, rs_d, ctx_d, outs[i])
                sfi.sfi_advance(h, ctx_d, rs_d)

        def reset():
            ctx_d.copy_(ctx0)
            rs_d.copy_(rs0)
            for o in outs:
                o.fill_(float("nan"))
            sel.fill_(-7)
            nsel.fill_(-7)

        _step("graph test: eager segment")
        reset()
        segment()
        t.cuda.synchronize()
        assert sfi.sfi_query_splits(h)[1] > 1
        ref = [o.clone() for o in outs] + [sel.clone(), nsel.clone(), ctx_d.clone(), rs_d.clone()]
        check_out(ref[0].cpu().numpy(), oracle.dense(w.q(0), w.K, w.V, w.ctx_len(0)))
        sel_np, nsel_np = ref[4].cpu().numpy(), ref[5].cpu().numpy()
        for i in range(1, 4):
            check_out(ref[i].cpu().numpy(),
                      oracle.sparse(w.q(i), w.K, w.V, sel_np, nsel_np, w.recent_start(i), w.ctx_len(i), w.n_sink))

        _step("graph test: capture")
        reset()
        t.cuda.synchronize()
        side = t.cuda.Stream()  # default priority
        side.wait_stream(t.cuda.current_stream())
        graph = t.cuda.CUDAGraph()
        with t.cuda.stream(side):
            graph.capture_begin()
            segment()
            graph.capture_end()
        t.cuda.current_stream().wait_stream(side)
        t.cuda.synchronize()
        assert t.equal(ctx_d, ctx0), "capture must not execute anything"

        other_q = to_dev(w.q(2))
        for rep in range(3):
            _step(f"graph test: replay {rep}")
            reset()
            graph.replay()
            t.cuda.synchronize()
            got = outs + [sel, nsel, ctx_d, rs_d]
            for k, (g_, r_) in enumerate(zip(got, ref)):
                assert t.equal(g_, r_), f"replay {rep}: tensor {k} differs from the eager run"
            # eager work of the library between the replays (same context, same workspace)
            r.dense(w.q(3), w.ctx_len(1))
            sfi.sfi_fast_step(h, other_q, r.K, r.V, sel, nsel, w.budget, rs0, ctx0, r.out)
            t.cuda.synchronize()
    finally:
        r.close()


def test_context_on_a_dirty_workspace(oracle, tiny):
    """sfi_create must not rely on what the workspace holds: a workspace of 0xFF bytes gives the same split
    fast step (in-kernel merge, arrival counters) and the same slow step as a fresh one."""
    import torch
    w, r = tiny
    sfi = r.sfi
    cfg = r.ctx.cfg
    nbytes = sfi.sfi_workspace_bytes(cfg)
    ws = torch.full((nbytes,), 0xFF, dtype=torch.uint8, device="cuda")
    h = sfi.sfi_create(cfg, ws, nbytes)
    try:
        q0, ctx0 = w.q(0), w.ctx_len(0)
        out_ref, sel, nsel = r.slow(q0, ctx0, w.budget)
        q1, ctx1, rs1 = w.q(1), w.ctx_len(1), w.recent_start(1)
        fast_ref = r.fast(q1, sel, nsel, rs1, ctx1)
        assert sfi.sfi_query_splits(r.ctx.handle)[1] > 1
        out = torch.full((w.B, w.Hq, w.d), float("nan"), dtype=torch.float32, device="cuda")
        sel_d = torch.full((w.B, w.Hkv, w.budget), -7, dtype=torch.int32, device="cuda")
        nsel_d = torch.full((w.B, w.Hkv), -7, dtype=torch.int32, device="cuda")
        sfi.sfi_fast_step(h, to_dev(q1), r.K, r.V, i32_dev(sel), i32_dev(nsel), w.budget, i32_dev(rs1), i32_dev(ctx1), out)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), fast_ref)
        sfi.sfi_slow_step(h, to_dev(q0), r.K, r.V, i32_dev(ctx0), r.max_ctx, w.budget, out, sel_d, nsel_d)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), out_ref)
        assert np.array_equal(sel_d.cpu().numpy(), sel) and np.array_equal(nsel_d.cpu().numpy(), nsel)
    finally:
        sfi.sfi_destroy(h)


@pytest.mark.parametrize("n_sink,L", [(33, 23), (70, 10), (70, 69), (33, 33), (4, 2)])
def test_context_shorter_than_the_sink(oracle, n_sink, L):
    """ctx_len <= n_sink: every row is a sink row, nothing is selected, the recent window is empty
    (sfi_advance leaves recent_start = n_sink > ctx_len).  Slow step, fast step and the compact fast step,
    whose buffers were filled before the last rows were appended."""
    w = syn.make_tiny(L0=200, steps=3, budget=16, recent=8, n_support=4, B=2, Hq=6, Hkv=2)
    w.n_sink = n_sink
    w.L0 = np.array([L, max(1, L - 3)], np.int32)
    r = Runner(w)
    try:
        _step(f"context inside the sink: n_sink={n_sink} L={L}")
        q0, c0 = w.q(0), w.ctx_len(0)
        out, sel, nsel = r.slow(q0, c0, w.budget)
        check_out(out, oracle.dense(q0, w.K, w.V, c0))
        assert (nsel == 0).all() and (sel == -1).all()
        r.reorg(sel, nsel, c0)
        for t in (1, 2):
            q, ct, rt = w.q(t), w.ctx_len(t), w.recent_start(t)
            if (ct > n_sink).any():
                break  # the sink has filled up: the next step has to be a slow one for the compact path
            ref = oracle.sparse(q, w.K, w.V, sel, nsel, rt, ct, w.n_sink)
            check_out(r.fast(q, sel, nsel, rt, ct), ref)
            check_out(r.fast_compact(q, nsel, sel.shape[2], rt, ct), ref)
    finally:
        r.close()


def test_selector_twice_on_the_same_evidence(oracle, tiny):
    """sfi_slow_attn once, sfi_slow_select twice with two budgets: the second pass must not count into the first
    pass's histogram and candidate list."""
    import torch
    import paper_2603_12038_amd as sfi

    w, r = tiny
    _step("two Selector passes over one evidence")
    q, ctx = w.q(0), w.ctx_len(0)
    ctx_d = i32_dev(ctx)
    r.out.fill_(float("nan"))
    sfi.sfi_slow_attn(r.ctx.handle, to_dev(q), r.K, r.V, ctx_d, 0, r.out)
    for budget in (w.budget, w.budget // 3, w.budget):
        sel = torch.full((w.B, w.Hkv, budget), -7, dtype=torch.int32, device="cuda")
        nsel = torch.full((w.B, w.Hkv), -7, dtype=torch.int32, device="cuda")
        sfi.sfi_slow_select(r.ctx.handle, ctx_d, 0, budget, sel, nsel)
        torch.cuda.synchronize()
        sel_ref, nsel_ref, z = oracle.selector(q, w.K, ctx, budget, w.n_sink, w.recent)
        check_selection(sel.cpu().numpy(), nsel.cpu().numpy(), sel_ref, nsel_ref, z, ctx, w.n_sink, w.recent, budget)
    check_out(r.out.cpu().numpy(), oracle.dense(q, w.K, w.V, ctx))
    assert r.sfi.sfi_device_status(r.ctx.handle) == 0


@pytest.mark.parametrize("path", ["gather", "compact"])
def test_ragged_decode_loop_against_the_oracles_driver(oracle, path):
    """Algorithm 1 for five ragged sequences with their own slow/fast schedules, twelve steps, all state on the device
    (sfi_mixed_step or sfi_mixed_step_compact + sfi_advance), against the oracle's driver: outputs of every step, the
    state each step ran on, the index sets after it.  On the compact path the buffers of a sequence are refilled only
    by its own slow steps; poison in the untouched rows would show in the outputs."""
    import torch
    import paper_2603_12038_amd as sfi

    w = syn.make_serving(steps=12, B=5, Hq=16, Hkv=2, len_lo=300, len_hi=1400, budget=64, recent=32, mean_gap=4.0)
    T = w.steps
    g = w.slow.astype(np.uint8)
    assert g[0].all() and 0 < g[1:].sum() < g[1:].size
    qs = np.stack([w.q(t) for t in range(T)])
    ref = oracle.decode_loop(qs, w.K, w.V, w.ctx_len(0), w.recent_start(0), g, w.budget, w.n_sink, w.recent)
    r = Runner(w)
    try:
        B = w.B
        ctx_d, rs_d = i32_dev(w.ctx_len(0)), i32_dev(w.recent_start(0))
        sel_d = torch.full((B, w.Hkv, w.budget), -7, dtype=torch.int32, device="cuda")
        nsel_d = torch.zeros((B, w.Hkv), dtype=torch.int32, device="cuda")
        c_rows = w.n_sink + w.budget
        Kc = to_dev(np.full((B, w.Hkv, c_rows, w.d), 0x7FC1, np.uint16))
        Vc = to_dev(np.full((B, w.Hkv, c_rows, w.d), 0x7FC1, np.uint16))
        for t in range(T):
            _step(f"ragged decode loop ({path}) step {t}: slow {g[t].tolist()}")
            flags = torch.from_numpy(g[t]).cuda()
            assert (ctx_d.cpu().numpy() == ref["ctx_hist"][t]).all() and (rs_d.cpu().numpy() == ref["rs_hist"][t]).all()
            r.out.fill_(float("nan"))
            if path == "compact":
                sfi.sfi_mixed_step_compact(r.ctx.handle, to_dev(qs[t]), r.K, r.V, flags, ctx_d, rs_d, 0, w.budget, r.out, sel_d,
                                           nsel_d, Kc, Vc)
            else:
                sfi.sfi_mixed_step(r.ctx.handle, to_dev(qs[t]), r.K, r.V, flags, ctx_d, rs_d, 0, w.budget, r.out, sel_d, nsel_d)
            torch.cuda.synchronize()
            check_out(r.out.cpu().numpy(), ref["out"][t])
            assert (sel_d.cpu().numpy() == ref["sel_hist"][t]).all() and (nsel_d.cpu().numpy() == ref["nsel_hist"][t]).all()
            sfi.sfi_advance(r.ctx.handle, ctx_d, rs_d)
        torch.cuda.synchronize()
        assert (ctx_d.cpu().numpy() == ref["ctx_len"]).all() and (rs_d.cpu().numpy() == ref["recent_start"]).all()
        assert r.sfi.sfi_device_status(r.ctx.handle) == 0
    finally:
        r.close()


def test_decode_loop_from_the_packed_descriptor(oracle):
    """Algorithm 1 driven by the packed per-step descriptor alone: sfi_step_begin (state update + trigger policy, one
    launch per decoding step) and sfi_mixed_step_desc (every kernel reads the descriptor) for three ragged sequences
    over fourteen steps, no host decision in between.  Expected: the oracle's trigger schedule per sequence fed to the
    oracle's Algorithm 1 driver."""
    import torch
    import paper_2603_12038_amd as sfi

    w = syn.make_serving(steps=14, B=3, Hq=8, Hkv=2, len_lo=400, len_hi=1200, budget=48, recent=24)
    T, B, t_max, vocab = w.steps, w.B, 4, 300
    trig = [7, 31, 64, 250]
    rng = syn.rng_for(5, 4242)
    tokens = rng.integers(0, 40, size=(T, B)).astype(np.int32)   # tokens[t, b]: generated by step t
    g = np.stack([oracle.trigger_schedule(tokens[:, b], trig, t_max) for b in range(B)], axis=1)
    assert g[0].all() and 0 < g[1:].sum() < g[1:].size
    qs = np.stack([w.q(t) for t in range(T)])
    ref = oracle.decode_loop(qs, w.K, w.V, w.ctx_len(0), w.recent_start(0), g, w.budget, w.n_sink, w.recent)
    bitmap = np.zeros((vocab + 31) // 32, np.uint32)
    for i in trig:
        bitmap[i >> 5] |= np.uint32(1 << (i & 31))
    r = Runner(w)
    try:
        _step("decode loop from the packed descriptor")
        desc0 = np.zeros((B, 4), np.int32)
        desc0[:, 0] = w.ctx_len(0)
        desc0[:, 1] = -99            # filled in by sfi_step_begin
        desc0[:, 3] = t_max          # g_0 = 1
        desc = torch.from_numpy(desc0).cuda()
        bm = torch.from_numpy(bitmap.view(np.int32)).cuda()
        sel_d = torch.full((B, w.Hkv, w.budget), -7, dtype=torch.int32, device="cuda")
        nsel_d = torch.zeros((B, w.Hkv), dtype=torch.int32, device="cuda")
        last = torch.zeros(B, dtype=torch.int32, device="cuda")
        for t in range(T):
            sfi.sfi_step_begin(r.ctx.handle, desc, last if t > 0 else None, bm, vocab, t_max, t > 0)
            r.out.fill_(float("nan"))
            sfi.sfi_mixed_step_desc(r.ctx.handle, to_dev(qs[t]), r.K, r.V, desc, 0, w.budget, r.out, sel_d, nsel_d)
            torch.cuda.synchronize()
            d = desc.cpu().numpy()
            assert (d[:, 0] == ref["ctx_hist"][t]).all() and (d[:, 1] == ref["rs_hist"][t]).all() and (d[:, 2] == g[t]).all()
            check_out(r.out.cpu().numpy(), ref["out"][t])
            assert (sel_d.cpu().numpy() == ref["sel_hist"][t]).all() and (nsel_d.cpu().numpy() == ref["nsel_hist"][t]).all()
            last = torch.from_numpy(tokens[t]).cuda()
        assert r.sfi.sfi_device_status(r.ctx.handle) == 0
    finally:
        r.close()


def test_dense_kernel_with_whole_line_k_loads(oracle, tiny):
    """The dense kernel's other K layout (sfi_set_dense_k_layout: whole 128-byte lines, halves joined by lane
    exchanges): same outputs within the tolerance, same index sets."""
    w, r = tiny
    _step("dense kernel, whole-line K loads")
    q, ctx = w.q(0), w.ctx_len(0)
    ref_out, ref_sel, ref_nsel = r.slow(q, ctx, w.budget)
    r.sfi.sfi_set_dense_k_layout(r.ctx.handle, True)
    try:
        out, sel, nsel = r.slow(q, ctx, w.budget)
        check_out(out, oracle.dense(q, w.K, w.V, ctx))
        sel_o, nsel_o, z = oracle.selector(q, w.K, ctx, w.budget, w.n_sink, w.recent)
        check_selection(sel, nsel, sel_o, nsel_o, z, ctx, w.n_sink, w.recent, w.budget)
        assert (sel == ref_sel).all() and (nsel == ref_nsel).all()
        for L in (1, 5, 37, 70, 1000):
            c = np.array([L, max(1, L // 3)], np.int32)
            check_out(r.dense(q, c), oracle.dense(q, w.K, w.V, c))
    finally:
        r.sfi.sfi_set_dense_k_layout(r.ctx.handle, False)


def test_measurement_skeletons_run_and_leave_the_path_alone(oracle, tiny):
    """The memory skeletons bench.py times next to the kernels (sfi_fast_step_floor, sfi_dense_attn_floor) take the same
    arguments as the launches they mirror, refuse variants that are not defined, and leave nothing behind that a
    following real step could trip over: a slow step and a fast step after them still match the oracle."""
    import torch
    w, r = tiny
    _step("measurement skeletons")
    sfi, h = r.sfi, r.ctx.handle
    q, ctx = w.q(0), w.ctx_len(0)
    out0, sel, nsel = r.slow(q, ctx, w.budget)
    q_d, ctx_d, rs_d = to_dev(w.q(1)), i32_dev(w.ctx_len(1)), i32_dev(w.recent_start(1))
    sel_d, nsel_d = i32_dev(sel), i32_dev(nsel)
    scratch_out = torch.zeros_like(r.out)
    for v in (0, 1, 2, 4, 8):
        sfi.sfi_fast_step_floor(h, q_d, r.K, r.V, sel_d, nsel_d, sel.shape[2], rs_d, ctx_d, scratch_out, v)
    for v in (0, 1, 16 * 4, 16 * 4 + 1, 2048, 4096 + 16 * 2 + 1):
        sfi.sfi_dense_attn_floor(h, r.K, r.V, ctx_d, 0, v)
    torch.cuda.synchronize()
    for v in (3, 5, 12, 16, -1):
        with pytest.raises(sfi.SfiError):
            sfi.sfi_fast_step_floor(h, q_d, r.K, r.V, sel_d, nsel_d, sel.shape[2], rs_d, ctx_d, scratch_out, v)
    for v in (2, 15, 16 * 65, 3 * 2048, -1):
        with pytest.raises(sfi.SfiError):
            sfi.sfi_dense_attn_floor(h, r.K, r.V, ctx_d, 0, v)
    assert sfi.sfi_device_status(h) == 0
    got = r.fast(w.q(1), sel, nsel, w.recent_start(1), w.ctx_len(1))
    check_out(got, oracle.sparse(w.q(1), w.K, w.V, sel, nsel, w.recent_start(1), w.ctx_len(1), w.n_sink))
    out1, sel1, nsel1 = r.slow(q, ctx, w.budget)
    assert (sel1 == sel).all() and (nsel1 == nsel).all()
    check_out(out1, oracle.dense(q, w.K, w.V, ctx))


@pytest.mark.parametrize("case", ["random", "ties", "all_equal"])
def test_top_k_over_several_segments(oracle, case):
    """Top-K (Eq. topk_out) where a (sequence, KV head) pair spans several 2048-position segments of the Selector's
    launches, with ragged lengths: random scores, a tie class that spans two segments and is larger than a segment, and
    all scores equal.  Several budgets on the same evidence, from 1 to more than |J|."""
    w = syn.make_tiny(L0=9000, steps=1, budget=700, recent=64, n_support=24, B=2)
    w.L0 = np.array([9000, 4300], np.int32)
    if case == "ties":
        for j in range(3000, 5200):
            w.K[:, :, j] = w.K[:, :, 3000]
    if case == "all_equal":
        w.K[:] = 0
    r = Runner(w, max_budget=9000)
    try:
        _step(f"top-k over several segments, {case}")
        q, ctx = w.q(0), w.ctx_len(0)
        for budget in (700, 1, 64, 2500, 9000):
            sel_o, nsel_o, z = oracle.selector(q, w.K, ctx, budget, w.n_sink, w.recent)
            _, sel, nsel = r.slow(q, ctx, budget)
            check_selection(sel, nsel, sel_o, nsel_o, z, ctx, w.n_sink, w.recent, budget)
            if case == "all_equal":
                for b in range(w.B):
                    k = int(nsel[b, 0])
                    assert sel[b, 0, :k].tolist() == list(range(w.n_sink, w.n_sink + k))
        assert r.sfi.sfi_device_status(r.ctx.handle) == 0
    finally:
        r.close()


@pytest.mark.parametrize("paged", [False, True])
def test_ragged_step_planned_on_the_device(oracle, paged):
    """sfi_mixed_step's dense launch plans itself on the device (sfi_set_mixed_plan, default): the slow sequences and
    their splits by length.  Eleven ragged sequences from empty to the whole cache, every kind of mix -- none slow, one (the
    longest, the shortest, an empty one), several, all -- against the oracle per sequence, and bit for bit against
    the launch with one workgroup per cell of the batch (same records in other slots, merged in a fixed order: the
    outputs may differ in the last bits, the index sets may not)."""
    import torch
    import paper_2603_12038_amd as sfi

    w = syn.make_serving(steps=2, B=11, Hq=16, Hkv=2, len_lo=300, len_hi=9000, budget=96, recent=32)
    w.L0 = np.array([int(w.L_alloc) - 4, 0, 33, 4100, 36, 1500, 7000, 5, 610, 0, 2800], np.int32)
    r = Runner(w, page_size=16 if paged else 0)
    try:
        B, h = w.B, r.ctx.handle
        ctx0, rs0 = w.ctx_len(0), w.recent_start(0)
        ctx_d, rs_d = i32_dev(ctx0), i32_dev(rs0)
        q0 = w.q(0)
        sel_d = torch.full((B, w.Hkv, w.budget), -7, dtype=torch.int32, device="cuda")
        nsel_d = torch.full((B, w.Hkv), -7, dtype=torch.int32, device="cuda")
        ones = torch.ones(B, dtype=torch.uint8, device="cuda")
        _step(f"ragged step planned on the device (paged={paged}): all slow")
        sfi.sfi_mixed_step(h, to_dev(q0), r.K, r.V, ones, ctx_d, rs_d, 0, w.budget, r.out, sel_d, nsel_d)
        torch.cuda.synchronize()
        sel0, nsel0 = sel_d.cpu().numpy().copy(), nsel_d.cpu().numpy().copy()
        ref_dense = oracle.dense(q0, w.K, w.V, ctx0)
        check_out(r.out.float().cpu().numpy(), ref_dense)
        sel_ref, nsel_ref, z = oracle.selector(q0, w.K, ctx0, w.budget, w.n_sink, w.recent)
        check_selection(sel0, nsel0, sel_ref, nsel_ref, z, ctx0, w.n_sink, w.recent, w.budget)
        ref_sparse = oracle.sparse(q0, w.K, w.V, sel0, nsel0, rs0, ctx0, w.n_sink)
        mixes = [[], [0], [2], [1], [7, 9], [0, 6], [3, 5, 8, 10], [0, 1, 2, 3, 4], list(range(B))]
        for mix in mixes:
            _step(f"ragged step planned on the device (paged={paged}): slow {mix}")
            fl = np.zeros(B, np.uint8)
            fl[mix] = 1
            got = {}
            for plan in (1, 0):
                sfi.sfi_set_mixed_plan(h, plan)
                sel_d.copy_(torch.from_numpy(sel0)); nsel_d.copy_(torch.from_numpy(nsel0))
                r.out.fill_(float("nan"))
                sfi.sfi_mixed_step(h, to_dev(q0), r.K, r.V, torch.from_numpy(fl).cuda(), ctx_d, rs_d, 0, w.budget, r.out, sel_d, nsel_d)
                torch.cuda.synchronize()
                got[plan] = (r.out.float().cpu().numpy().copy(), sel_d.cpu().numpy().copy(), nsel_d.cpu().numpy().copy())
            out, sel, nsel = got[1]
            for b in range(B):
                check_out(out[b], ref_dense[b] if fl[b] else ref_sparse[b])
            assert (sel == got[0][1]).all() and (nsel == got[0][2]).all()
            assert (sel == sel0).all() and (nsel == nsel0).all()   # the same evidence: the same sets, slow or frozen
            np.testing.assert_allclose(out, got[0][0], rtol=0, atol=2e-3 * max(1e-30, float(np.abs(ref_dense).max())))
        assert sfi.sfi_device_status(h) == 0
        with pytest.raises(sfi.SfiError):
            sfi.sfi_set_mixed_plan(h, 2)
    finally:
        sfi.sfi_set_mixed_plan(r.ctx.handle, 1)
        r.close()
