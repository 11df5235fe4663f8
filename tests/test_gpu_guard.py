"""Device-side inputs out of range: the kernels clamp lengths, counts, stored indices and block ids before they
address memory and report what they clamped through sfi_device_status.  Every case here stays inside the
buffers by construction of those clamps; the expected output is the run on the host-clamped input, bit for bit
(same launch geometry, same arithmetic)."""
import numpy as np
import pytest

import sfi_synth as syn
from helpers import Runner, check_out

pytestmark = pytest.mark.gpu

CTX_LEN, N_SEL, SEL_IDX, BLOCK = 1, 2, 4, 8


def _step(msg):
    print(f"[gpu-guard] {msg}", flush=True)


def _status(r, clear=True):
    return r.sfi.sfi_device_status(r.ctx.handle, clear)


def test_clean_inputs_raise_nothing(oracle):
    """Slow step, fast steps in both launch shapes, reorg and the compact fast step on legal inputs, the last
    sequence empty: the status word stays 0."""
    w = syn.make_tiny(L0=3000, steps=4, budget=96, recent=64, n_support=16, B=3)
    w.L0 = np.array([3000, 1100, 0], np.int32)
    r = Runner(w)
    try:
        assert _status(r) == 0
        _step("clean: slow step")
        q0, ctx = w.q(0), w.ctx_len(0)
        out, sel, nsel = r.slow(q0, ctx, w.budget)
        check_out(out[:2], oracle.dense(q0, w.K, w.V, ctx)[:2])
        assert (nsel[2] == 0).all() and not out[2].any()
        for tpw in (1, 3):
            _step(f"clean: fast step, {tpw} tiles per wave")
            r.sfi.sfi_set_tuning(r.ctx.handle, 0, tpw)
            q, ctx_t, rs = w.q(1), w.ctx_len(1), w.recent_start(1)
            ctx_t[2], rs[2] = 0, 0
            r.fast(q, sel, nsel, rs, ctx_t)
        _step("clean: reorg + compact fast step")
        r.reorg(sel, nsel, ctx)
        r.fast_compact(q, nsel, sel.shape[2], rs, ctx_t)
        assert _status(r) == 0
    finally:
        r.close()


FULL = dict(gamma=0.5, beta=1.0, p=2.0, eta=0.5, lambda_clip=0.9, alpha_soft=0.5, alpha_cross=0.3, temp=1.0,
            eps=1e-8, nms_radius=2)


@pytest.mark.parametrize("selector", [None, FULL], ids=["evidence", "full"])
def test_ctx_len_out_of_range_is_clamped_and_reported(selector):
    """ctx_len above max_len reads as max_len, a negative one as 0, in the dense kernel, the merge and every
    Selector kernel alike."""
    w = syn.make_tiny(L0=2600, steps=2, budget=80, recent=48, n_support=8, B=3)
    r = Runner(w, selector=selector)
    try:
        ml = 2500
        q = w.q(0)
        bad = np.array([ml + 777, -5, 1 << 30], np.int32)
        ok = np.array([ml, 0, ml], np.int32)
        _step(f"ctx_len out of range, selector mode {0 if selector is None else 1}: clamped reference run")
        out_ok, sel_ok, nsel_ok = r.slow(q, ok, w.budget, max_len=ml)
        assert _status(r) == 0
        _step("ctx_len out of range: slow step")
        out, sel, nsel = r.slow(q, bad, w.budget, max_len=ml)
        assert _status(r, clear=False) == CTX_LEN
        assert _status(r) == CTX_LEN and _status(r) == 0  # read twice, cleared by the second read
        assert np.array_equal(out, out_ok) and np.array_equal(sel, sel_ok) and np.array_equal(nsel, nsel_ok)
        _step("ctx_len out of range: dense attention alone")
        d_ok = r.dense(q, ok, max_len=ml)
        d = r.dense(q, bad, max_len=ml)
        assert _status(r) == CTX_LEN and np.array_equal(d, d_ok)
        _step("ctx_len out of range: fast step (bound: max_ctx)")
        cap = r.max_ctx
        rs = np.array([cap - w.recent, 0, cap - w.recent], np.int32)
        f_ok = r.fast(q, sel_ok, nsel_ok, rs, np.array([cap, 0, cap], np.int32))
        f = r.fast(q, sel_ok, nsel_ok, rs, np.array([cap + 1, -1, 1 << 30], np.int32))
        assert _status(r) == CTX_LEN and np.array_equal(f, f_ok)
    finally:
        r.close()


@pytest.mark.parametrize("tpw", [1, 3])
def test_stored_indices_and_counts_out_of_range(tpw):
    """sel_idx entries outside the context are read as its last row, n_sel outside [0, sel_stride] as the nearest
    bound; padding entries are never looked at."""
    w = syn.make_tiny(L0=2200, steps=2, budget=96, recent=64, n_support=8, B=2)
    r = Runner(w)
    try:
        r.sfi.sfi_set_tuning(r.ctx.handle, 0, tpw)
        q0, ctx = w.q(0), w.ctx_len(0)
        _, sel, nsel = r.slow(q0, ctx, w.budget)
        assert _status(r) == 0 and (nsel == w.budget).all()
        q, ctx_t, rs = w.q(1), w.ctx_len(1), w.recent_start(1)
        bad_sel = sel.copy()
        bad_sel[0, 0, 3], bad_sel[0, 1, 17], bad_sel[1, 0, 95], bad_sel[1, 1, 0] = -5, 1 << 30, int(ctx_t[1]), -(1 << 31)
        last = np.broadcast_to(ctx_t[:, None, None] - 1, bad_sel.shape)
        ok_sel = np.where((bad_sel < 0) | (bad_sel > last), last, bad_sel).astype(np.int32)  # what the header says
        _step(f"bad stored indices, {tpw} tiles per wave")
        f_ok = r.fast(q, ok_sel, nsel, rs, ctx_t)
        assert _status(r) == 0
        f = r.fast(q, bad_sel, nsel, rs, ctx_t)
        assert _status(r) == SEL_IDX and np.array_equal(f, f_ok)
        _step("bad stored indices: reorg")
        Kc_ok, Vc_ok = r.reorg(ok_sel, nsel, ctx_t)
        assert _status(r) == 0
        Kc, Vc = r.reorg(bad_sel, nsel, ctx_t)
        assert _status(r) == SEL_IDX and np.array_equal(Kc, Kc_ok) and np.array_equal(Vc, Vc_ok)
        _step("bad counts")
        bad_n = nsel.copy()
        bad_n[0, 0], bad_n[1, 1] = w.budget + 1000, -3
        ok_n = np.clip(bad_n, 0, w.budget).astype(np.int32)
        f_ok = r.fast(q, sel, ok_n, rs, ctx_t)
        f = r.fast(q, sel, bad_n, rs, ctx_t)
        assert _status(r) == N_SEL and np.array_equal(f, f_ok)
        c_ok = r.fast_compact(q, ok_n, sel.shape[2], rs, ctx_t)
        c = r.fast_compact(q, bad_n, sel.shape[2], rs, ctx_t)
        assert _status(r) == N_SEL and np.array_equal(c, c_ok)
        _step("padding entries past n_sel are not looked at")
        short_n = np.minimum(nsel, 40).astype(np.int32)
        junk = sel.copy()
        junk[:, :, 40:] = 1 << 29
        f_ok = r.fast(q, sel, short_n, rs, ctx_t)
        f = r.fast(q, junk, short_n, rs, ctx_t)
        assert _status(r) == 0 and np.array_equal(f, f_ok)
    finally:
        r.close()


def test_block_ids_out_of_range():
    """A block id outside the pool among the entries that cover a context is read as the nearest block of the
    pool; entries past the context are never read."""
    w = syn.make_tiny(L0=1500, steps=2, budget=64, recent=48, n_support=8, B=2)
    r = Runner(w, page_size=16)
    try:
        t = r.torch
        for pool in (r.K, r.V):  # the spare blocks' NaN pattern -> 1.0: whatever block a clamp lands on is finite
            bits = pool.view(t.int16)
            bits[bits == 0x7FC1] = 0x3F80
        n_blocks = int(r.K.shape[0])
        q0, q = w.q(0), w.q(1)
        ctx = np.array([1190, 900], np.int32)
        ctx_t = ctx + 1
        rs = np.maximum(w.n_sink, ctx_t - w.recent).astype(np.int32)
        used = (ctx_t + 15) // 16
        _step("bad block ids: reference run")
        out0, sel, nsel = r.slow(q0, ctx, w.budget)
        assert _status(r) == 0
        table = r.table.cpu().numpy().copy()
        for b in range(2):
            table[b, used[b]:] = 1 << 28  # past the context: never read
        r.table.copy_(t.from_numpy(table))
        out1, sel1, nsel1 = r.slow(q0, ctx, w.budget)
        assert _status(r) == 0 and np.array_equal(out1, out0) and np.array_equal(sel1, sel)
        bad = table.copy()
        bad[0, 5], bad[1, 11], bad[1, 40] = n_blocks + 12345, -1, 1 << 30
        ok = bad.copy()
        ok[0, 5], ok[1, 11], ok[1, 40] = n_blocks - 1, 0, n_blocks - 1
        results = []
        for name, tbl in (("clamped on the host", ok), ("left to the kernels", bad)):
            _step(f"bad block ids: {name}")
            r.table.copy_(t.from_numpy(tbl))
            t.cuda.synchronize()
            got = [r.slow(q0, ctx, w.budget)]
            st = [_status(r)]
            r.sfi.sfi_set_tuning(r.ctx.handle, 0, 1)
            got.append(r.fast(q, sel, nsel, rs, ctx_t))
            st.append(_status(r))
            r.sfi.sfi_set_tuning(r.ctx.handle, 0, 3)
            got.append(r.fast(q, sel, nsel, rs, ctx_t))
            st.append(_status(r))
            got.append(r.reorg(sel, nsel, ctx_t))
            st.append(_status(r))
            got.append(r.fast_compact(q, nsel, sel.shape[2], rs, ctx_t))
            st.append(_status(r))
            results.append((got, st))
        (g_ok, st_ok), (g_bad, st_bad) = results
        assert st_ok == [0, 0, 0, 0, 0]
        # dense reads every row of both contexts; the sparse calls only report blocks they touch
        assert st_bad[0] == BLOCK and all(s in (0, BLOCK) for s in st_bad[1:])
        for a, b in zip(g_ok, g_bad):
            if isinstance(a, tuple):
                assert all(np.array_equal(x, y) for x, y in zip(a, b))
            else:
                assert np.array_equal(a, b) and np.isfinite(a).all()
    finally:
        r.close()
