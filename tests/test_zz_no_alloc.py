"""The fast step on the library's static scratch (sfi_fast_step_static: no context, no workspace, no allocation)
against sfi_fast_step through the C ABI, and against the oracle, on two calls in a row, the second smaller."""
import numpy as np
import pytest

import sfi_synth as syn
from helpers import Runner, check_out, i32_dev, to_dev

pytestmark = pytest.mark.gpu


def _step(msg):
    print(f"[gpu-no-alloc] {msg}", flush=True)


def _case(oracle, w, n_sel_val, seed):
    """One fast step of workload w both ways; returns (static output, context output, planned splits)."""
    import torch
    import paper_2603_12038_amd as sfi

    r = Runner(w)
    try:
        ctx, rs = w.ctx_len(1), w.recent_start(1)
        q = w.q(1)
        nsel = np.full((w.B, w.Hkv), n_sel_val, np.int32)
        sel = syn.random_sel(seed, w.B, w.Hkv, w.budget, nsel, w.n_sink, rs)
        ref = r.fast(q, sel, nsel, rs, ctx)
        splits = r.sfi.sfi_query_splits(r.ctx.handle)[1]
        out = torch.full((w.B, w.Hq, w.d), float("nan"), dtype=torch.float32, device="cuda")
        sfi.sfi_fast_step_static(r.ctx.cfg, to_dev(q), r.K, r.V, i32_dev(sel), i32_dev(nsel), sel.shape[2], i32_dev(rs),
                                 i32_dev(ctx), out)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        check_out(got, oracle.sparse(q, w.K, w.V, sel, nsel, rs, ctx, w.n_sink))
        check_out(ref, oracle.sparse(q, w.K, w.V, sel, nsel, rs, ctx, w.n_sink))
        return got, ref, splits
    finally:
        r.close()


def test_static_scratch_fast_step_two_calls_second_smaller(oracle):
    # first call: several split workgroups per pair (records and arrival counters in use)
    w1 = syn.make_tiny(L0=6000, steps=2, budget=1536, recent=96, n_support=16, B=2, Hq=16, Hkv=4)
    _step(f"call 1: B={w1.B} Hq={w1.Hq} Hkv={w1.Hkv} budget={w1.budget}")
    got1, ref1, s1 = _case(oracle, w1, w1.budget - 3, 11)
    assert s1 > 1, "the first case is meant to split"
    assert np.array_equal(got1, ref1), "same launch plan, same arithmetic: bit-identical outputs expected"
    # second call, smaller in every dimension: fewer sequences, heads, rows, another group size
    w2 = syn.make_tiny(L0=900, steps=2, budget=200, recent=40, n_support=8, B=1, Hq=6, Hkv=2)
    _step(f"call 2: B={w2.B} Hq={w2.Hq} Hkv={w2.Hkv} budget={w2.budget}")
    got2, ref2, s2 = _case(oracle, w2, w2.budget, 12)
    assert np.array_equal(got2, ref2)
    # and the first shape once more: what the smaller call left in the scratch must not matter
    _step("call 3: the first shape again")
    got3, ref3, _ = _case(oracle, w1, w1.budget - 3, 11)
    assert np.array_equal(got3, got1) and np.array_equal(got3, ref3)


def test_static_scratch_limits_and_coarser_split(oracle):
    """A shape whose records would not fit the scratch at sfi_fast_step's split runs with a coarser one (equal within
    the output tolerance); shapes beyond the scratch are refused with SFI_EUNSUPPORTED before any launch."""
    import torch
    import paper_2603_12038_amd as sfi
    from paper_2603_12038_amd.binding import SfiConfig, SfiError

    # 6144 query heads leave room for one record per head; 384 pairs on 256 compute units make sfi_fast_step split in two
    w = syn.make_tiny(L0=2600, steps=2, budget=2048, recent=64, n_support=8, B=384, Hq=16, Hkv=1)
    _step(f"coarser split: B={w.B} Hq={w.Hq} Hkv={w.Hkv}")
    got, ref, splits = _case(oracle, w, w.budget, 13)
    room = 8192 // (w.B * w.Hq)
    _step(f"  sfi_fast_step planned {splits} workgroups per pair; the static scratch holds {room} record(s) per head")
    assert splits > room, "the case is meant to need more records than the scratch holds"
    check_out(got, ref.astype(np.float64))
    cfg = SfiConfig()
    cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim = 129, 64, 8, 128   # 8256 query heads > 8192
    cfg.max_ctx, cfg.max_budget, cfg.n_sink, cfg.recent = 256, 64, 4, 16
    cfg.k_stride_b = cfg.v_stride_b = 8 * 256 * 128
    cfg.k_stride_h = cfg.v_stride_h = 256 * 128
    cfg.k_stride_t = cfg.v_stride_t = 128
    dummy = torch.zeros(64, dtype=torch.int32, device="cuda")
    with pytest.raises(SfiError) as e:
        sfi.sfi_fast_step_static(cfg, dummy, dummy, dummy, dummy, dummy, 64, dummy, dummy, dummy)
    assert e.value.code == -2
    cfg.batch, cfg.page_size = 1, 16
    cfg.k_stride_b = cfg.v_stride_b = 0
    with pytest.raises(SfiError) as e:
        sfi.sfi_fast_step_static(cfg, dummy, dummy, dummy, dummy, dummy, 64, dummy, dummy, dummy)
    assert e.value.code == -2
