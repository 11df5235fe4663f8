"""Comparison rules and device plumbing shared by the GPU parity tests, the smoke check and the benchmark's
parity sample: uploads, the output and index-set acceptance rules, one-call wrappers around the C ABI.

No arithmetic of the method lives here and nothing here imports the oracle: expected values are handed in by
the caller (who got them from the oracle), results come from libsfi.
"""
from __future__ import annotations

import numpy as np

OUT_TOL = 2e-3       # max relative error of an output row (bf16 in, fp32 accumulate)
TIE_BAND = 1e-5      # ranking-score gap below which several index sets are acceptable


def to_dev(bits: np.ndarray):
    """bf16 bit patterns (uint16) -> torch.bfloat16 tensor on the GPU, same bits."""
    import torch
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def i32_dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def row_rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max over rows of  max_c |got - ref| / max_c |ref|  (rows = last axis)."""
    num = np.abs(got.astype(np.float64) - ref).max(axis=-1)
    den = np.abs(ref).max(axis=-1)
    return float((num / np.maximum(den, 1e-30)).max())


def check_out_bf16(got, ref):
    """Outputs stored as bf16 (handed over widened to fp32): every element within one bf16 ulp of itself (the
    rounding, plus one ulp where the fp32 result sits next to a rounding boundary) plus 5e-5 of its row's
    largest magnitude (the fp32 path's own error, three times the largest observed) of the fp64 reference."""
    assert np.isfinite(got).all()
    rowmax = np.abs(ref).max(axis=-1, keepdims=True)
    err = np.abs(got.astype(np.float64) - ref)
    bound = np.abs(ref) * 2.0 ** -8 + 5e-5 * rowmax + 1e-30
    worst = float((err / bound).max())
    assert worst <= 1.0, f"bf16 output off by {worst:.3f} of its bound"
    assert np.array_equal(got.astype(np.float32).view(np.uint32) & 0xFFFF, np.zeros_like(got, np.uint32)), "not bf16 values"
    return worst


def check_out(got, ref, tol=OUT_TOL):
    assert np.isfinite(got).all()
    err = row_rel_err(got, ref)
    assert err <= tol, f"row-relative error {err:.3e} > {tol}"
    return err


def check_selection(sel, nsel, sel_ref, nsel_ref, z, ctx_len, n_sink, recent, budget, band=TIE_BAND):
    """Selected sets must equal the oracle's wherever the k-th and (k+1)-th ranking scores differ by
    more than TIE_BAND; inside the band any set whose members sit at or above the threshold (and whose
    non-members sit at or below it) within the band is valid.  Structure is always checked."""
    B, Hkv = nsel.shape
    n_exact = 0
    for b in range(B):
        L = int(ctx_len[b])
        lo, hi = n_sink, L - recent
        nJ = max(0, hi - lo)
        for h in range(Hkv):
            k = int(nsel[b, h])
            assert k == int(nsel_ref[b, h]) == min(budget, nJ)
            row = sel[b, h]
            assert (row[k:budget] == -1).all()
            got = row[:k]
            if k == 0:
                continue
            assert (np.diff(got) > 0).all(), "not ascending / not unique"
            assert got[0] >= lo and got[-1] < hi
            ref = sel_ref[b, h, :k]
            if k == nJ:
                assert (got == ref).all()
                n_exact += 1
                continue
            zz = z[b, h, lo:hi]
            part = np.partition(zz, nJ - k - 1)
            zk1, zk = part[nJ - k - 1], part[nJ - k:].min()
            if zk - zk1 > band:
                assert (got == ref).all(), f"selection differs at (b={b}, h={h}) with gap {zk - zk1:.2e}"
                n_exact += 1
            else:
                mask = np.zeros(nJ, bool)
                mask[got - lo] = True
                viol = max(zk - zz[mask].min(), zz[~mask].max() - zk)
                assert viol <= band, f"(b={b}, h={h}): a member / non-member sits {viol:.2e} on the wrong side of the cut"
                n_exact += int((got == ref).all())
    return n_exact


def make_paged(K: np.ndarray, V: np.ndarray, ctx_max: np.ndarray, page: int, seed: int, spare: int = 3, layout: str = "thd"):
    """Scatter flat caches [B, Hkv, L, d] into block pools [n_blocks, page, Hkv, d] through a random block
    table [B, pages].  Spare blocks, and the blocks of table entries wholly beyond ctx_max[b], hold a NaN
    pattern (a valid address, so a wrong lookup shows up as a wrong result, never as a fault)."""
    B, Hkv, L, d = K.shape
    pages = (L + page - 1) // page
    rng = np.random.default_rng(seed)
    n_blocks = B * pages + spare
    perm = rng.permutation(n_blocks)
    table = perm[:B * pages].reshape(B, pages).astype(np.int32)
    poison_block = int(perm[B * pages])
    Kp = np.full((n_blocks, page, Hkv, d), 0x7FC1, np.uint16)
    Vp = np.full((n_blocks, page, Hkv, d), 0x7FC1, np.uint16)
    for b in range(B):
        for i in range(pages):
            lo, hi = i * page, min(L, (i + 1) * page)
            if lo >= int(ctx_max[b]):
                table[b, i] = poison_block
                continue
            Kp[table[b, i], :hi - lo] = K[b, :, lo:hi].transpose(1, 0, 2)
            Vp[table[b, i], :hi - lo] = V[b, :, lo:hi].transpose(1, 0, 2)
    if layout == "htd":  # [n_blocks, Hkv, page, d]: a head's rows of a block are contiguous
        Kp, Vp = np.ascontiguousarray(Kp.transpose(0, 2, 1, 3)), np.ascontiguousarray(Vp.transpose(0, 2, 1, 3))
    return Kp, Vp, table


class Runner:
    """Device copies of one workload's K/V plus an sfi context; thin wrappers over the C-ABI calls."""

    def __init__(self, w, max_budget=None, selector=None, alpha=0.0, page_size=0, ctx_max=None, page_layout="thd",
                 scale=0.0, out_bf16=False):
        """page_size > 0: the cache is handed over as block pools + block table (valid up to ctx_max[b] rows,
        default every allocated row); self.K / self.V are then the pools."""
        import torch
        import paper_2603_12038_amd as sfi
        self.sfi, self.torch, self.w = sfi, torch, w
        self.max_ctx = int(w.L_alloc)
        if page_size:
            cm = np.full(w.B, w.L_alloc) if ctx_max is None else np.asarray(ctx_max)
            Kp, Vp, table = make_paged(w.K, w.V, cm, page_size, seed=page_size + 17, layout=page_layout)
            self.K, self.V = to_dev(Kp), to_dev(Vp)
            self.table = torch.from_numpy(table).cuda()
        else:
            self.K, self.V = to_dev(w.K), to_dev(w.V)
        self.ctx = sfi.SfiContext(w.B, w.Hq, w.Hkv, self.max_ctx, w.budget if max_budget is None else max_budget,
                                  w.n_sink, w.recent, self.K, self.V, scale=scale, selector=selector, alpha=alpha,
                                  page_size=page_size, page_layout=page_layout, out_bf16=out_bf16)
        if page_size:
            sfi.sfi_set_block_table(self.ctx.handle, self.table, self.K.shape[0])
        # with bf16 outputs the wrappers below return the values widened to fp32 (exact)
        self.out = torch.zeros(w.B, w.Hq, w.d, dtype=torch.bfloat16 if out_bf16 else torch.float32, device="cuda")

    def dense(self, q_bits, ctx_len, max_len=0):
        self.out.fill_(float("nan"))
        self.sfi.sfi_dense_attn(self.ctx.handle, to_dev(q_bits), self.K, self.V, i32_dev(ctx_len), max_len, self.out)
        self.torch.cuda.synchronize()
        return self.out.float().cpu().numpy()

    def slow(self, q_bits, ctx_len, budget, max_len=0):
        t = self.torch
        self.out.fill_(float("nan"))
        sel = t.full((self.w.B, self.w.Hkv, max(budget, 1)), -7, dtype=t.int32, device="cuda")
        nsel = t.full((self.w.B, self.w.Hkv), -7, dtype=t.int32, device="cuda")
        self.sfi.sfi_slow_step(self.ctx.handle, to_dev(q_bits), self.K, self.V, i32_dev(ctx_len), max_len, budget,
                               self.out, sel, nsel)
        t.cuda.synchronize()
        return self.out.float().cpu().numpy(), sel.cpu().numpy(), nsel.cpu().numpy()

    def fast(self, q_bits, sel, nsel, recent_start, ctx_len):
        self.out.fill_(float("nan"))
        sel_d, nsel_d = i32_dev(sel), i32_dev(nsel)
        self.sfi.sfi_fast_step(self.ctx.handle, to_dev(q_bits), self.K, self.V, sel_d, nsel_d, sel.shape[2],
                               i32_dev(recent_start), i32_dev(ctx_len), self.out)
        self.torch.cuda.synchronize()
        return self.out.float().cpu().numpy()

    def reorg(self, sel, nsel, ctx_len, c_rows=None, is_slow=None, poison=0x7FC1):
        """Compact buffers (uint16 views of bf16 device tensors) after sfi_reorg; unfilled rows keep `poison`."""
        t = self.torch
        c_rows = self.w.n_sink + sel.shape[2] if c_rows is None else c_rows
        shape = (self.w.B, self.w.Hkv, c_rows, self.w.d)
        self.Kc = to_dev(np.full(shape, poison, np.uint16))
        self.Vc = to_dev(np.full(shape, poison, np.uint16))
        self.sfi.sfi_reorg(self.ctx.handle, self.K, self.V, i32_dev(sel), i32_dev(nsel), sel.shape[2], i32_dev(ctx_len),
                           None if is_slow is None else t.from_numpy(np.asarray(is_slow, np.uint8)).cuda(),
                           self.Kc, self.Vc)
        t.cuda.synchronize()
        return self.Kc.view(t.int16).cpu().numpy().view(np.uint16), self.Vc.view(t.int16).cpu().numpy().view(np.uint16)

    def fast_compact(self, q_bits, nsel, sel_stride, recent_start, ctx_len):
        """Fast step over the compact buffers of the last reorg() call."""
        self.out.fill_(float("nan"))
        self.sfi.sfi_fast_step_compact(self.ctx.handle, to_dev(q_bits), self.Kc, self.Vc, i32_dev(nsel), sel_stride,
                                       self.K, self.V, i32_dev(recent_start), i32_dev(ctx_len), self.out)
        self.torch.cuda.synchronize()
        return self.out.float().cpu().numpy()

    def close(self):
        self.ctx.close()
