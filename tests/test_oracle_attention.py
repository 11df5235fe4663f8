"""Pins for the oracle's dense and sparse attention (CPU only).

Each test ties the oracle to something other than itself: a brute-force loop written
here from the textbook definition of softmax attention, closed forms, invariants,
or torch's fp64 SDPA on the CPU.
"""
import math
import struct

import numpy as np
import pytest

import sfi_synth as syn


def bf16_to_float(u: int) -> float:
    """Decode one bf16 bit pattern without numpy views (independent of the generator's helper)."""
    return struct.unpack("<f", struct.pack("<I", (int(u) & 0xFFFF) << 16))[0]


def rand_bf16(seed, shape):
    return syn.normal_bf16(syn.rng_for(seed, 99), shape)


def brute_attention(q, K, V, rows, scale):
    """softmax(scale * q.K[rows]) @ V[rows] with python floats; q [d], K/V [L, d] (bf16 bits)."""
    d = len(q)
    qf = [bf16_to_float(x) for x in q]
    ls = []
    for j in rows:
        ls.append(scale * sum(qf[c] * bf16_to_float(K[j][c]) for c in range(d)))
    m = max(ls)
    ws = [math.exp(l - m) for l in ls]
    tot = sum(ws)
    return [sum(w * bf16_to_float(V[j][c]) for w, j in zip(ws, rows)) / tot for c in range(d)]


@pytest.mark.parametrize("d", [1, 3, 4])
def test_dense_brute_force_tiny(oracle, d):
    B, Hq, Hkv, Lmax = 2, 4, 2, 16
    q = rand_bf16(1, (B, Hq, d))
    K = rand_bf16(2, (B, Hkv, Lmax, d))
    V = rand_bf16(3, (B, Hkv, Lmax, d))
    ctx = np.array([16, 11], np.int32)
    out = oracle.dense(q, K, V, ctx)
    G = Hq // Hkv
    for b in range(B):
        for g in range(Hq):
            ref = brute_attention(q[b, g], K[b, g // G], V[b, g // G], range(int(ctx[b])), 1.0 / math.sqrt(d))
            np.testing.assert_allclose(out[b, g], ref, rtol=1e-12, atol=1e-14)


def test_dense_matches_torch_sdpa_fp64(oracle):
    import torch

    B, Hq, Hkv, L, d = 2, 8, 2, 257, 128
    q = rand_bf16(4, (B, Hq, d))
    K = rand_bf16(5, (B, Hkv, L, d))
    V = rand_bf16(6, (B, Hkv, L, d))
    out = oracle.dense(q, K, V, np.full(B, L, np.int32))
    tq = torch.from_numpy(syn.bf16_bits_to_f32(q).astype(np.float64)).unsqueeze(2)          # [B,Hq,1,d]
    tk = torch.from_numpy(syn.bf16_bits_to_f32(K).astype(np.float64)).repeat_interleave(Hq // Hkv, dim=1)
    tv = torch.from_numpy(syn.bf16_bits_to_f32(V).astype(np.float64)).repeat_interleave(Hq // Hkv, dim=1)
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv).squeeze(2).numpy()
    np.testing.assert_allclose(out, ref, rtol=1e-11, atol=1e-13)


def test_dense_closed_forms(oracle):
    B, Hq, Hkv, L, d = 1, 4, 2, 50, 8
    q = rand_bf16(7, (B, Hq, d))
    K = rand_bf16(8, (B, Hkv, L, d))
    V = rand_bf16(9, (B, Hkv, L, d))
    one = syn.f32_to_bf16_bits(np.ones((B, Hkv, L, d), np.float32))
    # weights sum to one: V == 1 -> out == 1
    np.testing.assert_allclose(oracle.dense(q, K, one, [L]), 1.0, rtol=0, atol=1e-14)
    # a single row -> that row's value
    o1 = oracle.dense(q, K, V, [1])
    for g in range(Hq):
        np.testing.assert_allclose(o1[0, g], syn.bf16_bits_to_f32(V[0, g // 2, 0]), rtol=1e-15)
    # all keys zero -> uniform weights -> mean of V
    zero = np.zeros_like(K)
    om = oracle.dense(q, zero, V, [L])
    vf = syn.bf16_bits_to_f32(V).astype(np.float64)
    for g in range(Hq):
        np.testing.assert_allclose(om[0, g], vf[0, g // 2].mean(axis=0), rtol=1e-13, atol=1e-15)


def test_dense_shift_invariance_and_scale(oracle):
    """A component that adds the same constant to every logit leaves the output unchanged;
    the default scale is 1/sqrt(d)."""
    B, Hq, Hkv, L, d = 1, 2, 1, 40, 4
    q = rand_bf16(10, (B, Hq, d))
    K = rand_bf16(11, (B, Hkv, L, d))
    V = rand_bf16(12, (B, Hkv, L, d))
    base = oracle.dense(q, K, V, [L], scale=0.5)
    q2 = np.concatenate([q, syn.f32_to_bf16_bits(np.full((B, Hq, 1), 3.0, np.float32))], axis=2)
    K2 = np.concatenate([K, syn.f32_to_bf16_bits(np.full((B, Hkv, L, 1), -2.0, np.float32))], axis=3)
    V2 = np.concatenate([V, V[..., :1]], axis=3)
    shifted = oracle.dense(q2, K2, V2, [L], scale=0.5)
    np.testing.assert_allclose(shifted[..., :d], base, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(oracle.dense(q, K, V, [L]), oracle.dense(q, K, V, [L], scale=1.0 / math.sqrt(d)),
                               rtol=0, atol=0)


def test_dense_strided_layout(oracle):
    """K/V given as strided views (head-major vs token-major storage) give the same result."""
    B, Hq, Hkv, L, d = 2, 4, 2, 33, 8
    q = rand_bf16(13, (B, Hq, d))
    K = rand_bf16(14, (B, Hkv, L, d))
    V = rand_bf16(15, (B, Hkv, L, d))
    ref = oracle.dense(q, K, V, [L, L - 5])
    Kt = np.ascontiguousarray(K.transpose(0, 2, 1, 3)).transpose(0, 2, 1, 3)   # token-major storage
    Vpad = np.zeros((B, Hkv, L + 7, d + 8), np.uint16)
    Vpad[:, :, :L, :d] = V
    out = oracle.dense(q, Kt, Vpad[:, :, :L, :d], [L, L - 5])
    np.testing.assert_array_equal(out, ref)


def test_logits_brute(oracle):
    B, Hq, Hkv, L, d = 1, 4, 2, 9, 5
    q = rand_bf16(16, (B, Hq, d))
    K = rand_bf16(17, (B, Hkv, L, d))
    lg = oracle.logits(q, K, [L], scale=0.25)
    for g in range(Hq):
        for j in range(L):
            ref = 0.25 * sum(bf16_to_float(q[0, g, c]) * bf16_to_float(K[0, g // 2, j, c]) for c in range(d))
            assert abs(lg[0, g, j] - ref) < 1e-13


# ------------------------------------------------------------------ sparse

def _full_sel(B, Hkv, n_sink, recent_start):
    width = int(max(recent_start)) - n_sink
    sel = np.full((B, Hkv, max(width, 1)), -1, np.int32)
    nsel = np.zeros((B, Hkv), np.int32)
    for b in range(B):
        n = int(recent_start[b]) - n_sink
        sel[b, :, :n] = np.arange(n_sink, n_sink + n)
        nsel[b, :] = n
    return sel, nsel


def test_sparse_full_index_set_equals_dense(oracle):
    B, Hq, Hkv, L, d = 2, 8, 2, 300, 16
    q = rand_bf16(20, (B, Hq, d))
    K = rand_bf16(21, (B, Hkv, L, d))
    V = rand_bf16(22, (B, Hkv, L, d))
    ctx = np.array([300, 211], np.int32)
    n_sink, R = 4, 32
    rs = np.maximum(n_sink, ctx - R)
    sel, nsel = _full_sel(B, Hkv, n_sink, rs)
    out = oracle.sparse(q, K, V, sel, nsel, rs, ctx, n_sink)
    np.testing.assert_allclose(out, oracle.dense(q, K, V, ctx), rtol=1e-12, atol=1e-14)
    # n_sink = 0 and an empty recent window: the selected set alone carries everything
    sel0, nsel0 = _full_sel(B, Hkv, 0, ctx)
    out0 = oracle.sparse(q, K, V, sel0, nsel0, ctx, ctx, 0)
    np.testing.assert_allclose(out0, oracle.dense(q, K, V, ctx), rtol=1e-12, atol=1e-14)


def test_sparse_brute_force_and_set_semantics(oracle):
    B, Hq, Hkv, L, d = 1, 4, 2, 24, 3
    q = rand_bf16(23, (B, Hq, d))
    K = rand_bf16(24, (B, Hkv, L, d))
    V = rand_bf16(25, (B, Hkv, L, d))
    n_sink, rs = 2, 20
    sel = np.array([[[5, 9, 13, -1], [3, 4, 17, 19]]], np.int32)
    nsel = np.array([[3, 4]], np.int32)
    out = oracle.sparse(q, K, V, sel, nsel, [rs], [L], n_sink)
    for g in range(Hq):
        h = g // 2
        rows = sorted(set(range(n_sink)) | set(int(x) for x in sel[0, h, :nsel[0, h]]) | set(range(rs, L)))
        ref = brute_attention(q[0, g], K[0, h], V[0, h], rows, 1.0 / math.sqrt(d))
        np.testing.assert_allclose(out[0, g], ref, rtol=1e-12, atol=1e-14)
    # permutation and duplication of sel_idx, and entries overlapping sink / recent, change nothing
    sel2 = np.array([[[13, 5, 9, 5, 0, 21], [19, 17, 4, 3, 3, 23]]], np.int32)
    nsel2 = np.array([[6, 6]], np.int32)
    out2 = oracle.sparse(q, K, V, sel2, nsel2, [rs], [L], n_sink)
    np.testing.assert_allclose(out2, out, rtol=1e-13, atol=1e-15)
    # entries past n_sel are ignored
    sel3 = sel.copy()
    sel3[0, 0, 3] = 11
    np.testing.assert_array_equal(oracle.sparse(q, K, V, sel3, nsel, [rs], [L], n_sink), out)
    with pytest.raises(ValueError):
        oracle.sparse(q, K, V, np.array([[[L, 1, 1, 1], [1, 1, 1, 1]]], np.int32), nsel, [rs], [L], n_sink)


def test_sparse_planted_mass_approximates_dense(oracle):
    """If (1 - 1e-9) of the attention mass sits on known rows, attending to those rows alone ~ dense."""
    B, Hq, Hkv, L, d = 1, 2, 1, 200, 8
    rng = syn.rng_for(26, 1)
    qf = np.zeros((B, Hq, d), np.float32)
    qf[..., 0] = 16.0
    Kf = rng.standard_normal((B, Hkv, L, d), dtype=np.float32) * 0.01
    planted = [50, 77, 120]
    Kf[0, 0, planted, 0] = 8.0          # logit = 16*8/sqrt(8) ~ 45 above the rest
    V = rand_bf16(27, (B, Hkv, L, d))
    q, K = syn.f32_to_bf16_bits(qf), syn.f32_to_bf16_bits(Kf)
    sel = np.array([[planted]], np.int32)
    out = oracle.sparse(q, K, V, sel, np.array([[3]], np.int32), [L], [L], 0)
    np.testing.assert_allclose(out, oracle.dense(q, K, V, [L]), rtol=0, atol=1e-8)


def test_sparse_short_context(oracle):
    """ctx_len below n_sink + recent: sink and recent windows overlap-free by construction, J empty."""
    B, Hq, Hkv, L, d = 1, 2, 1, 6, 4
    q = rand_bf16(28, (B, Hq, d))
    K = rand_bf16(29, (B, Hkv, L, d))
    V = rand_bf16(30, (B, Hkv, L, d))
    sel = np.full((1, 1, 4), -1, np.int32)
    for ctx in (1, 3, 6):
        rs = max(4, ctx - 64)
        out = oracle.sparse(q, K, V, sel, np.zeros((1, 1), np.int32), [min(rs, ctx)], [ctx], 4)
        np.testing.assert_allclose(out, oracle.dense(q, K, V, [ctx]), rtol=1e-13, atol=1e-15)


def test_reorg_is_a_row_gather(oracle):
    """Reorg against numpy fancy indexing written here; untouched rows keep their poison; and the
    two-segment reading of a fast step -- dense attention over the compact rows followed by the recent
    rows, as one cache -- equals sparse attention on the original cache."""
    B, Hkv, Hq, L, d, n_sink, R = 2, 2, 4, 300, 128, 4, 16
    K, V = rand_bf16(1, (B, Hkv, L, d)), rand_bf16(2, (B, Hkv, L, d))
    q = rand_bf16(3, (B, Hq, d))
    ctx = np.array([300, 211], np.int32)
    rs = (ctx - R).astype(np.int32)
    nsel = np.array([[40, 17], [0, 33]], np.int32)
    sel = syn.random_sel(5, B, Hkv, 48, nsel, n_sink, rs)
    c_rows = n_sink + 48
    Kc = np.full((B, Hkv, c_rows, d), 0x7FC1, np.uint16)  # a NaN pattern
    Vc = np.full((B, Hkv, c_rows, d), 0x7FC1, np.uint16)
    oracle.reorg(K, V, sel, nsel, ctx, n_sink, Kc, Vc)
    for b in range(B):
        for h in range(Hkv):
            n = int(nsel[b, h])
            rows = np.concatenate([np.arange(n_sink), sel[b, h, :n]])
            assert (Kc[b, h, :n_sink + n] == K[b, h][rows]).all() and (Vc[b, h, :n_sink + n] == V[b, h][rows]).all()
            assert (Kc[b, h, n_sink + n:] == 0x7FC1).all() and (Vc[b, h, n_sink + n:] == 0x7FC1).all()
    ref = oracle.sparse(q, K, V, sel, nsel, rs, ctx, n_sink)
    for b in range(B):
        for h in range(Hkv):
            n = int(nsel[b, h])
            K2 = np.concatenate([Kc[b, h, :n_sink + n], K[b, h, rs[b]:ctx[b]]])[None, None]
            V2 = np.concatenate([Vc[b, h, :n_sink + n], V[b, h, rs[b]:ctx[b]]])[None, None]
            G = Hq // Hkv
            got = oracle.dense(q[b:b + 1, h * G:(h + 1) * G], K2, V2, np.array([K2.shape[2]], np.int32))
            assert np.abs(got[0] - ref[b, h * G:(h + 1) * G]).max() < 1e-12


def test_reorg_rejects_bad_input(oracle):
    K, V = rand_bf16(1, (1, 1, 40, 128)), rand_bf16(2, (1, 1, 40, 128))
    Kc = np.zeros((1, 1, 12, 128), np.uint16)
    Vc = np.zeros_like(Kc)
    with pytest.raises(ValueError):
        oracle.reorg(K, V, np.array([[[5, 41]]], np.int32), np.array([[2]], np.int32), np.array([40], np.int32), 4, Kc, Vc)
    with pytest.raises(ValueError):
        oracle.reorg(K, V, np.arange(4, 13, dtype=np.int32)[None, None], np.array([[9]], np.int32),
                     np.array([40], np.int32), 4, Kc, Vc)
