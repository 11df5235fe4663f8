"""Host logic of the seeded input generator (no method arithmetic lives there)."""
import numpy as np

import sfi_synth as syn


def test_bf16_rounding_matches_torch():
    import torch

    x = syn.rng_for(1, 1).standard_normal(100000, dtype=np.float32) * 37.0
    x[:6] = [0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38]   # ties: to even both ways
    ours = syn.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(ours, ref)
    np.testing.assert_array_equal(syn.f32_to_bf16_bits(syn.bf16_bits_to_f32(ours)), ours)


def test_workloads_are_deterministic_and_structured():
    a = syn.make_tiny(L0=512, steps=4, budget=32, recent=16, n_support=8)
    b = syn.make_tiny(L0=512, steps=4, budget=32, recent=16, n_support=8)
    assert syn.checksum(a.K) == syn.checksum(b.K) and syn.checksum(a.V) == syn.checksum(b.V)
    np.testing.assert_array_equal(a.q(3), b.q(3))
    assert syn.checksum(a.q(0)) != syn.checksum(a.q(1))
    c = syn.make_tiny(L0=512, steps=4, budget=32, recent=16, n_support=8, seed=1)
    assert syn.checksum(a.K) != syn.checksum(c.K)
    norms = np.sqrt((syn.bf16_bits_to_f32(a.K).astype(np.float64) ** 2).sum(-1))
    for h in range(a.Hkv):
        sup = a.support[0, h]
        assert len(set(sup.tolist())) == 8 and sup.min() >= a.n_sink and sup.max() < 512 - 16
        assert norms[0, h, sup].min() > 30 and norms[0, h, 0] > 30     # x4 rows: norm ~ 45
        rest = np.setdiff1d(np.arange(1, 516), sup)
        assert norms[0, h, rest].max() < 20                            # plain rows: norm ~ 11
    assert a.slow[:, 0].tolist() == [True, False, False, False]
    assert a.ctx_len(2).tolist() == [514] and a.recent_start(2).tolist() == [498]


def test_serving_mix_is_ragged_with_geometric_schedule():
    w = syn.make_serving(steps=64, B=6, Hq=16, Hkv=2, len_lo=300, len_hi=900, budget=64, recent=16)
    assert w.slow[0].all()
    assert 300 <= w.L0.min() and w.L0.max() <= 900 and len(set(w.L0.tolist())) > 1
    assert w.K.shape == (6, 2, int(w.L0.max()) + 64, 128)
    gaps = np.diff(np.flatnonzero(w.slow[:, 0]))
    assert (gaps >= 1).all()


def test_drift_moves_ten_percent_of_support():
    w = syn.make_llama8b(L0=2048, steps=4, B=1, Hq=8, Hkv=2, budget=64, recent=16)
    before = w.support.copy()
    K0 = w.K.copy()
    patches = syn.drift_support(w, epoch=1)
    n = before.shape[2]
    for b, h, pos, rows in patches:
        kept = len(np.intersect1d(before[b, h], w.support[b, h]))
        assert kept == n - max(1, round(0.1 * n))
        np.testing.assert_array_equal(w.K[b, h, pos], rows)
    changed = np.flatnonzero((w.K != K0).any(axis=(0, 3)).any(axis=0))
    assert 0 < len(changed) <= 2 * 2 * max(1, round(0.1 * n))


def test_long_config_clusters():
    w = syn.make_long(L0=4096, steps=2, Hq=8, Hkv=2, budget=128, recent=32, n_clusters=4)
    norms = np.sqrt((syn.bf16_bits_to_f32(w.K).astype(np.float64) ** 2).sum(-1))
    for h in range(2):
        for c in w.support[0, h]:
            assert norms[0, h, c] > 30 and norms[0, h, c - 16:c + 16].mean() > 14
