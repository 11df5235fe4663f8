"""Pins for the oracle's trigger schedule (CPU only): Eq. trigger plus the forced refresh after T_max fast
steps, against a loop written here from the paper's sentences, and against closed forms."""
import numpy as np

import sfi_synth as syn


def brute_schedule(tokens, trig, t_max):
    g = []
    for t in range(len(tokens)):
        if t == 0:
            g.append(1)  # Algorithm 1: g_0 = 1
            continue
        boundary = tokens[t - 1] in trig                       # Eq. trigger
        stale = len(g) >= t_max and not any(g[-t_max:])         # no slow step for T_max decoding steps
        g.append(1 if (boundary or stale) else 0)
    return np.array(g, np.uint8)


def test_trigger_matches_brute_force(oracle):
    for seed in range(6):
        r = syn.rng_for(seed, 4242)
        n = int(r.integers(1, 400))
        vocab = int(r.integers(2, 50))
        trig = set(int(i) for i in r.choice(vocab, size=int(r.integers(0, max(1, vocab // 4))), replace=False))
        t_max = int(r.integers(1, 40))
        tokens = r.integers(0, vocab, size=n)
        assert (oracle.trigger_schedule(tokens, trig, t_max) == brute_schedule(list(tokens), trig, t_max)).all()


def test_trigger_closed_forms(oracle):
    n = 200
    tokens = np.zeros(n, np.int64)
    # no trigger token ever: slow exactly every T_max + 1 steps
    g = oracle.trigger_schedule(tokens, [], 7)
    assert (np.nonzero(g)[0] == np.arange(0, n, 8)).all()
    # every token a trigger: every step slow
    assert oracle.trigger_schedule(tokens, [0], 7).all()
    # T_max = 0: every step slow even without triggers
    assert oracle.trigger_schedule(tokens, [], 0).all()
    # one trigger token at step 10: step 11 is slow, and the forced refresh counts from there
    tokens[10] = 5
    g = oracle.trigger_schedule(tokens, [5], 64)
    assert list(np.nonzero(g)[0]) == [0, 11, 76, 141]
