#!/usr/bin/env python3
"""Writes tests/golden/tiny_oracle.json: what the fp64 oracle computes on a small seeded workload.

Calls only the input generator and oracle/ (never the HIP library).  The file is a regression pin for the
oracle itself: tests/test_oracle_golden.py recomputes these values and compares (floats to 1e-12 relative,
integers exactly), so a change to the oracle's arithmetic cannot slip in unnoticed.  The paper prints no
worked numeric example for this path, so none of the values is the paper's.

Run from the repository root:  python tests/golden/make_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import sfi_synth as syn  # noqa: E402
from oracle import sfi_oracle as oracle  # noqa: E402


def compute():
    w = syn.make_tiny(L0=700, steps=3, budget=24, recent=32, n_support=8, B=2, Hq=8, Hkv=2)
    w.L0 = np.array([700, 431], np.int32)
    q0, ctx0 = w.q(0), w.ctx_len(0)
    dense = oracle.dense(q0, w.K, w.V, ctx0)
    sel0, nsel0, z0 = oracle.selector(q0, w.K, ctx0, w.budget, w.n_sink, w.recent)
    sp = oracle.SelectorParams(mode=1)
    sel1, nsel1, z1 = oracle.selector(q0, w.K, ctx0, w.budget, w.n_sink, w.recent, sp=sp)
    spa = oracle.SelectorParams(mode=0, alpha=0.5)
    sela, _, _ = oracle.selector(q0, w.K, ctx0, w.budget, w.n_sink, w.recent, sp=spa)
    q1, ctx1, rs1 = w.q(1), w.ctx_len(1), w.recent_start(1)
    sparse = oracle.sparse(q1, w.K, w.V, sel0, nsel0, rs1, ctx1, w.n_sink)
    toks = syn.rng_for(3, 777).integers(0, 50, size=80)
    trig = oracle.trigger_schedule(toks, [7, 11, 13], 9)
    return {
        "workload": "make_tiny(L0=700, steps=3, budget=24, recent=32, n_support=8, B=2, Hq=8, Hkv=2), ctx = [700, 431]",
        "input_checksum_K": syn.checksum(w.K), "input_checksum_V": syn.checksum(w.V),
        "dense_out_b0_head0_first8": [float(x) for x in dense[0, 0, :8]],
        "dense_out_abs_sum": float(np.abs(dense).sum()),
        "sparse_out_b1_head5_first8": [float(x) for x in sparse[1, 5, :8]],
        "sparse_out_abs_sum": float(np.abs(sparse).sum()),
        "mode0_sel": sel0.tolist(), "mode0_n_sel": nsel0.tolist(),
        "mode0_z_at_sel_b0_h0_first4": [float(z0[0, 0, j]) for j in sel0[0, 0, :4]],
        "mode1_sel": sel1.tolist(), "mode1_z_at_sel_b0_h1_first4": [float(z1[0, 1, j]) for j in sel1[0, 1, :4]],
        "mode0_alpha_half_sel": sela.tolist(),
        "trigger_tokens_seed": "rng_for(3, 777).integers(0, 50, 80); triggers {7, 11, 13}; T_max 9",
        "trigger_schedule": [int(x) for x in trig],
    }


if __name__ == "__main__":
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_oracle.json")
    with open(out, "w") as f:
        json.dump(compute(), f, indent=1)
    print("wrote", out)
