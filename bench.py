#!/usr/bin/env python3
"""Benchmark of the slow/fast decode-attention path on one MI355X.

Workload (default): the Llama-3-8B-shaped layer of the baseline configs — batch 4, 32 query / 8 KV
heads, head_dim 128, context 32768 (+1 per decode step), budget K = 2048, recent window 128,
sink 4, one slow step every 16 decode steps, bf16 K/V ~ N(0,1) with 1 % planted x4 support rows.

A benchmark "step" is one refresh segment = 16 decode steps (1 slow + 15 fast, with the device-side
state update after each) run over `--layers` virtual layers, every layer with its own K/V buffers
and its own selected index sets, visited round-robin inside each decode step the way a model's
layers are.  With 16 layers the fast steps touch ~570 MB between two visits of the same layer, so
neither L2 nor the 256 MB last-level cache can serve the re-reads (cold-cache numbers).
The timed region is captured into one HIP graph and replayed once (inputs resident in HBM).

Reported value: decode-attention tokens/s of ONE attention layer for the slow+fast mix
(batch x decode steps x layers / time).

Without --workload the line's value is the default workload above and a "workloads" object carries
short runs of the other stated configurations (one long stream at 131072, the long-CoT window, the
ragged serving mix), each with its own roofline object, parity sample and oracle baseline.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
FAST_MERGE = {None: 0, "kernel": 1, "launch": 2}  # sfi_set_tuning codes

# Fixed-schedule workloads (one slow step every `seg` decode steps).  Default: the Llama-3-8B-shaped layer.
# layers: virtual layers, chosen so that one round of fast steps over all layers moves more than the 256 MB
# last-level cache holds.
WORKLOADS = {
    "llama8b": dict(make="make_llama8b", ctx=32768, batch=4, seg=16, layers=16,
                    label="llama8b-shaped layer"),
    "long": dict(make="make_long", ctx=131072, batch=1, seg=32, layers=32,
                 label="long single stream"),
    "cot": dict(make="make_cot", ctx=24576, batch=8, seg=24, layers=16,
                label="long-CoT window (G=5)"),
}


def kernel_source_hash():
    """First 16 hex digits of the sha256 over the library's kernel sources (what a committed profile was taken on)."""
    import glob
    import hashlib
    h = hashlib.sha256()
    for f in sorted(glob.glob(os.path.join(ROOT, "paper_2603_12038_amd", "csrc", "*"))):
        h.update(open(f, "rb").read())
    return h.hexdigest()[:16]


def committed_traffic(kernel_key):
    """HBM bytes per launch of a kernel from the committed rocprofv3 --pmc summary (FETCH_SIZE + WRITE_SIZE, each scaled
    by what the counter reads for a plain copy), if that summary was taken on the kernel sources of this tree; it is not
    measured in this run (counters need the profiler).  Returns (bytes or None, where it comes from)."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_llama8b.txt")
    if not os.path.exists(path):
        return None, "no committed counter profile"
    prof = json.load(open(path))
    if prof.get("kernel_source_sha256_16") != kernel_source_hash():
        return None, "profiles/hbm_traffic_llama8b.txt was taken on other kernel sources than this tree's: not quoted"
    if kernel_key not in prof:
        return None, "kernel not in profiles/hbm_traffic_llama8b.txt"
    return prof[kernel_key].get("hbm_bytes_per_launch"), "profiles/hbm_traffic_llama8b.txt (rocprofv3 --pmc on these kernel sources; not measured in this run)"


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def _emit(res):
    print(json.dumps(res))


def _event_us(torch, fn, reps):
    """Mean microseconds of fn() over reps back-to-back calls (HIP events on the current stream)."""
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for r in range(reps):
        fn(r)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / reps


def bench_serving(args):
    """Config 5: batch 32, 64 query / 8 KV heads (G = 8), ragged contexts U{16384..65536}, K = 2048, recent 128;
    every sequence draws its slow-step gaps from Geometric(1/20); each decode step is one sfi_mixed_step per layer
    (per-sequence mode flags on the device).  K/V ~ N(0,1) bf16 generated on the device (8.6 GB per layer), 0.5 %
    support rows scaled x4 in K.  A benchmark step is 16 decode steps over the virtual layers."""
    import numpy as np
    import torch

    import paper_2603_12038_amd as sfi
    import sfi_synth as syn
    from sfi_check import check_out, check_selection, i32_dev

    SEG = 16
    NL = args.layers or 4
    B = args.batch or 32
    n_dec = SEG * (args.steps + args.warmup)
    w = syn.make_serving(steps=n_dec + SEG, B=B, alloc=False)
    Hq, Hkv, d = w.Hq, w.Hkv, w.d
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(77)
    Ks, Vs = [], []
    for l in range(NL):
        k = torch.empty(B, Hkv, w.L_alloc, d, dtype=torch.bfloat16, device=dev)
        v = torch.empty_like(k)
        for b in range(B):
            k[b] = torch.randn(Hkv, w.L_alloc, d, device=dev, generator=gen).to(torch.bfloat16)
            v[b] = torch.randn(Hkv, w.L_alloc, d, device=dev, generator=gen).to(torch.bfloat16)
        sup = torch.from_numpy(w.support).to(dev)  # [B, Hkv, n]
        rows = (sup + l * 13) % int(w.L0.min() - w.recent)
        for b in range(B):
            for hh in range(Hkv):
                k[b, hh, rows[b, hh]] *= 4.0
        Ks.append(k)
        Vs.append(v)
    log(f"serving workload on device: B={B} Hq={Hq} Hkv={Hkv} ctx {int(w.L0.min())}..{int(w.L0.max())} layers={NL} "
        f"({torch.cuda.memory_allocated() / 1e9:.1f} GB)")
    max_ctx = int(w.L_alloc)
    ctx = sfi.SfiContext(B, Hq, Hkv, max_ctx, w.budget, w.n_sink, w.recent, Ks[0], Vs[0])
    h = ctx.handle
    if args.dense_wgs or args.fast_tpw or args.fast_merge:
        sfi.sfi_set_tuning(h, args.dense_wgs, args.fast_tpw, FAST_MERGE[args.fast_merge])
    if args.mixed_dense == "grid":
        sfi.sfi_set_mixed_plan(h, False)
    q_all = torch.randn(n_dec + SEG, NL, B, Hq, d, device=dev, generator=gen).to(torch.bfloat16)
    outs = [torch.zeros(B, Hq, d, dtype=torch.float32, device=dev) for _ in range(NL)]
    sels = [torch.full((B, Hkv, w.budget), -1, dtype=torch.int32, device=dev) for _ in range(NL)]
    nsels = [torch.zeros(B, Hkv, dtype=torch.int32, device=dev) for _ in range(NL)]
    flags = torch.from_numpy(w.slow.astype(np.uint8)).to(dev)  # [steps, B]
    ctx_d, rs_d = i32_dev(w.ctx_len(0)), i32_dev(w.recent_start(0))

    def decode_step(t):
        for l in range(NL):
            sfi.sfi_mixed_step(h, q_all[t, l], Ks[l], Vs[l], flags[t], ctx_d, rs_d, max_ctx, w.budget, outs[l], sels[l],
                               nsels[l])
        sfi.sfi_advance(h, ctx_d, rs_d)

    # ---- parity sample + CPU baseline on layer 0: step 0 (every sequence slow) and a step of fast sequences, each
    # checked against the oracle on three sequences (the longest, the shortest, one in between) copied back to the host
    cpu_baseline, parity = None, {}
    if not args.no_cpu_baseline:
        from oracle import sfi_oracle as oracle

        order = np.argsort(w.L0)
        sample = [int(order[-1]), int(order[0]), int(order[B // 2])]
        bits = lambda t: t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
        Kh = {b: bits(Ks[0][b:b + 1]) for b in sample}
        Vh = {b: bits(Vs[0][b:b + 1]) for b in sample}
        all_slow = torch.ones(B, dtype=torch.uint8, device=dev)
        c0, c1, rs1 = w.ctx_len(0), w.ctx_len(1), w.recent_start(1)
        sfi.sfi_mixed_step(h, q_all[0, 0], Ks[0], Vs[0], all_slow, ctx_d, rs_d, max_ctx, w.budget, outs[0], sels[0], nsels[0])
        torch.cuda.synchronize()
        g_out, g_sel, g_nsel = outs[0].cpu().numpy(), sels[0].cpu().numpy(), nsels[0].cpu().numpy()
        q0 = bits(q_all[0, 0])
        t_slow, rows_slow, errs, exact = 0.0, 0, [], 0
        for b in sample:
            t1 = time.time()
            o_d = oracle.dense(q0[b:b + 1], Kh[b], Vh[b], c0[b:b + 1])
            o_sel, o_nsel, o_z = oracle.selector(q0[b:b + 1], Kh[b], c0[b:b + 1], w.budget, w.n_sink, w.recent)
            t_slow += time.time() - t1
            rows_slow += int(c0[b])
            errs.append(check_out(g_out[b:b + 1], o_d))
            exact += check_selection(g_sel[b:b + 1], g_nsel[b:b + 1], o_sel, o_nsel, o_z, c0[b:b + 1], w.n_sink, w.recent, w.budget)
        parity["slow_out_row_rel_err"] = max(errs)
        parity["selection_sets_exact"] = f"{exact}/{len(sample) * Hkv}"
        none = torch.zeros(B, dtype=torch.uint8, device=dev)
        sfi.sfi_mixed_step(h, q_all[1, 0], Ks[0], Vs[0], none, i32_dev(c1), i32_dev(rs1), max_ctx, w.budget, outs[0], sels[0], nsels[0])
        torch.cuda.synchronize()
        g_out, q1 = outs[0].cpu().numpy(), bits(q_all[1, 0])
        t_fast, errs = 0.0, []
        for b in sample:
            t1 = time.time()
            o_s = oracle.sparse(q1[b:b + 1], Kh[b], Vh[b], g_sel[b:b + 1], g_nsel[b:b + 1], rs1[b:b + 1], c1[b:b + 1], w.n_sink)
            t_fast += time.time() - t1
            errs.append(check_out(g_out[b:b + 1], o_s))
        parity["fast_out_row_rel_err"] = max(errs)
        # the mix as scheduled: a sequence is slow once per 20 steps on average; a slow sequence costs the oracle in
        # proportion to its context (scaled from the sample's rows to the batch's mean context)
        s_slow = t_slow / rows_slow * float(w.L0.mean())
        s_fast = t_fast / len(sample)
        per_seq_step = s_slow / 20.0 + s_fast * 19.0 / 20.0
        cpu_baseline = {"value": 1.0 / per_seq_step, "unit": "tokens/s per attention layer", "cores": oracle.num_threads(),
                        "kind": "oracle",
                        "sample": f"3 of the {B} sequences (ctx {[int(c0[b]) for b in sample]}): one slow step (dense + Selector) "
                                  "and one fast step each, scaled to the batch's mean context and to one slow step in 20",
                        "slow_step_s_per_sequence_at_mean_ctx": s_slow, "fast_step_s_per_sequence": s_fast}
        log(f"serving parity sample ok {parity}; oracle {s_slow:.2f}s per slow sequence, {s_fast:.4f}s per fast one")
        del Kh, Vh

    for t in range(args.warmup * SEG):
        decode_step(t)
    torch.cuda.synchronize()
    t0 = args.warmup * SEG
    n_t = args.steps * SEG
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        graph.capture_begin()
        for t in range(t0, t0 + n_t):
            decode_step(t)
        graph.capture_end()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    graph.replay()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t1
    # KV bytes the timed steps had to read: whole prefix for slow sequences, sink + selected + recent otherwise
    kv = 0
    n_slow = 0
    for t in range(t0, t0 + n_t):
        L = w.ctx_len(t).astype(np.int64)
        slow = w.slow[t]
        rows = np.where(slow, L, w.n_sink + w.budget + (L - w.recent_start(t)))
        kv += int(rows.sum()) * Hkv * d * 2 * 2 * NL
        n_slow += int(slow.sum())
    # per-kernel times of an all-fast step and of the mixed steps as scheduled (events around every kernel)
    t_p = t0 + n_t
    none = torch.zeros(B, dtype=torch.uint8, device=dev)
    sfi.sfi_set_profiling(h, 4 * NL)
    for r in range(4):
        for l in range(NL):
            sfi.sfi_mixed_step(h, q_all[t_p + r, l], Ks[l], Vs[l], none, ctx_d, rs_d, max_ctx, w.budget, outs[l], sels[l],
                               nsels[l])
    torch.cuda.synchronize()
    ms, cnt = sfi.sfi_stage_times(h)
    sfi.sfi_set_profiling(h, 0)
    gather_us = ms[6] / max(cnt[6], 1) * 1e3
    # the ragged step by the number of slow sequences in it (chosen across the lengths): the dense launch's time (event
    # pair, about 2 us above the trace's duration) against the rows it has to read
    by_slow = []
    order = np.argsort(w.L0)
    for which in ([], [order[B // 2]], [order[-1]], [order[3], order[-3]], list(order[::8]), list(order[::4]), list(order[::2]), list(order)):
        fl = np.zeros(B, np.uint8)
        fl[[int(b) for b in which]] = 1
        fd = torch.from_numpy(fl).to(dev)
        sfi.sfi_set_profiling(h, 4 * NL)
        for r in range(4):
            for l in range(NL):
                sfi.sfi_mixed_step(h, q_all[t_p + r, l], Ks[l], Vs[l], fd, ctx_d, rs_d, max_ctx, w.budget, outs[l], sels[l], nsels[l])
        torch.cuda.synchronize()
        ms2, cnt2 = sfi.sfi_stage_times(h)
        sfi.sfi_set_profiling(h, 0)
        us2 = [ms2[i] / max(cnt2[i], 1) * 1e3 for i in range(len(ms2))]
        slow_bytes = int(sum(int(w.ctx_len(t_p)[int(b)]) for b in which)) * Hkv * d * 2 * 2
        by_slow.append({"slow_sequences": len(which), "dense_kv_bytes": slow_bytes, "dense_us": us2[0],
                        "dense_frac_of_8TBps": slow_bytes / (us2[0] * 1e-6) / 1e9 / HBM_PEAK_GBS if which else None,
                        "gather_us": us2[6], "score_us": us2[2], "cand_us": us2[3], "write_us": us2[5]})
    L_p = w.ctx_len(t_p).astype(np.int64)
    fast_bytes = int((w.n_sink + w.budget + (L_p - w.recent_start(t_p))).sum()) * Hkv * d * 2 * 2
    fast_gbs = fast_bytes / (gather_us * 1e-6) / 1e9
    tokens = B * n_t * NL
    res = {
        "metric": "decode attn tokens/s (slow+fast mix)", "value": tokens / wall, "unit": "tokens/s per attention layer",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": wall * 1e3 / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"serving mix: B{B} Hq{Hq} Hkv{Hkv} d{d} ragged ctx {int(w.L0.min())}..{int(w.L0.max())} "
                               f"k{w.budget} R{w.recent} sink{w.n_sink}, per-sequence slow gaps ~ Geometric(1/20)",
                   "step": f"{SEG} decode steps (sfi_mixed_step) x {NL} virtual layers", "virtual_layers": NL,
                   "launch": "graph", "mixed_dense": args.mixed_dense, "slow_sequence_steps_in_timed_region": n_slow},
        "roofline": {"bound": "hbm", "kernel": "sfi::attn_gather_stream_kernel (all-fast step)", "achieved": fast_gbs,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": fast_gbs / HBM_PEAK_GBS, "traffic": None,
                     "algorithmic_bytes_per_launch": fast_bytes, "us_per_launch": gather_us},
        "whole_run_kv_GBps": kv / wall / 1e9, "whole_run_frac_of_8TBps": kv / wall / 1e9 / HBM_PEAK_GBS,
        "all_fast_step_stage_us": {"gather": gather_us, "merge": ms[1] / max(cnt[1], 1) * 1e3},
        "ragged_step_by_slow_sequences": by_slow,
        "us_per_decode_step_per_layer": wall * 1e6 / (n_t * NL),
        "parity_sample": parity,
        "device_status": sfi.sfi_device_status(ctx.handle),  # 0: no device-side input had to be clamped
        "cpu_baseline": cpu_baseline,
    }
    res["roofline"]["traffic_source"] = "not measured in this run (counters need the profiler); no committed counter profile of this workload"
    ctx.close()
    del Ks, Vs, q_all, graph
    torch.cuda.empty_cache()
    return res


def bench_retention(args):
    """Shape of the paper's kernel table (Table "kernel_speedup": KV length 16K, batch 16, bf16): latency of the
    sparse attention (gather kernel + merge) over the dense attention (dense kernel + merge) at the table's
    retention ratios, each timed with HIP events around back-to-back launches cycling over virtual layers."""
    import numpy as np
    import torch

    import paper_2603_12038_amd as sfi
    import sfi_synth as syn
    from sfi_check import i32_dev

    B, Hq, Hkv, d, L, R, n_sink = args.batch or 16, 32, 8, 128, args.ctx or 16384, 128, 4
    NL = args.layers or 4
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(5)
    Ks = [torch.randn(B, Hkv, L, d, device=dev, generator=gen).to(torch.bfloat16) for _ in range(NL)]
    Vs = [torch.randn(B, Hkv, L, d, device=dev, generator=gen).to(torch.bfloat16) for _ in range(NL)]
    max_budget = L - R - n_sink
    ctx = sfi.SfiContext(B, Hq, Hkv, L, max_budget, n_sink, R, Ks[0], Vs[0])
    h = ctx.handle
    if args.dense_wgs or args.fast_tpw or args.fast_merge:
        sfi.sfi_set_tuning(h, args.dense_wgs, args.fast_tpw, FAST_MERGE[args.fast_merge])
    q = torch.randn(B, Hq, d, device=dev, generator=gen).to(torch.bfloat16)
    out = torch.zeros(B, Hq, d, dtype=torch.float32, device=dev)
    ctx_d = i32_dev(np.full(B, L))
    rs_d = i32_dev(np.full(B, L - R))
    reps = 6 * NL
    dense_us = _event_us(torch, lambda r: sfi.sfi_dense_attn(h, q, Ks[r % NL], Vs[r % NL], ctx_d, L, out), NL)
    dense_us = min(_event_us(torch, lambda r: sfi.sfi_dense_attn(h, q, Ks[r % NL], Vs[r % NL], ctx_d, L, out), reps)
                   for _ in range(3))  # (the one figure every row of the table is divided into: best of three)
    paper = {1.6: 10.67, 6.3: 9.56, 12.5: 7.15, 25.0: 3.96, 37.5: 2.75, 50.0: 2.10, 75.0: 1.43, 98.4: 1.10, 100.0: 1.00}
    rows = []
    for pct, paper_x in paper.items():
        budget = max(0, min(max_budget, int(round(pct / 100.0 * L)) - R - n_sink))  # rows kept = sink + budget + recent
        sel = torch.full((NL, B, Hkv, max(budget, 1)), -1, dtype=torch.int32, device=dev)
        for l in range(NL):
            for b in range(B):
                for hh in range(Hkv):
                    if budget > 0:
                        perm = torch.randperm(max_budget, device=dev, generator=gen)[:budget].sort().values
                        sel[l, b, hh, :budget] = (perm + n_sink).to(torch.int32)
        nsel = torch.full((B, Hkv), budget, dtype=torch.int32, device=dev)
        fn = lambda r: sfi.sfi_fast_step(h, q, Ks[r % NL], Vs[r % NL], sel[r % NL], nsel, max(budget, 1), rs_d, ctx_d, out)
        _event_us(torch, fn, NL)
        sparse_us = min(_event_us(torch, fn, reps) for _ in range(3))
        kept = n_sink + budget + R
        rows.append({"retention_pct": pct, "rows_kept": kept, "sparse_us": sparse_us, "dense_us": dense_us,
                     "speedup": dense_us / sparse_us, "paper_speedup_b200": paper_x,
                     "sparse_GBps": B * Hkv * kept * d * 4 / (sparse_us * 1e-6) / 1e9})
        log(f"retention {pct:5.1f}%: sparse {sparse_us:7.1f} us, dense {dense_us:7.1f} us, x{dense_us / sparse_us:5.2f} "
            f"(paper, B200: x{paper_x})")
    dense_bytes = B * Hkv * L * d * 4
    res = {
        "metric": "sparse over dense attention latency ratio", "value": rows[0]["speedup"], "unit": "x at 1.6 % retention",
        "n_gpus": 1, "steps": reps, "warmup": NL, "ms_per_step": dense_us * 1e-3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"kernel table shape: B{B} Hq{Hq} Hkv{Hkv} d{d} KV length {L}, recent {R}, sink {n_sink}",
                   "virtual_layers": NL, "timing": "dense kernel + merge vs gather kernel + merge, HIP events"},
        "roofline": {"bound": "hbm", "kernel": "sfi::attn_dense_kernel<0> + merge", "achieved": dense_bytes / (dense_us * 1e-6) / 1e9,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": dense_bytes / (dense_us * 1e-6) / 1e9 / HBM_PEAK_GBS,
                     "traffic": None},
        "table": rows, "device_status": sfi.sfi_device_status(ctx.handle), "cpu_baseline": None,
    }
    ctx.close()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=8, help="timed refresh segments (16 decode steps each)")
    ap.add_argument("--warmup", type=int, default=2, help="untimed refresh segments")
    ap.add_argument("--workload", choices=sorted(WORKLOADS) + ["serving", "retention"], default=None,
                    help="llama8b (the baseline's metric workload), long, cot: slow+fast mix on a fixed schedule; "
                         "serving: ragged batch-32 mix with per-sequence modes; retention: sparse vs dense kernel "
                         "latency at KV length 16K")
    ap.add_argument("--layers", type=int, default=0, help="virtual layers (distinct K/V buffers); 0 = workload default")
    ap.add_argument("--ctx", type=int, default=0, help="context length at step 0; 0 = workload default")
    ap.add_argument("--batch", type=int, default=0, help="sequences; 0 = workload default")
    ap.add_argument("--launch", choices=["graph", "stream"], default="graph")
    ap.add_argument("--fast-path", choices=["gather", "compact"], default="gather",
                    help="gather: fast steps read the selected rows in place through sel_idx; compact: every slow "
                         "step is followed by Reorg into a compact buffer and fast steps read the two-segment layout")
    ap.add_argument("--slow-schedule", choices=["sync", "async"], default="sync",
                    help="sync: each layer's Selector runs on the main stream after its dense attention; async: "
                         "layer-wise asynchronous execution -- Selector (and Reorg) of layer i on a second stream "
                         "under the dense attention of layer i+1, ring of --ring workspaces, one barrier at the end")
    ap.add_argument("--ring", type=int, default=4, help="workspace slots of the asynchronous slow step")
    ap.add_argument("--page-size", type=int, default=0,
                    help="0: flat K/V tensors; a power of two >= 16: K/V handed over as block pools of that many rows "
                         "with one randomly permuted block table shared by the layers (fixed-schedule workloads)")
    ap.add_argument("--page-layout", choices=["thd", "htd"], default="htd",
                    help="block layout of a paged cache: [blocks][page][Hkv][d] or [blocks][Hkv][page][d]")
    ap.add_argument("--selector-mode", type=int, choices=[0, 1], default=0,
                    help="0: evidence-only ranking (the measured baseline); 1: Algorithm 2 in full, oracle defaults")
    ap.add_argument("--kv-layout", choices=["separate", "interleaved"], default="separate",
                    help="flat cache only: K and V as two tensors, or as one [B, Hkv, L, 2, d] tensor whose row t "
                         "holds k_t then v_t (the library sees two base pointers and a row stride of 2 d either way)")
    ap.add_argument("--out-bf16", action="store_true",
                    help="outputs stored as bf16 (cfg.out_bf16) instead of fp32; slow+fast mix workloads only")
    ap.add_argument("--mixed-dense", choices=["planned", "grid"], default="planned",
                    help="serving workload, A/B of the ragged step's dense launch: planned on the device (one workgroup per "
                         "compute unit, splits per slow sequence by length; default) or one workgroup per cell of the batch")
    ap.add_argument("--dense-k", choices=["pieces", "whole-lines"], default="pieces",
                    help="A/B of the dense kernel's K loads: four 64-byte pieces per row (default) or whole 128-byte lines")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--dense-wgs", type=int, default=0)
    ap.add_argument("--fast-tpw", type=int, default=0)
    ap.add_argument("--fast-merge", choices=["kernel", "launch"], default=None,
                    help="merge of a fast step's split records: inside the attention kernel (default) or in a launch of its own")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (no collectives, no sharding); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    if args.workload == "serving":
        return _emit(bench_serving(args))
    if args.workload == "retention":
        return _emit(bench_retention(args))
    if args.workload is not None:
        return _emit(bench_mix(args))
    # Default run: the metric's workload in full, then short runs of the other stated configurations.
    import copy
    args.workload = "llama8b"
    res = bench_mix(args)
    others = {}
    for name in ("long", "cot", "serving"):
        a = copy.copy(args)
        a.workload, a.steps, a.warmup, a.layers, a.ctx, a.batch = name, 2, 1, 0, 0, 0
        log(f"--- workload {name} (short run: {a.steps} timed + {a.warmup} warm-up steps)")
        r = bench_serving(a) if name == "serving" else bench_mix(a)
        others[name] = {k: r[k] for k in ("value", "unit", "ms_per_step", "steps", "warmup", "config", "roofline", "kernels",
                                            "us_per_decode_step_per_layer", "parity_sample", "device_status", "cpu_baseline",
                                            "whole_run_frac_of_8TBps", "all_fast_step_stage_us") if k in r}
    res["workloads"] = others
    _emit(res)


def bench_mix(args):
    """A fixed-schedule slow+fast mix (WORKLOADS): returns the result object."""
    wl = WORKLOADS[args.workload]
    SEG = wl["seg"]
    args.ctx = args.ctx or wl["ctx"]
    args.batch = args.batch or wl["batch"]
    args.layers = args.layers or wl["layers"]

    import numpy as np
    import torch

    import paper_2603_12038_amd as sfi
    import sfi_synth as syn
    from sfi_check import check_out, check_out_bf16, check_selection, i32_dev, to_dev

    if args.out_bf16:  # the parity sample then uses the bf16 rule (an ulp of the element + the fp32 path's error)
        check_out = check_out_bf16
    err_key = "out_frac_of_bf16_bound" if args.out_bf16 else "out_row_rel_err"
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    sfi.load_library()  # fails loudly if libsfi.so is not built
    dev = torch.device("cuda:0")
    K_seg, W_seg, NL = args.steps, args.warmup, args.layers
    n_dec = SEG * (K_seg + W_seg)

    t0 = time.time()
    w = getattr(syn, wl["make"])(L0=args.ctx, steps=n_dec + SEG, B=args.batch)  # rows for the schedule + a spare segment
    log(f"generated workload in {time.time() - t0:.1f}s: B={w.B} Hq={w.Hq} Hkv={w.Hkv} L0={args.ctx} "
        f"K={w.budget} R={w.recent} layers={NL}")
    B, Hq, Hkv, d, L0 = w.B, w.Hq, w.Hkv, w.d, args.ctx

    # ---- device state: NL virtual layers = base K/V with rows [0, L0) rolled by a layer-specific shift
    K0, V0 = to_dev(w.K), to_dev(w.V)
    shift = lambda l: (l * 4099) % L0
    Ks, Vs = [K0], [V0]
    for l in range(1, NL):
        k = K0.clone()
        v = V0.clone()
        k[:, :, :L0] = torch.roll(K0[:, :, :L0], shift(l), dims=2)
        v[:, :, :L0] = torch.roll(V0[:, :, :L0], shift(l), dims=2)
        Ks.append(k)
        Vs.append(v)
    max_ctx = int(w.L_alloc)
    if args.kv_layout == "interleaved":
        assert not args.page_size, "--kv-layout interleaved is for the flat cache"
        for l in range(NL):
            kv = torch.empty(B, Hkv, Ks[l].shape[2], 2, d, dtype=Ks[l].dtype, device=dev)
            kv[:, :, :, 0] = Ks[l]
            kv[:, :, :, 1] = Vs[l]
            Ks[l], Vs[l] = kv[:, :, :, 0], kv[:, :, :, 1]
        K0, V0 = Ks[0], Vs[0]
        torch.cuda.synchronize()
    n_blocks = 0
    if args.page_size:
        # scatter every layer's flat cache into a block pool [n_blocks, page, Hkv, d] through one block table
        P = args.page_size
        pages = (max_ctx + P - 1) // P
        n_blocks = B * pages
        gperm = torch.Generator(device="cpu")
        gperm.manual_seed(99)
        perm = torch.randperm(n_blocks, generator=gperm).to(dev)
        table_d = perm.view(B, pages).to(torch.int32).contiguous()

        def to_pool(x):
            pad = pages * P - x.shape[2]
            if pad:
                x = torch.cat([x, torch.zeros(B, Hkv, pad, d, dtype=x.dtype, device=dev)], dim=2)
            if args.page_layout == "thd":
                blocks = x.view(B, Hkv, pages, P, d).permute(0, 2, 3, 1, 4).reshape(n_blocks, P, Hkv, d)
            else:
                blocks = x.view(B, Hkv, pages, P, d).permute(0, 2, 1, 3, 4).reshape(n_blocks, Hkv, P, d)
            pool = torch.empty_like(blocks)
            pool[perm] = blocks
            return pool

        Ks = [to_pool(k) for k in Ks]
        Vs = [to_pool(v) for v in Vs]
        K0, V0 = Ks[0], Vs[0]
        torch.cuda.synchronize()
    sel_params = None
    if args.selector_mode == 1:
        sel_params = dict(gamma=0.5, beta=1.0, p=2.0, eta=0.5, lambda_clip=0.02, alpha_soft=0.5, alpha_cross=0.35,
                          temp=1.0, eps=1e-8, nms_radius=2)
    mk = lambda: sfi.SfiContext(B, Hq, Hkv, max_ctx, w.budget, w.n_sink, w.recent, K0, V0, selector=sel_params,
                                page_size=args.page_size, page_layout=args.page_layout, out_bf16=args.out_bf16)
    ctx = mk()
    h = ctx.handle
    use_async = args.slow_schedule == "async"
    ring = [ctx] + [mk() for _ in range(args.ring - 1)] if use_async else [ctx]
    if args.page_size:
        for c in ring:
            sfi.sfi_set_block_table(c.handle, table_d, n_blocks)
    aux = torch.cuda.Stream() if use_async else None  # default priority
    if args.dense_wgs or args.fast_tpw or args.fast_merge:
        for c in ring:
            sfi.sfi_set_tuning(c.handle, args.dense_wgs, args.fast_tpw, FAST_MERGE[args.fast_merge])
    if args.dense_k == "whole-lines":
        for c in ring:
            sfi.sfi_set_dense_k_layout(c.handle, True)
    gen = torch.Generator(device=dev)
    gen.manual_seed(1234)
    q_all = torch.randn(n_dec + SEG, NL, B, Hq, d, device=dev, generator=gen).to(torch.bfloat16)
    outs = [torch.zeros(B, Hq, d, dtype=torch.bfloat16 if args.out_bf16 else torch.float32, device=dev) for _ in range(NL)]
    sels = [torch.full((B, Hkv, w.budget), -1, dtype=torch.int32, device=dev) for _ in range(NL)]
    nsels = [torch.zeros(B, Hkv, dtype=torch.int32, device=dev) for _ in range(NL)]
    ctx_d, rs_d = i32_dev(w.ctx_len(0)), i32_dev(w.recent_start(0))
    torch.cuda.synchronize()
    log(f"device state ready ({torch.cuda.memory_allocated() / 1e9:.1f} GB)")

    compact = args.fast_path == "compact"
    if compact:
        Kcs = [torch.zeros(B, Hkv, w.n_sink + w.budget, d, dtype=torch.bfloat16, device=dev) for _ in range(NL)]
        Vcs = [torch.zeros(B, Hkv, w.n_sink + w.budget, d, dtype=torch.bfloat16, device=dev) for _ in range(NL)]

    def slow(l, step):
        sfi.sfi_slow_step(h, q_all[step, l], Ks[l], Vs[l], ctx_d, max_ctx, w.budget, outs[l], sels[l], nsels[l])
        if compact:
            sfi.sfi_reorg(h, Ks[l], Vs[l], sels[l], nsels[l], w.budget, ctx_d, None, Kcs[l], Vcs[l])

    def fast(l, step):
        if compact:
            sfi.sfi_fast_step_compact(h, q_all[step, l], Kcs[l], Vcs[l], nsels[l], w.budget, Ks[l], Vs[l], rs_d, ctx_d,
                                      outs[l])
        else:
            sfi.sfi_fast_step(h, q_all[step, l], Ks[l], Vs[l], sels[l], nsels[l], w.budget, rs_d, ctx_d, outs[l])

    def slow_all_layers_async(step):
        """Sec. 4.1 schedule: Attn_1 .. Attn_NL back to back on the main stream; Sel_i (+ Reorg_i) on the second
        stream as soon as Attn_i is done; a ring slot is reused only after the Selector that last used it; one
        barrier before the fast steps."""
        main = torch.cuda.current_stream()
        slot_free = [None] * len(ring)
        for l in range(NL):
            slot = l % len(ring)
            hs = ring[slot].handle
            if slot_free[slot] is not None:
                main.wait_event(slot_free[slot])
            sfi.sfi_slow_attn(hs, q_all[step, l], Ks[l], Vs[l], ctx_d, max_ctx, outs[l])
            done = torch.cuda.Event()
            done.record(main)
            aux.wait_event(done)
            with torch.cuda.stream(aux):
                sfi.sfi_slow_select(hs, ctx_d, max_ctx, w.budget, sels[l], nsels[l])
                if compact:
                    sfi.sfi_reorg(hs, Ks[l], Vs[l], sels[l], nsels[l], w.budget, ctx_d, None, Kcs[l], Vcs[l])
                slot_free[slot] = torch.cuda.Event()
                slot_free[slot].record(aux)
        main.wait_stream(aux)

    def segment(step0):
        for t in range(SEG):
            if t == 0 and use_async:
                slow_all_layers_async(step0)
            else:
                for l in range(NL):
                    (slow if t == 0 else fast)(l, step0 + t)
            sfi.sfi_advance(h, ctx_d, rs_d)

    # ---- parity sample + CPU baseline: 1 slow + 2 fast steps of layer 0 at step 0 ---------------------
    cpu_baseline = None
    parity = {}
    if not args.no_cpu_baseline:
        from oracle import sfi_oracle as oracle

        qs = [q_all[t, 0].view(torch.int16).cpu().numpy().view(np.uint16) for t in range(3)]
        c0 = w.ctx_len(0)
        slow(0, 0)
        torch.cuda.synchronize()
        g_out, g_sel, g_nsel = outs[0].float().cpu().numpy(), sels[0].cpu().numpy(), nsels[0].cpu().numpy()
        t1 = time.time()
        o_dense = oracle.dense(qs[0], w.K, w.V, c0)
        o_sp = oracle.SelectorParams(mode=1, **sel_params) if sel_params else None
        o_sel, o_nsel, o_z = oracle.selector(qs[0], w.K, c0, w.budget, w.n_sink, w.recent, sp=o_sp)
        t_slow = time.time() - t1
        parity[f"slow_{err_key}"] = check_out(g_out, o_dense)
        n_exact = check_selection(g_sel, g_nsel, o_sel, o_nsel, o_z, c0, w.n_sink, w.recent, w.budget)
        parity["selection_sets_exact"] = f"{n_exact}/{B * Hkv}"
        t_fast = 0.0
        for t in (1, 2):
            ct, rt = w.ctx_len(t), w.recent_start(t)
            sfi.sfi_fast_step(h, q_all[t, 0], K0, V0, sels[0], nsels[0], w.budget, i32_dev(rt), i32_dev(ct), outs[0])
            torch.cuda.synchronize()
            t1 = time.time()
            o_sp = oracle.sparse(qs[t], w.K, w.V, g_sel, g_nsel, rt, ct, w.n_sink)
            t_fast += time.time() - t1
            parity[f"fast{t}_{err_key}"] = check_out(outs[0].float().cpu().numpy(), o_sp)
        t_fast /= 2
        cpu_baseline = {
            "value": B * SEG / (t_slow + (SEG - 1) * t_fast), "unit": "tokens/s per attention layer",
            "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"1 slow step (dense + Selector) + 2 fast steps of layer 0, extrapolated to 1 slow + {SEG - 1} fast",
            "slow_step_s": t_slow, "fast_step_s": t_fast,
        }
        log(f"parity sample ok {parity}; oracle slow {t_slow:.2f}s fast {t_fast:.3f}s on {oracle.num_threads()} threads")

    # ---- warm-up (eager), then the timed region ---------------------------------------------------------
    for s in range(W_seg):
        segment(s * SEG)
    torch.cuda.synchronize()
    step0 = W_seg * SEG
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    if args.launch == "graph":
        state = [ctx_d.clone(), rs_d.clone()]
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            graph.capture_begin()
            for s in range(K_seg):
                segment(step0 + s * SEG)
            graph.capture_end()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        assert (ctx_d == state[0]).all(), "capture must not have executed anything"
        t1 = time.perf_counter()
        ev0.record()
        graph.replay()
        ev1.record()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t1
    else:
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ev0.record()
        for s in range(K_seg):
            segment(step0 + s * SEG)
        ev1.record()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t1
    gpu_ms = ev0.elapsed_time(ev1)
    assert int(ctx_d[0]) == L0 + n_dec, "state did not advance as scheduled"
    # spread of the timed region: the same graph replayed a few more times from the same state (untimed for
    # `value`; GPU events around each replay)
    spread = None
    if args.launch == "graph":
        reps_ms = []
        for _ in range(7):
            ctx_d.copy_(state[0])
            rs_d.copy_(state[1])
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            graph.replay()
            e1.record()
            torch.cuda.synchronize()
            reps_ms.append(e0.elapsed_time(e1))
        assert int(ctx_d[0]) == L0 + n_dec
        reps_ms = np.sort(np.array(reps_ms))
        spread = {"n": len(reps_ms), "median_ms": float(np.median(reps_ms)), "min_ms": float(reps_ms[0]),
                  "max_ms": float(reps_ms[-1]), "p10_ms": float(np.percentile(reps_ms, 10)),
                  "p90_ms": float(np.percentile(reps_ms, 90))}
    total_s = wall
    tokens = B * SEG * K_seg * NL
    value = tokens / total_s

    # ---- per-kernel times: every kernel bracketed by HIP events on the launch stream (recorded by the
    # library into a ring, read back after the pass: no host sync between the profiled calls).  Slow and
    # fast calls are recorded in separate passes over all virtual layers, at the context the timed
    # region ended on.
    step_p = step0 + K_seg * SEG

    def stage_avg_ms(fn, reps):
        sfi.sfi_set_profiling(h, 2 * reps * NL)
        for r in range(reps):
            for l in range(NL):
                fn(l, step_p + r)
        torch.cuda.synchronize()
        ms_sum, cnt = sfi.sfi_stage_times(h)
        sfi.sfi_set_profiling(h, 0)
        return np.array(ms_sum) / np.maximum(np.array(cnt), 1)

    def stream_avg_ms(fn, reps):
        """Average duration of a call whose work is one kernel: two events around reps x NL launches in a row
        on the launch stream (what the kernel costs inside a stream of dependent kernels, as a trace shows it)."""
        for l in range(NL):
            fn(l, step_p)
        ea, eb = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ea.record()
        for r in range(reps):
            for l in range(NL):
                fn(l, step_p + r)
        eb.record()
        torch.cuda.synchronize()
        return ea.elapsed_time(eb) / (reps * NL)

    def graph_avg_ms(fn, reps):
        """The same average with the reps x NL launches captured into one HIP graph and replayed: no host call sits
        between two launches, so launches shorter than the host's launch rate are timed correctly too."""
        for l in range(NL):
            fn(l, step_p)
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        g = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            g.capture_begin()
            for r in range(reps):
                for l in range(NL):
                    fn(l, step_p + r)
            g.capture_end()
        torch.cuda.current_stream().wait_stream(side)
        g.replay()
        torch.cuda.synchronize()
        ea, eb = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ea.record()
        g.replay()
        eb.record()
        torch.cuda.synchronize()
        return ea.elapsed_time(eb) / (reps * NL)

    slow_ms = stage_avg_ms(slow, 2)
    fast_ms = stage_avg_ms(fast, 8)
    fast_bracketed_us = float(fast_ms[0] * 1e3)
    if fast_ms[1] == 0.0:  # the fast step is a single kernel (merge on board): time it without the event pair per launch
        fast_ms[0] = graph_avg_ms(fast, 8)
    L_mid = L0 + step_p
    dense_bytes = B * Hkv * L_mid * d * 2 * 2
    nsel_mean = float(torch.stack(nsels).float().mean())
    fast_rows = w.n_sink + nsel_mean + w.recent
    fast_bytes = B * Hkv * fast_rows * d * 2 * 2
    dense_gbs = dense_bytes / (slow_ms[0] * 1e-3) / 1e9
    fast_gbs = fast_bytes / (fast_ms[0] * 1e-3) / 1e9
    # the kernel with the largest share of a segment's time is the one the roofline object describes
    seg_dense_ms = slow_ms[0]
    seg_fast_ms = fast_ms[0] * (SEG - 1)
    fast_kernel = "compact" if compact else "gather"
    dominant = fast_kernel if seg_fast_ms > seg_dense_ms else "dense"
    # HBM bytes per launch: from the committed counter profile of this workload, if it was taken on these kernel sources
    traffic, traffic_source = None, "not measured in this run (counters need the profiler); no committed counter profile of this workload"
    if args.workload == "llama8b" and args.ctx == 32768 and args.batch == 4 and not compact:
        traffic, traffic_source = committed_traffic("attn_gather_stream_kernel" if dominant != "dense" else "attn_dense_kernel")
    # The floor of the fast-step launch: its memory skeleton (same grid, scalars, indices and row loads, same record
    # hand-over, no arithmetic), timed the same way, and the shorter chains underneath it.
    floor = None
    if not compact and not args.page_size:
        def skeleton(variant):
            return lambda l, step: sfi.sfi_fast_step_floor(h, q_all[step, l], Ks[l], Vs[l], sels[l], nsels[l], w.budget, rs_d,
                                                            ctx_d, outs[l], variant)
        floor = {"loads_and_record_handover_us": float(graph_avg_ms(skeleton(1), 8) * 1e3),
                 "loads_only_us": float(graph_avg_ms(skeleton(0), 8) * 1e3),
                 "scalars_and_indices_only_us": float(graph_avg_ms(skeleton(4), 8) * 1e3),
                 "bare_launch_us": float(graph_avg_ms(skeleton(8), 8) * 1e3)}
        fast(0, step_p)  # leave real outputs behind
    # the dense launch's streaming ceiling: its memory skeleton (same grid and tile dealing, loads only, no logits
    # written), with K rows requested in the kernel's own layout and as whole 128-byte lines
    dense_floor = None
    if not args.page_size:
        dskel = lambda v: (lambda l, step: sfi.sfi_dense_attn_floor(h, Ks[l], Vs[l], ctx_d, max_ctx, v))
        dense_floor = {"kernel_k_layout_us": float(graph_avg_ms(dskel(0), 2) * 1e3),
                       "whole_line_k_us": float(graph_avg_ms(dskel(1), 2) * 1e3),
                       # the same with every wave asleep 2 x 1024 cycles per tile, where the kernel has its arithmetic
                       "kernel_k_layout_with_2048_idle_cycles_per_tile_us": float(graph_avg_ms(dskel(0 + 16 * 16), 2) * 1e3),
                       # the same with a fifth wave per workgroup that stores what the slow step would expose (G x 128
                       # bytes per tile) while the four waves read; and with all those stores going to the same 2 KB
                       "kernel_k_layout_with_a_writer_wave_us": float(graph_avg_ms(dskel(2048), 2) * 1e3),
                       "kernel_k_layout_with_a_writer_wave_on_2KB_us": float(graph_avg_ms(dskel(4096), 2) * 1e3),
                       # what exposing the logits to the Selector costs: dense attention + merge launch without them
                       # (sfi_dense_attn) and with them (sfi_slow_attn), both timed like the skeletons
                       "attention_and_merge_without_logits_us": float(graph_avg_ms(
                           lambda l, step: sfi.sfi_dense_attn(h, q_all[step, l], Ks[l], Vs[l], ctx_d, max_ctx, outs[l]), 2) * 1e3),
                       "attention_and_merge_with_logits_us": float(graph_avg_ms(
                           lambda l, step: sfi.sfi_slow_attn(h, q_all[step, l], Ks[l], Vs[l], ctx_d, max_ctx, outs[l]), 2) * 1e3)}
    roof = {
        "bound": "hbm", "kernel": f"sfi::attn_{dominant}_kernel",
        "achieved": fast_gbs if dominant != "dense" else dense_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": (fast_gbs if dominant != "dense" else dense_gbs) / HBM_PEAK_GBS, "traffic": traffic,
        "traffic_source": traffic_source,
        "algorithmic_bytes_per_launch": fast_bytes if dominant != "dense" else dense_bytes,
        "us_per_launch": float((fast_ms[0] if dominant != "dense" else slow_ms[0]) * 1e3),
    }
    if floor is not None and dominant != "dense":
        # what the launch shape costs with the matrix and vector units idle, and how close the kernel is to it
        roof["floor_us"] = floor["loads_and_record_handover_us"]
        roof["frac_of_floor"] = floor["loads_and_record_handover_us"] / roof["us_per_launch"]
        roof["floor_frac_of_peak"] = fast_bytes / (floor["loads_and_record_handover_us"] * 1e-6) / 1e9 / HBM_PEAK_GBS
        roof["floor_without_handover_frac_of_peak"] = fast_bytes / (floor["loads_only_us"] * 1e-6) / 1e9 / HBM_PEAK_GBS
    dsp, fsp = sfi.sfi_query_splits(h)
    # SFI_GUARD_* bits the kernels raised since the contexts were created: 0 = no length, count, stored index
    # or block id of the run had to be clamped
    device_status = 0
    for c in ring:
        device_status |= sfi.sfi_device_status(c.handle)
    # fewer workgroups per pair than one tile per wave needs: the pipelined gather kernel ran
    fast_tiles = -(-(w.n_sink + w.budget + w.recent) // 32)
    if not compact and fsp * 4 < fast_tiles and roof["kernel"] == "sfi::attn_gather_kernel":
        roof["kernel"] = "sfi::attn_gather_stream_kernel"
    res = {
        "metric": "decode attn tokens/s (slow+fast mix)", "value": value, "unit": "tokens/s per attention layer",
        "n_gpus": 1, "steps": K_seg, "warmup": W_seg, "ms_per_step": total_s * 1e3 / K_seg,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"{wl['label']}: B{B} Hq{Hq} Hkv{Hkv} d{d} ctx{L0} k{w.budget} R{w.recent} "
                               f"sink{w.n_sink} slow every {SEG}",
                   "step": f"{SEG} decode steps (1 slow + {SEG - 1} fast) x {NL} virtual layers",
                   "virtual_layers": NL, "launch": args.launch, "out_dtype": "bf16" if args.out_bf16 else "fp32", "kv_layout": args.kv_layout, "fast_path": args.fast_path, "selector_mode": args.selector_mode, "page_size": args.page_size, "page_layout": args.page_layout if args.page_size else None,
                   "slow_schedule": args.slow_schedule + (f" (ring {len(ring)})" if use_async else ""),
                   "dense_splits": dsp, "fast_splits": fsp,
                   "fast_merge": args.fast_merge or "kernel"},
        "roofline": roof,
        "kernels": {
            "dense_attn": {"us": slow_ms[0] * 1e3, "kv_bytes": dense_bytes, "GBps": dense_gbs,
                           "frac_of_8TBps": dense_gbs / HBM_PEAK_GBS, "us_is": "event pair around the launch (about 2 us above the trace's duration)",
                           "memory_skeleton_us": dense_floor,
                           # what this machine streams when nothing is computed (the whole-line skeleton), beside the nominal peak
                           "streaming_read_ceiling_GBps": dense_bytes / (dense_floor["whole_line_k_us"] * 1e-6) / 1e9 if dense_floor else None,
                           "frac_of_streaming_read_ceiling": dense_gbs / (dense_bytes / (dense_floor["whole_line_k_us"] * 1e-6) / 1e9) if dense_floor else None},
            f"{fast_kernel}_attn": {"us": fast_ms[0] * 1e3, "kv_bytes": fast_bytes, "GBps": fast_gbs,
                            "frac_of_8TBps": fast_gbs / HBM_PEAK_GBS,
                            "us_with_an_event_pair_per_launch": fast_bracketed_us},
            "slow_step_stage_us": {n: float(slow_ms[i] * 1e3) for i, n in enumerate(sfi.binding.STAGE_NAMES)
                                   if i < 6 or (compact and n == "reorg")},
            "fast_step_stage_us": {n: float(fast_ms[i] * 1e3) for i, n in enumerate(sfi.binding.STAGE_NAMES[:2])},
            "fast_step_floor_us": floor,
        },
        "us_per_decode_step_per_layer": total_s * 1e6 / (K_seg * SEG * NL),
        "gpu_event_ms": gpu_ms,
        "timed_region_repeats": spread,
        "parity_sample": parity,
        "device_status": device_status,
        "cpu_baseline": cpu_baseline,
    }
    for c in ring:
        c.close()
    del Ks, Vs, K0, V0, q_all
    torch.cuda.empty_cache()
    return res


if __name__ == "__main__":
    main()
