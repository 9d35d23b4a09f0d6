#!/usr/bin/env python3
"""Benchmark of the Orthrus dual-view decode step's hot path on one MI355X.

One step = diffusion-view block attention + AR-view verification attention over the same paged
KV cache + greedy consensus + in-place commit of the accepted tokens' K/V (one attention layer,
synthetic seeded inputs resident in HBM before the timed region).  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload long|layer8b|mixed|stress|tiny]

Multi-GPU runs are not part of this build: --gpus above 1 exits with a message.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E published peak
N_SETS = 4              # rotating sets of block inputs / logits (fresh data every step, cycled)


def measured_traffic(workload, block_k, splits, algorithmic_bytes):
    """HBM bytes per attention call from the rocprofv3 --pmc summary committed for this very configuration.

    A summary under profiles/ that was made from FETCH_SIZE / WRITE_SIZE runs of this script carries a line
    `traffic-per-call: workload=<w> block_k=<K> splits=<S> read_bytes=<n> write_bytes=<n> algorithmic_bytes=<n>`
    (counters of the split and combine kernels, scaled by what they read for a plain copy of known size, and the
    algorithmic K/V bytes of a call at the lengths of those counter runs).  The figure returned is that measured /
    algorithmic ratio applied to this run's algorithmic bytes (the cache grows from step to step).  No such line
    for the configuration at hand: null.
    """
    import glob
    import re
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.md"))):
        for line in open(path):
            m = re.match(r"\s*traffic-per-call: workload=(\S+) block_k=(\d+) splits=(\S+) read_bytes=(\d+) "
                         r"write_bytes=(\d+) algorithmic_bytes=(\d+)", line)
            if m and m.group(1) == workload and int(m.group(2)) == block_k and m.group(3) == str(splits) \
                    and int(m.group(6)) > 0:
                ratio = (int(m.group(4)) + int(m.group(5))) / float(m.group(6))
                return {"traffic": int(ratio * algorithmic_bytes), "traffic_over_algorithmic": round(ratio, 4),
                        "traffic_source": os.path.relpath(path, ROOT)}
    return {"traffic": None, "traffic_over_algorithmic": None, "traffic_source": None}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="long")
    ap.add_argument("--num-splits", default="workload",
                    help="workload: the workload's setting; 0: library chooses; N: fixed splits; "
                         "balanced: even partition of the batch's tiles over the resident workgroups")
    ap.add_argument("--temperature", type=float, default=0.0,
                    help="0: greedy consensus (Eq. 8); > 0: lossless sampling consensus at that temperature")
    ap.add_argument("--paging", default="", help="override the workload's page-table layout: contiguous|shuffled|scattered")
    ap.add_argument("--layers", type=int, default=1,
                    help="> 1 (or --graph): time whole decode cycles over a stack of layers: the diffusion pass "
                         "through every layer, the AR pass through every layer, consensus + commit into all of them")
    ap.add_argument("--graph", action="store_true", help="replay each cycle as one HIP graph instead of eager launches")
    ap.add_argument("--diffusion-passes", type=int, default=1,
                    help="with --layers/--graph: diffusion-view passes per cycle (2 = the paper's multi-step ablation)")
    ap.add_argument("--block-k", type=int, default=0, help="override the workload's block size K (latency-vs-K sweeps)")
    ap.add_argument("--prefill", type=int, default=0,
                    help="> 0: time orthrus_prefill_attn (AR prefill of one layer) for that many new tokens per "
                         "sequence on an empty cache, with the workload's head shapes and batch")
    ap.add_argument("--train-mask", type=int, default=0,
                    help="> 0: time the diffusion view's training block-mask forward (Eq. 6) for that many packed "
                         "sequences of 2048 tokens with 256 anchor blocks of K=32 each (the paper's training "
                         "geometry), with the workload's head shapes")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--prewarm-ms", type=float, default=600.0,
                    help="untimed attention-only steps issued for this long before the warm-up steps, so that the "
                         "GPU clocks have settled when the timed region starts")
    ap.add_argument("--kernel-steps", type=int, default=48,
                    help="whole steps run after the timed region with HIP events attached to the attention "
                         "kernels (two attention calls each; 0: no kernel timing, no roofline)")
    ap.add_argument("--repeats", type=int, default=5,
                    help="the timed region is run this many times in all, each from the same cache lengths (the "
                         "first is `value`; all of them and their median go to detail.repeats); 1 = no repeat")
    ap.add_argument("--kernel-every", type=int, default=1,
                    help="attach the events to every Nth of those steps only")
    ap.add_argument("--ceiling-launches", type=int, default=50,
                    help="launches of the no-arithmetic K/V stream probe that measure the ceiling")
    ap.add_argument("--no-prescribed-splits", action="store_true",
                    help="long workload: skip the side-by-side timing of the 64-split plan the workload names "
                         "(counter runs, where its launches would be averaged into the same kernel name)")
    ap.add_argument("--pools", type=int, default=0,
                    help="copies of the cache to rotate over (0: 4 for a workload without a commit step, else 1)")
    ap.add_argument("--calibrate-read", action="store_true",
                    help="only time the no-arithmetic K/V stream probe on the workload's cache (the measured "
                         "ceiling of the paged read pattern) and print it")
    ap.add_argument("--calibrate-after-steps", type=int, default=0,
                    help="with --calibrate-read: run this many whole steps first (ragged, grown lengths)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain 1 GiB device-to-device copy a few times (known traffic, used to "
                         "scale the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    return ap.parse_args()


def settle_clocks(torch, ms, one):
    """Issues `one()` (a state-preserving launch sequence) for about `ms` milliseconds, untimed: after idle the
    GPU needs tens of milliseconds of load before its clocks reach their steady state."""
    t0, n = time.perf_counter(), 0
    while (time.perf_counter() - t0) * 1e3 < ms:
        for _ in range(10):
            one()
            n += 1
        torch.cuda.synchronize()
    return n


def cpu_baseline(w, cache, host_sets, cons_sets):
    """Times the CPU oracle, as it stands, on whole steps of the same workload (initial cache lengths).

    One oracle step = both attention views over every sequence + consensus (consensus only: the
    commit is a few KB of copies).  Steps are repeated until about 10 s have passed (at most 5).
    """
    import oracle
    cores = oracle.num_threads()
    pools = (cache["k_pool"], cache["v_pool"], cache["page_table"], cache["seq_lens"])
    times = []
    t_all = time.perf_counter()
    for rep in range(5):
        d, a = host_sets[rep % len(host_sets)]
        t0 = time.perf_counter()
        oracle.dual_view_attn(oracle.VIEW_DIFFUSION, w.sm_scale, d["q"], d["k_blk"], d["v_blk"], *pools)
        oracle.dual_view_attn(oracle.VIEW_AR_VERIFY, w.sm_scale, a["q"], a["k_blk"], a["v_blk"], *pools)
        if cons_sets:
            cs = cons_sets[rep % len(cons_sets)]
            if "diff_logits" in cs:
                oracle.sampling_consensus_commit(cs["ar_logits"], cs["diff_logits"], cs["draft_tokens"],
                                                 cs["accept_u"], cs["gumbel"], cs["temperature"])
            else:
                oracle.consensus_commit(cs["ar_logits"], cs["draft_tokens"])
        times.append(time.perf_counter() - t0)
        log("oracle step %d: %.2f s" % (rep, times[-1]))
        if time.perf_counter() - t_all > 10.0:
            break
    mean = sum(times) / len(times)
    return {"value": round(1.0 / mean, 4), "unit": "steps/s", "cores": cores, "kind": "oracle",
            "sample": "%d whole step(s) of the same workload at the initial cache lengths: both attention views "
                      "over all %d sequences%s; mean %.2f s per step" %
                      (len(times), w.batch, " + consensus" if cons_sets else "", mean)}


def run_prefill(args, torch, rt, w):
    """AR prefill attention of one layer: T new tokens per sequence on an empty cache (Section 3.1)."""
    import oracle
    from orthrus_inputs import f32_to_bf16_bits, make_cache
    T, B = args.prefill, w.batch
    w = w.with_(context=0, context_range=None, steps=(T + w.block_k - 1) // w.block_k + 1)
    cache = make_cache(w)
    rng = np.random.default_rng(w.seed + 77)
    mk = lambda h: f32_to_bf16_bits(rng.standard_normal((B, T, h, w.head_dim), dtype=np.float32))
    hq, hk, hv = mk(w.num_q_heads), mk(w.num_kv_heads), mk(w.num_kv_heads)
    D = rt.to_device_bits
    q, kn, vn = D(hq), D(hk), D(hv)
    k_pool, v_pool = D(cache["k_pool"]), D(cache["v_pool"])
    page_table = D(cache["page_table"])
    new_lens = torch.full((B,), T, dtype=torch.int32, device="cuda:0")
    zero = torch.zeros((B,), dtype=torch.int32, device="cuda:0")
    seq_lens = zero.clone()
    out = torch.empty_like(q)
    step = rt.DecodeStep(batch=B, num_q_heads=w.num_q_heads, num_kv_heads=w.num_kv_heads, head_dim=w.head_dim,
                         block_k=w.block_k, page_size=w.page_size, max_pages_per_seq=cache["page_table"].shape[1],
                         max_seq_len=T, num_pages=cache["num_pages"])
    stream = torch.cuda.current_stream()

    def one():
        seq_lens.copy_(zero)   # every timed call prefills the same empty cache again
        step.prefill(T, q, kn, vn, new_lens, k_pool, v_pool, page_table, seq_lens, out)
    settle_clocks(torch, args.prewarm_ms, one)
    for _ in range(args.warmup):
        one()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(args.steps):
        one()
    e1.record(stream)
    torch.cuda.synchronize()
    if step.device_error() != 0:
        log("bench.py: device error after the timed region")
        sys.exit(4)
    ms = e0.elapsed_time(e1) / args.steps
    # 2 contractions x 2 flop per multiply-add x d per (query, visible key) pair, causal: T(T+1)/2 pairs
    flops = 4.0 * w.head_dim * w.num_q_heads * B * (T * (T + 1) / 2.0)
    tf = flops / (ms * 1e-3) / 1e12
    res = {
        "metric": "AR prefill attention of one layer (causal, paged), whole call", "value": round(B * T / (ms * 1e-3), 1),
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s head shapes, prefill of %d tokens x %d sequences on an empty cache" % (w.name, T, B),
                   "batch": B, "num_q_heads": w.num_q_heads, "num_kv_heads": w.num_kv_heads, "head_dim": w.head_dim,
                   "page_size": w.page_size, "new_tokens": T},
        "roofline": {"bound": "mfma", "achieved": round(tf, 1), "peak": 2500.0, "unit": "TFLOP/s",
                     "frac": round(tf / 2500.0, 4), "traffic": None,
                     "kernel": "orthrus_prefill_attn = plan + append + attn_split_kernel (prefill form); ordinary "
                               "events around the whole call, so launch gaps are inside",
                     "avg_launch_us": round(ms * 1e3, 2), "algorithmic_flops_per_launch": int(flops)},
    }
    if not args.no_cpu_baseline:
        n = min(T, 256)   # bounded sample: the first n tokens of every sequence
        c = np.ascontiguousarray
        t0 = time.perf_counter()
        oracle.prefill_attn(w.sm_scale, c(hq[:, :n]), c(hk[:, :n]), c(hv[:, :n]), np.full(B, n, np.int32),
                            cache["k_pool"].copy(), cache["v_pool"].copy(), cache["page_table"],
                            np.zeros(B, np.int32))
        dt = time.perf_counter() - t0
        res["cpu_baseline"] = {"value": round(B * n / dt, 1), "unit": "tokens/s", "cores": oracle.num_threads(),
                               "kind": "oracle", "sample": "prefill of the first %d tokens of each sequence "
                               "(cost grows with the square of the length: not comparable beyond that)" % n}
    step.close()
    print(json.dumps(res), flush=True)


def run_train_mask(args, torch, rt, w, splits):
    """Forward of the diffusion view under the training block mask (Section 3.2 Eq. 6, Appendix A geometry):
    every anchor block is one batch entry of orthrus_dual_view_attn(DIFFUSION) over the clean context before
    its anchor; the context's K/V stay in their plain [tokens, H_kv, d] layout (described by the pool strides)."""
    from orthrus_inputs import f32_to_bf16_bits
    NS, L, NB, K, P = args.train_mask, 2048, 256, 32, 16
    Hq, Hkv, d = w.num_q_heads, w.num_kv_heads, w.head_dim
    rng = np.random.default_rng(w.seed + 99)
    mk = lambda n, h: f32_to_bf16_bits(rng.standard_normal((n, h, d), dtype=np.float32))
    D = rt.to_device_bits
    anchors = np.sort(rng.integers(1, L + 1, size=(NS, NB)), axis=1).astype(np.int32)
    pages = L // P
    page_table = (np.arange(NS, dtype=np.int32)[:, None, None] * pages +
                  np.arange(pages, dtype=np.int32)[None, None, :]).repeat(NB, axis=1).reshape(NS * NB, pages)
    q = D(mk(NS * NB * K, Hq).reshape(NS * NB, K, Hq, d))
    kd, vd = (D(mk(NS * NB * K, Hkv).reshape(NS * NB, K, Hkv, d)) for _ in range(2))
    k_ar, v_ar = D(mk(NS * L, Hkv)), D(mk(NS * L, Hkv))
    out = torch.empty_like(q)
    step = rt.DecodeStep(batch=NS * NB, num_q_heads=Hq, num_kv_heads=Hkv, head_dim=d, block_k=K, page_size=P,
                         max_pages_per_seq=pages, max_seq_len=L, num_pages=NS * pages, num_splits=splits,
                         pool_strides=(0, P * Hkv * d, d, Hkv * d))
    pt, sl = D(np.ascontiguousarray(page_table)), D(anchors.reshape(-1))
    stream = torch.cuda.current_stream()
    one = lambda: step.attn(0, q, kd, vd, k_ar, v_ar, pt, sl, out)
    settle_clocks(torch, args.prewarm_ms, one)
    for _ in range(args.warmup):
        one()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(args.steps):
        one()
    e1.record(stream)
    torch.cuda.synchronize()
    if step.device_error() != 0:
        sys.exit(4)
    ms = e0.elapsed_time(e1) / args.steps
    pairs = float((anchors.astype(np.int64) + K).sum()) * K           # (query, visible key) pairs per query head
    flops = 4.0 * d * Hq * pairs
    tf = flops / (ms * 1e-3) / 1e12
    print(json.dumps({
        "metric": "diffusion-view training block-mask attention forward (Eq. 6)", "value": round(NS * L / (ms * 1e-3), 1),
        "unit": "packed tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%d packed sequences of %d tokens, %d anchor blocks of K=%d each, %s head shapes" %
                               (NS, L, NB, K, w.name), "num_q_heads": Hq, "num_kv_heads": Hkv, "head_dim": d,
                   "num_splits": "balanced" if splits == -1 else step.num_splits},
        "roofline": {"bound": "mfma", "achieved": round(tf, 1), "peak": 2500.0, "unit": "TFLOP/s",
                     "frac": round(tf / 2500.0, 4), "traffic": None,
                     "kernel": "orthrus_dual_view_attn(DIFFUSION) with one batch entry per anchor block",
                     "avg_launch_us": round(ms * 1e3, 2), "algorithmic_flops_per_launch": int(flops)}}), flush=True)
    step.close()


def run_stack(args, torch, rt, w, cache, host_sets, cons_sets, splits):
    """Whole decode cycles over --layers layers (Fig. 2(b)): eager launches or one HIP graph per cycle.

    The layers share one layer's synthetic cache and block inputs (replicated on the device: values do
    not change the timing); the N_SETS rotating input sets are N_SETS stacks over the same pools.
    """
    T, nl = args.temperature, args.layers
    B, K = w.batch, w.block_k
    D = rt.to_device_bits
    rep = lambda t: t.unsqueeze(0).repeat(nl, *([1] * t.dim())).contiguous()
    k_pool, v_pool = rep(D(cache["k_pool"])), rep(D(cache["v_pool"]))
    page_table, seq_lens = D(cache["page_table"]), D(cache["seq_lens"])
    cap = min(w.capacity_tokens(), cache["page_table"].shape[1] * w.page_size)
    stacks = []
    for i in range(N_SETS):
        st = rt.DecodeStack(num_layers=nl, batch=B, num_q_heads=w.num_q_heads, num_kv_heads=w.num_kv_heads,
                            head_dim=w.head_dim, block_k=K, page_size=w.page_size, k_pool=k_pool, v_pool=v_pool,
                            page_table=page_table, seq_lens=seq_lens, max_seq_len=cap, vocab=w.vocab,
                            num_splits=splits, temperature=T, diffusion_passes=args.diffusion_passes)
        d, a = host_sets[i]
        for name, blk, key in (("q_diff", d, "q"), ("k_blk_diff", d, "k_blk"), ("v_blk_diff", d, "v_blk"),
                               ("q_ar", a, "q"), ("k_blk_ar", a, "k_blk"), ("v_blk_ar", a, "v_blk")):
            getattr(st, name).copy_(rep(D(blk[key])))
        cs = cons_sets[i]
        for name in ("ar_logits", "draft_tokens") + (("diff_logits", "accept_u", "gumbel") if T > 0 else ()):
            getattr(st, name).copy_(D(cs[name]))
        stacks.append(st)
    torch.cuda.synchronize()
    stream = torch.cuda.Stream()
    if args.graph:
        for st in stacks:
            st.capture()
    with torch.cuda.stream(stream):
        def run(i):
            st = stacks[i % N_SETS]
            if args.graph:
                st.replay(stream)
            else:
                st.cycle(stream)
        st0 = stacks[0]
        settle_clocks(torch, args.prewarm_ms,
                      lambda: st0.step.attn(0, st0.q_diff[0], st0.k_blk_diff[0], st0.v_blk_diff[0], st0.k_pool[0],
                                            st0.v_pool[0], st0.page_table, st0.seq_lens, st0.out_diff[0], None,
                                            stream))
        for i in range(args.warmup):
            run(i)
        stream.synchronize()
        lens_before = seq_lens.cpu().numpy().astype(np.int64)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for i in range(args.steps):
            run(args.warmup + i)
        e1.record(stream)
        stream.synchronize()
    total_ms = e0.elapsed_time(e1)
    lens_after = seq_lens.cpu().numpy().astype(np.int64)
    err = max(abs(st.step.device_error()) for st in stacks)
    if err != 0:
        log("bench.py: device error word -%d after the timed region" % err)
        sys.exit(4)
    ms = total_ms / args.steps
    mean_tokens = 0.5 * (lens_before.sum() + lens_after.sum())
    kv_bytes = mean_tokens * w.num_kv_heads * 2 * w.head_dim * 2          # one attention call
    committed = float((lens_after - lens_before).sum()) / args.steps       # tokens per cycle, whole batch
    passes = args.diffusion_passes + 1   # forward passes per cycle: the diffusion view's, then the AR view's
    whole = passes * nl * kv_bytes / (ms * 1e-3) / 1e9
    out = {
        "metric": "draft+verify block-attn steps/s and achieved KV-read HBM TB/s (1 MI355X)",
        "value": round(1000.0 / ms, 2), "unit": "steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "description": w.description, "batch": B, "num_q_heads": w.num_q_heads,
                   "num_kv_heads": w.num_kv_heads, "head_dim": w.head_dim, "block_k": K,
                   "context": int(lens_before.max()), "page_size": w.page_size, "vocab": w.vocab,
                   "num_splits": stacks[0].step.num_splits, "layers": nl, "graph": bool(args.graph), "temperature": T,
                   "diffusion_passes": args.diffusion_passes,
                   "step": "one decode cycle: %d diffusion attn + %d AR verify attn + consensus + commit into "
                           "%d layers" % (nl * args.diffusion_passes, nl, nl)},
        "roofline": {"bound": "hbm", "achieved": round(whole, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(whole / HBM_PEAK_GBS, 4), "traffic": None,
                     "kernel": "whole cycle (all attention launches + consensus + commit), not one kernel: "
                               "algorithmic KV bytes of the %d attention calls over the cycle time" % (passes * nl),
                     "avg_launch_us": round(ms * 1e3 / (passes * nl), 2), "algorithmic_bytes_per_launch": int(kv_bytes)},
        "detail": {"tokens_per_s": round(committed / (ms * 1e-3), 1),
                   "tokens_committed_per_cycle_per_sequence": round(committed / max(B, 1), 3),
                   "tokens_per_forward_pass": round(committed / max(B, 1) / passes, 3),
                   "cycle_us_per_layer": round(ms * 1e3 / nl, 2)},
    }
    for st in stacks:
        st.close()
    print(json.dumps(out), flush=True)


def main():
    args = parse()
    if args.gpus != 1:
        log("bench.py: this build measures one MI355X only (no collectives or sharding are part of it); "
            "--gpus %d is not supported" % args.gpus)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        log("bench.py: no HIP device visible; the hot path has no CPU fallback")
        sys.exit(3)
    if args.calibrate_copy:
        n = 1 << 30
        src = torch.empty(n, dtype=torch.uint8, device="cuda:0").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_read": n, "calibrate_copy_bytes_written": n, "launches": 5}))
        return
    from orthrus_inputs import WORKLOADS, make_block, make_cache, make_consensus_case, make_sampling_case
    from paper_2605_12825_amd import runtime as rt

    total_steps = args.warmup + args.steps
    w = WORKLOADS[args.workload]
    if args.block_k > 0:
        w = w.with_(block_k=args.block_k)
    # capacity: the cache grows by <= K tokens per committed step (never, for a workload without consensus)
    w = w.with_(steps=(total_steps + args.kernel_steps + 1) if w.vocab else 0)
    if args.paging:
        w = w.with_(paging=args.paging)
    splits = {"workload": w.num_splits, "balanced": -1}.get(args.num_splits)
    if splits is None:
        splits = int(args.num_splits)
    if args.prefill > 0:
        run_prefill(args, torch, rt, WORKLOADS[args.workload])
        return
    if args.train_mask > 0:
        run_train_mask(args, torch, rt, WORKLOADS[args.workload], 0 if args.num_splits == "workload" else splits)
        return
    t_gen = time.perf_counter()
    cache = make_cache(w)
    host_sets = []
    for i in range(N_SETS):
        base = w.seed * 1000 + 10 * i
        host_sets.append((make_block(w, base + 1), make_block(w, base + 2)))
    T = args.temperature
    if not w.vocab:
        cons_sets = []
    elif T > 0:
        cons_sets = [make_sampling_case(w, w.seed * 1000 + 10 * i + 3, temperature=T) for i in range(N_SETS)]
    else:
        cons_sets = [make_consensus_case(w, w.seed * 1000 + 10 * i + 3) for i in range(N_SETS)]
    log("generated %s inputs in %.1f s" % (w.name, time.perf_counter() - t_gen))
    if args.layers > 1 or args.graph:
        if not w.vocab:
            log("bench.py: --layers/--graph time whole cycles and need a workload with a consensus step")
            sys.exit(2)
        run_stack(args, torch, rt, w, cache, host_sets, cons_sets, splits)
        return

    dev = torch.device("cuda:0")
    D = rt.to_device_bits
    # Workloads without a commit step may rotate over several copies of the cache, so that the last-level
    # cache (256 MB) cannot serve a pass from what the previous one left there.
    n_pools = args.pools if args.pools > 0 else (4 if not w.vocab else 1)
    if w.vocab and n_pools > 1:
        log("bench.py: --pools needs a workload without a commit step (the commit writes one cache)")
        sys.exit(2)
    k_pools, v_pools = [D(cache["k_pool"])], [D(cache["v_pool"])]
    for _ in range(1, n_pools):
        k_pools.append(k_pools[0].clone())
        v_pools.append(v_pools[0].clone())
    k_pool, v_pool = k_pools[0], v_pools[0]
    page_table, seq_lens = D(cache["page_table"]), D(cache["seq_lens"])
    sets = [tuple({k: D(v) for k, v in blk.items()} for blk in pair) for pair in host_sets]
    csets = [{k: D(v) for k, v in c.items() if isinstance(v, np.ndarray) and not k.startswith("planted")}
             for c in cons_sets]
    B, K = w.batch, w.block_k
    o_d = torch.empty((B, K, w.num_q_heads, w.head_dim), dtype=torch.int16, device=dev)
    o_a = torch.empty_like(o_d)
    acc, ncm, anc = (torch.empty((B,), dtype=torch.int32, device=dev) for _ in range(3))
    toks = torch.empty((B, K), dtype=torch.int32, device=dev)
    len0 = int(cache["seq_lens"].max())
    cap = min(w.capacity_tokens(), cache["page_table"].shape[1] * w.page_size)
    mk_step = lambda ns: rt.DecodeStep(batch=B, num_q_heads=w.num_q_heads, num_kv_heads=w.num_kv_heads,
                                       head_dim=w.head_dim, block_k=K, page_size=w.page_size,
                                       max_pages_per_seq=cache["page_table"].shape[1], max_seq_len=cap,
                                       num_pages=cache["num_pages"], vocab=w.vocab, num_splits=ns,
                                       min_seq_len_bound=len0)
    step = mk_step(splits)
    stream = torch.cuda.current_stream()
    call_events = []

    def attn_pair(st, i):
        d, a = sets[i % N_SETS]
        kp, vp = k_pools[i % n_pools], v_pools[i % n_pools]
        st.attn(0, d["q"], d["k_blk"], d["v_blk"], kp, vp, page_table, seq_lens, o_d)
        st.attn(1, a["q"], a["k_blk"], a["v_blk"], kp, vp, page_table, seq_lens, o_a)

    def run_step(i, record=False):
        # the host's own upper bound on the lengths: initial maximum plus K tokens per step so far
        # (no device round trip); it sizes the attention grid of this step
        step.set_max_seq_len(min(cap, len0 + (i if w.vocab else 0) * K))
        attn_pair(step, i)
        if w.vocab:
            ev = None
            if record:
                ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
                ev[0].record(stream)
            a = sets[i % N_SETS][1]
            cs = csets[i % N_SETS]
            if T > 0:
                step.sampling_consensus_commit(T, cs["ar_logits"], cs["diff_logits"], cs["draft_tokens"],
                                               cs["accept_u"], cs["gumbel"], a["k_blk"], a["v_blk"], k_pool, v_pool,
                                               page_table, seq_lens, acc, ncm, toks, anc)
            else:
                step.consensus_commit(cs["ar_logits"], cs["draft_tokens"], a["k_blk"], a["v_blk"], k_pool, v_pool,
                                      page_table, seq_lens, acc, ncm, toks, anc)
            if record:
                ev[1].record(stream)
                call_events.append(ev)

    # ---- clock settling (untimed, changes no state): after idle the GPU needs tens of milliseconds of
    # load before its clocks reach their steady state (the first launches run up to 30 % slower), and a
    # decode loop runs for seconds; so the attention calls of this workload are issued for a while first
    step.set_max_seq_len(min(cap, len0))
    pre_i = [0]

    def pre_one():
        attn_pair(step, pre_i[0])
        pre_i[0] += 1
    n_pre = settle_clocks(torch, args.prewarm_ms, pre_one)

    def resettle(st):
        """The host-side work between two measurement phases (reading results back, parsing a profile, creating a
        context) leaves the GPU idle for milliseconds, enough for its clocks to drop: a short untimed run of the
        same attention calls before a phase that follows such a gap."""
        if args.prewarm_ms > 0:
            # ~60 ms of GPU work at the pace of the timed region, queued without a synchronisation, so that the
            # phase starts right behind it on the same stream
            for k in range(min(2000, max(20, int(60.0 / max(pace["ms_per_step"], 1e-3))))):
                attn_pair(st, k)
    pace = {"ms_per_step": 0.2}
    if args.calibrate_read:
        for i in range(args.calibrate_after_steps):   # optionally from the state that many whole steps reach
            run_step(i)
        torch.cuda.synchronize()
        step.attn_timing(True)
        for j in range(max(args.ceiling_launches, 1)):
            step.kv_stream_probe(k_pools[j % n_pools], v_pools[j % n_pools], page_table, seq_lens)
        step.attn_timing(False)
        torch.cuda.synchronize()
        pr = np.array([x[0] for x in step.attn_timing_samples()])
        nbytes = float(seq_lens.cpu().numpy().astype(np.int64).sum()) * w.num_kv_heads * 2 * w.head_dim * 2
        print(json.dumps({"calibrate_read": "the attention kernel with idle compute waves: the K/V loads of one attention "
                          "call over the %s cache, no arithmetic" % w.name, "bytes_per_launch": int(nbytes),
                          "launches": int(len(pr)), "avg_us": round(float(pr.mean()), 2),
                          "median_us": round(float(np.median(pr)), 2), "min_us": round(float(pr.min()), 2),
                          "max_us": round(float(pr.max()), 2),
                          "gbs": round(nbytes / (pr.mean() * 1e-6) / 1e9, 1),
                          "frac_of_peak": round(nbytes / (pr.mean() * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)}), flush=True)
        step.close()
        return
    # ---- W warm-up steps, then exactly K timed steps
    for i in range(args.warmup):
        run_step(i)
    torch.cuda.synchronize()
    lens_before = seq_lens.cpu().numpy().astype(np.int64)
    lens_start_dev = seq_lens.clone()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record(stream)
    for i in range(args.steps):
        run_step(args.warmup + i)
    e1.record(stream)
    torch.cuda.synchronize()
    total_ms = e0.elapsed_time(e1)
    pace["ms_per_step"] = total_ms / args.steps
    lens_after = seq_lens.cpu().numpy().astype(np.int64)

    # ---- kernel timing block (after the timed region, same stream, same state evolution): more whole
    # steps, now with HIP events attached to the attention kernels' own dispatches (kernel execution
    # time, no marker between kernels) and ordinary events around the consensus call
    n_post = args.kernel_steps
    samples = []
    if n_post > 0:
        for j in range(n_post):
            rec = j % args.kernel_every == 0
            step.attn_timing(rec)
            run_step(total_steps + j, record=rec)
        step.attn_timing(False)
        torch.cuda.synchronize()
        samples = step.attn_timing_samples()
    lens_post = seq_lens.cpu().numpy().astype(np.int64)

    # ---- repeats of the timed region: the lengths go back to where the region started (the commits then
    # rewrite the same rows), the same K steps run again; `value` stays the first region's
    region_ms = [total_ms / args.steps]
    lens_post_dev = seq_lens.clone()
    for _ in range(max(args.repeats, 1) - 1):
        seq_lens.copy_(lens_start_dev)
        torch.cuda.synchronize()
        r0, r1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        r0.record(stream)
        for i in range(args.steps):
            run_step(args.warmup + i)
        r1.record(stream)
        torch.cuda.synchronize()
        region_ms.append(r0.elapsed_time(r1) / args.steps)
    seq_lens.copy_(lens_post_dev)  # back to the state the blocks below describe (the rows up to there are in place)
    torch.cuda.synchronize()
    err = step.device_error()
    if err != 0:
        log("bench.py: device error word %d after the timed region" % err)
        sys.exit(4)

    ms_per_step = total_ms / args.steps
    # algorithmic KV bytes of one attention launch: 2*d*2 bytes per cached token per KV head,
    # at the mean cached length over the steps in question
    row_bytes = w.num_kv_heads * 2 * w.head_dim * 2
    kv_bytes = 0.5 * (lens_before.sum() + lens_after.sum()) * row_bytes
    kv_bytes_post = 0.5 * (lens_after.sum() + lens_post.sum()) * row_bytes
    R = w.group * K

    def stats(us):
        us = np.asarray(us, dtype=np.float64)
        return {"avg_us": round(float(us.mean()), 2), "median_us": round(float(np.median(us)), 2),
                "min_us": round(float(us.min()), 2), "max_us": round(float(us.max()), 2)}

    def rates(us_mean, nbytes):
        gbs = nbytes / (us_mean * 1e-6) / 1e9
        return {"achieved": round(gbs, 1), "frac": round(gbs / HBM_PEAK_GBS, 4)}

    roofline = None
    extra = {}
    if samples:
        sp = np.array([x[0] for x in samples])
        cb = np.array([x[1] for x in samples])
        call = sp + cb
        r_call, r_split = rates(call.mean(), kv_bytes_post), rates(sp.mean(), kv_bytes_post)
        tf = kv_bytes_post * R / (call.mean() * 1e-6) / 1e12     # R flop per K/V byte: 4 R d flop per 4 d bytes
        roofline = {"bound": "hbm", "achieved": r_call["achieved"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": r_call["frac"],
                    "kernel": "one orthrus_dual_view_attn call = attn_split_kernel" +
                              (" + attn_combine_kernel" if cb.max() > 0 else "") +
                              " (the call, not the split kernel alone, is what the fraction is of)",
                    "launches": int(len(samples)),
                    "events": "HIP events attached to the kernels' own dispatches in %d whole steps that follow "
                              "the timed region on the same stream" % n_post,
                    "avg_launch_us": stats(call)["avg_us"], "launch_us": stats(call),
                    "algorithmic_bytes_per_launch": int(kv_bytes_post),
                    "split_kernel": dict(stats(sp), **r_split),
                    "combine_kernel": stats(cb) if cb.max() > 0 else None,
                    "mfma": {"flop_per_byte": R, "achieved_tflops": round(tf, 1), "peak_tflops": 2500.0,
                             "frac": round(tf / 2500.0, 4)}}
        roofline.update(measured_traffic(w.name, K, "balanced" if splits == -1 else step.num_splits, kv_bytes_post))
        extra["attn_split_kernel_us"] = stats(sp)["avg_us"]
        extra["attn_combine_kernel_us"] = stats(cb)["avg_us"]
        extra["attn_call_kernels_us"] = stats(call)["avg_us"]
        extra["attn_call_frac_of_peak"] = r_call["frac"]
        if len(call) >= 2:  # calls alternate: diffusion view (follows the previous step's commit), AR view
            extra["attn_call_us_by_view"] = {"diffusion": round(float(call[0::2].mean()), 2),
                                             "ar_verify": round(float(call[1::2].mean()), 2)}
        # ---- the same calls back to back with nothing attached: wall time per call between two events
        # around the whole run.  Per-kernel durations include each kernel's dispatch and completion, which
        # overlap with the neighbours' in a queue of launches, so their sum (the figure above) is the larger.
        n_wall = max(8, n_post)
        w0, w1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        resettle(step)
        w0.record(stream)
        for j in range(n_wall):
            attn_pair(step, j)
        w1.record(stream)
        torch.cuda.synchronize()
        wall_us = w0.elapsed_time(w1) * 1e3 / (2 * n_wall)
        kv_wall = lens_post.sum() * row_bytes
        extra["attn_call_wall_us"] = dict(us=round(wall_us, 2), calls=2 * n_wall, **rates(wall_us, kv_wall))
        # ---- measured ceiling of the access pattern: the same bytes through the same page table, no arithmetic
        resettle(step)
        step.attn_timing(True)
        for j in range(args.ceiling_launches):
            step.kv_stream_probe(k_pools[j % n_pools], v_pools[j % n_pools], page_table, seq_lens)
        step.attn_timing(False)
        torch.cuda.synchronize()
        pr = np.array([x[0] for x in step.attn_timing_samples()])
        if len(pr):
            kv_now = lens_post.sum() * row_bytes
            c = rates(pr.mean(), kv_now)
            roofline["ceiling"] = dict(stats(pr), kernel="the attention kernel with idle compute waves (same grid, same "
                                       "K/V loads through the page table, no arithmetic)", launches=int(len(pr)),
                                       achieved=c["achieved"], frac_of_peak=c["frac"])
            roofline["ceiling_frac"] = round(r_call["achieved"] / c["achieved"], 4)
        # ---- the long workload names 64 splits per sequence: that plan, timed side by side
        if w.name == "long" and args.block_k == 0 and step.num_splits != 64 and not args.no_prescribed_splits:
            s64 = mk_step(64)
            s64.set_max_seq_len(min(cap, int(lens_post.max())))
            resettle(s64)
            s64.attn_timing(True)
            for j in range(max(8, n_post // 2)):
                attn_pair(s64, j)
            s64.attn_timing(False)
            torch.cuda.synchronize()
            x = s64.attn_timing_samples()
            sp64, cb64 = np.array([v[0] for v in x]), np.array([v[1] for v in x])
            kv_now = lens_post.sum() * row_bytes
            extra["prescribed_64_splits"] = {"split_kernel": dict(stats(sp64), **rates(sp64.mean(), kv_now)),
                                             "combine_kernel": stats(cb64),
                                             "call": dict(stats(sp64 + cb64), **rates((sp64 + cb64).mean(), kv_now)),
                                             "launches": int(len(x)), "library_choice_splits": step.num_splits}
            s64.close()
    if call_events:
        c_ms = np.array([ev[0].elapsed_time(ev[1]) for ev in call_events])
        extra["consensus_commit_us"] = round(float(c_ms.mean()) * 1e3, 2)
        nlog = 2 if T > 0 else 1
        extra["consensus_logits_gbs"] = round(nlog * B * K * w.vocab * 4 / (float(c_ms.mean()) * 1e-3) / 1e9, 1)
    extra["kv_read_tbs_whole_step"] = round(2 * kv_bytes / (ms_per_step * 1e-3) / 1e12, 3)
    extra["tokens_committed_per_step"] = round(float((lens_after - lens_before).sum()) / args.steps / max(B, 1), 3)
    extra["prewarm"] = "%d untimed attention-only steps over %.0f ms before the warm-up steps (clock settling)" % (
        n_pre, args.prewarm_ms)
    extra["pools"] = n_pools
    extra["repeats"] = {"ms_per_step": [round(x, 5) for x in region_ms],
                        "median_ms_per_step": round(float(np.median(region_ms)), 5),
                        "median_steps_per_s": round(1000.0 / float(np.median(region_ms)), 2),
                        "what": "the same %d steps from the same cache lengths, %d times; the first is `value`" % (
                            args.steps, len(region_ms))}

    out = {
        "metric": "draft+verify block-attn steps/s and achieved KV-read HBM TB/s (1 MI355X)",
        "value": round(1000.0 / ms_per_step, 2), "unit": "steps/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "description": w.description, "batch": B, "num_q_heads": w.num_q_heads,
                   "num_kv_heads": w.num_kv_heads, "head_dim": w.head_dim, "block_k": K,
                   "context": int(lens_before.max()), "page_size": w.page_size, "vocab": w.vocab,
                   "num_splits": "balanced" if splits == -1 else step.num_splits, "layers": 1, "temperature": T,
                   "step": "diffusion attn + AR verify attn" +
                           ((" + sampling consensus + commit" if T > 0 else " + greedy consensus + commit")
                            if w.vocab else "")},
        "roofline": roofline,
        "detail": extra,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, cache, host_sets, cons_sets)
    step.close()
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
