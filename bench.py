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
# HBM bytes per attn_split_kernel launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this
# script (counters scaled by what they read for a plain 1 GiB copy; see profiles/), keyed by
# (workload, splits, block size K): reads + writes of that kernel.
MEASURED_TRAFFIC_BYTES = {("long", 8, 16): int((539.08 + 8.52) * 1e6),
                          ("long", 8, 32): int((540.36 + 17.05) * 1e6),
                          ("stress", 1, 16): int((557.39 + 8.39) * 1e6),
                          ("mixed", 0, 32): int((163.48 + 38.89) * 1e6)}   # balanced partition


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
    ap.add_argument("--event-every", type=int, default=8,
                    help="time the kernels of every Nth timed step with HIP events (0: never)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain 1 GiB device-to-device copy a few times (known traffic, used to "
                         "scale the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    return ap.parse_args()


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
    w = w.with_(steps=(total_steps + 1) if w.vocab else 0)
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
    k_pool, v_pool = D(cache["k_pool"]), D(cache["v_pool"])
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
    step = rt.DecodeStep(batch=B, num_q_heads=w.num_q_heads, num_kv_heads=w.num_kv_heads, head_dim=w.head_dim,
                         block_k=K, page_size=w.page_size, max_pages_per_seq=cache["page_table"].shape[1],
                         max_seq_len=cap, num_pages=cache["num_pages"], vocab=w.vocab,
                         num_splits=splits, min_seq_len_bound=len0)
    stream = torch.cuda.current_stream()
    call_events = []

    def run_step(i, record):
        # the host's own upper bound on the lengths: initial maximum plus K tokens per step so far
        # (no device round trip); it sizes the attention grid of this step
        step.set_max_seq_len(min(cap, len0 + (i if w.vocab else 0) * K))
        d, a = sets[i % N_SETS]
        # sampled steps: the library attaches HIP events to its attention kernels' own dispatches
        # (kernel execution time, no marker between kernels); the consensus call sits between two
        # ordinary events on the same stream
        step.attn_timing(record)
        step.attn(0, d["q"], d["k_blk"], d["v_blk"], k_pool, v_pool, page_table, seq_lens, o_d)
        step.attn(1, a["q"], a["k_blk"], a["v_blk"], k_pool, v_pool, page_table, seq_lens, o_a)
        if record:
            step.attn_timing(False)
        if w.vocab:
            ev = None
            if record:
                ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
                ev[0].record(stream)
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

    for i in range(args.warmup):
        run_step(i, False)
    if args.event_every > 0:
        # let the library create the events the sampled steps will need now, outside the timed region
        # (it recycles them after a read); these untimed calls leave the cache as it is
        step.attn_timing(True)
        step.set_max_seq_len(min(cap, len0 + (args.warmup if w.vocab else 0) * K))
        d, a = sets[0]
        for _ in range((args.steps + args.event_every - 1) // args.event_every):
            step.attn(0, d["q"], d["k_blk"], d["v_blk"], k_pool, v_pool, page_table, seq_lens, o_d)
            step.attn(1, a["q"], a["k_blk"], a["v_blk"], k_pool, v_pool, page_table, seq_lens, o_a)
        step.attn_timing(False)
        step.attn_timing_read()
    torch.cuda.synchronize()
    lens_before = seq_lens.cpu().numpy().astype(np.int64)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record(stream)
    for i in range(args.steps):
        run_step(args.warmup + i, args.event_every > 0 and i % args.event_every == 0)
    e1.record(stream)
    torch.cuda.synchronize()
    total_ms = e0.elapsed_time(e1)
    lens_after = seq_lens.cpu().numpy().astype(np.int64)
    err = step.device_error()
    if err != 0:
        log("bench.py: device error word %d after the timed region" % err)
        sys.exit(4)

    ms_per_step = total_ms / args.steps
    # algorithmic KV bytes of one attention launch: 2*d*2 bytes per cached token per KV head,
    # at the mean cached length over the timed steps
    mean_tokens = 0.5 * (lens_before.sum() + lens_after.sum())
    kv_bytes = mean_tokens * w.num_kv_heads * 2 * w.head_dim * 2
    roofline = None
    extra = {}
    split_us, split_n, comb_us, comb_n = step.attn_timing_read()
    if split_n:
        split_avg = split_us / split_n
        comb_avg = comb_us / comb_n if comb_n else 0.0
        achieved = kv_bytes / (split_avg * 1e-6) / 1e9
        call_gbs = kv_bytes / ((split_avg + comb_avg) * 1e-6) / 1e9
        roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(achieved / HBM_PEAK_GBS, 4),
                    "traffic": MEASURED_TRAFFIC_BYTES.get((w.name, step.num_splits, K)),
                    "kernel": "attn_split_kernel",
                    "events": "HIP events attached to the kernel's own dispatches in every %d-th timed step "
                              "(%d launches)" % (args.event_every, split_n),
                    "avg_launch_us": round(split_avg, 2), "algorithmic_bytes_per_launch": int(kv_bytes)}
        extra["attn_split_kernel_us"] = round(split_avg, 2)
        extra["attn_combine_kernel_us"] = round(comb_avg, 2)
        extra["attn_call_kernels_us"] = round(split_avg + comb_avg, 2)
        extra["attn_call_kv_gbs"] = round(call_gbs, 1)
        extra["attn_call_frac_of_peak"] = round(call_gbs / HBM_PEAK_GBS, 4)
    if call_events:
        c_ms = np.array([ev[0].elapsed_time(ev[1]) for ev in call_events])
        extra["consensus_commit_us"] = round(float(c_ms.mean()) * 1e3, 2)
        nlog = 2 if T > 0 else 1
        extra["consensus_logits_gbs"] = round(nlog * B * K * w.vocab * 4 / (float(c_ms.mean()) * 1e-3) / 1e9, 1)
    extra["kv_read_tbs_whole_step"] = round(2 * kv_bytes / (ms_per_step * 1e-3) / 1e12, 3)
    extra["tokens_committed_per_step"] = round(float((lens_after - lens_before).sum()) / args.steps / max(B, 1), 3)

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
