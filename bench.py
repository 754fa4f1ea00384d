#!/usr/bin/env python3
"""Benchmark of the kvtrim hot path on one MI355X.

A "step" is one decode step of the long-context workload (32 layers x 8 KV heads x 32
query heads, head_dim 128, 131072 prefilled tokens, global budget 6.25 % = 2,097,152
entries): append one token per segment, score every cached entry, one global top-B
selection, stream compaction into the ragged per-(layer, head) caches, GQA decode
attention.  All inputs are synthetic, seeded and resident in HBM before the timed
region.  Prints ONE JSON line.
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
CPU_STEPS = 16                 # steps the CPU oracle replays after the timed region (a few seconds of host work)
# HBM bytes per launch of the dominant kernel from rocprofv3 --pmc FETCH_SIZE /
# WRITE_SIZE runs, scaled by a plain copy kernel; None until measured for this workload.
MEASURED_TRAFFIC = {("long", "k_cmp_attn"): 1.1011e9 + 1.1259e9, ("long", "k_cmp_copy"): None,
                    ("long-paged", "k_att_partial"): 1.0942e9 + 8.8e6, ("gate-1", "k_gate_hidden"): 136.5e6 + 65.5e3,
                    ("long-inplace", "k_cmp_attn"): 1.1012e9 + 0.2459e9}


def rows_moved_in_place(cache, keep):
    """Rows an in-place stable compaction has to write: the survivors behind the first evicted entry of their segment."""
    k = keep.cpu().numpy()
    st, ln = cache.seg_start.cpu().numpy(), cache.seg_len.cpu().numpy()
    moved = 0
    for g in range(len(st)):
        kk = k[st[g]:st[g] + ln[g]]
        ev = (kk == 0).nonzero()[0]
        if len(ev):
            moved += int(kk[ev[0]:].sum())
    return moved


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def algorithmic_bytes(w, n_cand, n_ret, horizon=1):
    """Bytes the method has to move per step (per-unit figures: 8 B/candidate for the score,
    5 B/candidate for the selection, 2*(4D+8) B per retained entry for the compaction,
    4D B per retained entry + 6D B per query head for the attention; a lookahead horizon other
    than 1 adds the 4-byte tail constant to the score's and the compaction's per-entry bytes)."""
    D = w.head_dim
    tail = 0 if horizon == 1 else 4
    R = 4 * D + 8 + tail
    return {
        "score": (8 + tail) * n_cand,
        "select": 5 * n_cand,
        "compact": 2 * R * n_ret,
        "attend": 4 * D * n_ret + 6 * D * w.n_seq * w.n_layers * w.n_q_heads,
    }


def bench_gate(args):
    """Retention-gate forward for tokens entering the cache (not part of the metric's step: there
    log beta is an input).  One JSON line of its own."""
    import numpy as np
    import torch
    import kvtrim_inputs as ki
    import paper_2605_09649_amd as kv

    dev = "cuda:0"
    torch.cuda.set_device(0)
    w = ki.workload("long")
    L, H, dm, dg, dp, n_tok = w.n_layers, w.n_kv_heads, w.n_q_heads * w.head_dim, 512, 128, args.gate
    K, W = args.steps, max(args.warmup, 1)
    wts = ki.gate_weights(L, H, dm, dg, dp, device=dev)
    gate = kv.Gate.from_dict(wts, dev)
    ctx = kv.Context(1, L, H, w.n_q_heads, w.head_dim, 1024)
    horizon = args.horizon
    xs = [ki.gate_inputs(L, n_tok, dm, device=dev, salt=i) for i in range(4)]
    scratch = torch.empty(kv.kvtrim_gate_scratch_bytes(gate, n_tok, L) // 4, dtype=torch.float32, device=dev)
    lb = torch.zeros(n_tok, L, H, dtype=torch.float32, device=dev)
    lt = torch.zeros(n_tok, L, H, dtype=torch.float32, device=dev) if horizon != 1 else None
    prepared = None
    if args.prepared:
        prepared = torch.empty(kv.kvtrim_gate_prepared_bytes(gate, L, H) // 4, dtype=torch.float32, device=dev)
        kv.kvtrim_gate_prepare(ctx, gate, prepared)

    def forward(x):
        if prepared is None:
            kv.kvtrim_gate_forward(ctx, gate, x, n_tok, 0, L, horizon, scratch, lb, lt)
        else:
            kv.kvtrim_gate_forward_prepared(ctx, gate, prepared, x, n_tok, 0, L, horizon, scratch, lb, lt)

    for i in range(W):
        forward(xs[i % 4])
    torch.cuda.synchronize()
    kv.kvtrim_profile_begin(ctx, (0x1F << 23) | (1 << 29))       # k_gate_hidden, _readout, _fold, _prefill, _retile, _dot
    t0 = time.perf_counter()
    for i in range(K):
        forward(xs[i % 4])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    prof = kv.kvtrim_profile_end(ctx)
    assert kv.kvtrim_poll_error(ctx) == 0
    ms = (t1 - t0) * 1e3 / K
    w1_bytes = L * dg * dm * 2
    w2_bytes = L * H * dp * dg * 2
    flops_hidden = 2.0 * n_tok * L * dg * dm
    if "k_gate_prefill" in prof:
        # prefill-sized call: the second layer is folded into one vector per (layer, head) and the first layer,
        # the activation and the readout run in one kernel (the dominant one, a dense contraction)
        first, second = "k_gate_prefill", "k_gate_fold"
        h_ms = prof[first][0] / prof[first][1]
        r_ms = prof[second][0] / prof[second][1] if second in prof else None    # prepared: no fold inside the call
        roof = {"bound": "mfma", "kernel": first, "achieved": flops_hidden / (h_ms * 1e-3) / 1e12,
                "peak": 2500.0, "unit": "TFLOP/s", "traffic": None, "flops_per_launch": flops_hidden}
        second_bytes = w2_bytes + L * H * (dg + 1) * 4
        if "k_gate_retile" in prof:
            t_ms = prof["k_gate_retile"][0] / prof["k_gate_retile"][1]
            roof["third_kernel"] = {"kernel": "k_gate_retile", "avg_launch_ms": t_ms,
                                    "achieved": 2 * w1_bytes / (t_ms * 1e-3) / 1e9, "unit": "GB/s"}
    else:
        first, second = "k_gate_hidden", "k_gate_dot" if "k_gate_dot" in prof else "k_gate_readout"
        h_ms = prof[first][0] / prof[first][1]
        r_ms = prof[second][0] / prof[second][1]
        # first layer: W1 once per 64 tokens of a call, x once per 16-row tile group (cached), u written once
        alg_hidden = w1_bytes + L * n_tok * dm * 2 + L * n_tok * dg * 4
        if n_tok <= 64:
            roof = {"bound": "hbm", "kernel": first, "achieved": alg_hidden / (h_ms * 1e-3) / 1e9,
                    "peak": HBM_PEAK_GBS, "unit": "GB/s", "traffic": MEASURED_TRAFFIC.get((f"gate-{n_tok}", first)),
                    "algorithmic_bytes_per_launch": alg_hidden}
        else:
            roof = {"bound": "mfma", "kernel": first, "achieved": flops_hidden / (h_ms * 1e-3) / 1e12,
                    "peak": 2500.0, "unit": "TFLOP/s", "traffic": None, "flops_per_launch": flops_hidden}
        second_bytes = (L * H * (dg + 1) * 4 if second == "k_gate_dot" else w2_bytes) + L * n_tok * dg * 4
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["avg_launch_ms"] = h_ms
    third = roof.pop("third_kernel", None)
    roof["second_kernel"] = None if r_ms is None else {"kernel": second, "avg_launch_ms": r_ms,
                                                       "achieved": second_bytes / (r_ms * 1e-3) / 1e9, "unit": "GB/s"}
    if third:
        roof["third_kernel"] = third
    log(f"[bench] gate forward{' (prepared)' if prepared is not None else ''}, {n_tok} token(s): {ms:.4f} ms/call; "
        f"{first} {h_ms * 1e3:.1f} us" + (f", {second} {r_ms * 1e3:.1f} us" if r_ms is not None else "") + (f", k_gate_retile {third['avg_launch_ms'] * 1e3:.1f} us" if third else "") +
        f"; {roof['achieved']:.0f} {roof['unit']}")
    result = {
        "metric": "retention-gate forward (32Lx8H, d_model 4096, d_g 512, d_p 128), tokens/s", "value": n_tok * 1e3 / ms,
        "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": ms, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"prepared_weights": prepared is not None,
                   "workload": f"gate forward for {n_tok} token(s) per call into all {L * H} (layer, KV head) lists; "
                               f"random weights, lookahead horizon {horizon if horizon > 0 else 'infinite'}"},
        "roofline": roof,
    }
    if not args.no_cpu_baseline:
        import oracle
        from helpers import bf16_bits
        og = oracle.Gate(bf16_bits(wts["w1"]), wts["c1"].cpu().numpy(), bf16_bits(wts["w2"]), wts["c2"].cpu().numpy(),
                         wts["w_g"].cpu().numpy(), wts["b_g"])
        ns = min(n_tok, 4)                       # bounded sample: tokens spread over the last call's input
        pick = sorted({(i * (n_tok - 1)) // max(ns - 1, 1) for i in range(ns)})
        ns = len(pick)
        x_last = xs[(K - 1) % 4][:, pick].contiguous()
        t_cpu = time.perf_counter()
        _, lb_ref, _ = oracle.gate_forward(og, bf16_bits(x_last))
        cpu_s = time.perf_counter() - t_cpu
        err = float(np.max(np.abs(lb[pick].cpu().numpy() - lb_ref) / np.abs(lb_ref)))
        log(f"[bench] oracle gate forward for {ns} token(s): {cpu_s:.2f} s; GPU vs oracle: max rel err of log beta {err:.2e}")
        assert err <= 2e-4, "GPU gate disagrees with the oracle"
        result["cpu_baseline"] = {"value": ns / cpu_s, "unit": "tokens/s", "cores": 1, "kind": "oracle",
                                  "sample": f"{ns} token(s) spread over one call, all layers and heads, one thread"}
        result["parity_on_sampled_step"] = {"log_beta_max_rel_err": err}
    print(json.dumps(result), flush=True)


def bench_chunk(args):
    """The chunked-prefill step of the multi-turn workload: every segment of all 16 sequences takes a chunk of
    CHUNK new tokens, then the cache is rescored, selected and compacted back to the per-sequence budgets (no
    attention in this step).  Starts from empty caches; the cache is at its budget after two chunks, the timed
    steps come after that.  One JSON line of its own; parity of this flow is covered by the GPU tests."""
    import numpy as np
    import torch
    import kvtrim_inputs as ki
    import paper_2605_09649_amd as kv

    dev = "cuda:0"
    torch.cuda.set_device(0)
    w = ki.workload("multiturn")
    chunk, K = args.chunk, args.steps
    W = max(args.warmup, -(-max(w.budget) // (chunk * w.n_layers * w.n_kv_heads)) + 1)   # past the fill-up phase
    nseg, D, S = w.nseg, w.head_dim, w.n_seq
    per_seq = w.n_layers * w.n_kv_heads
    reserve = chunk
    B = sum(w.budget)
    paged = args.paged
    if paged:
        # pages for the budget and the chunk that is live until the eviction, plus slack for partly filled pages
        n_pages = (B + nseg * chunk) // kv.PAGE_SIZE + 3 * nseg + 64
        cap = n_pages * kv.PAGE_SIZE
        ctx = kv.Context(S, w.n_layers, w.n_kv_heads, w.n_q_heads, D, cap)
        pc = kv.PagedCache(nseg, D, n_pages, n_pages, dev)
        empty = kv.Cache.empty(nseg, D, 8, dev)                     # the pool is initialised from an empty ragged cache
        kv.kvtrim_paged_build(ctx, empty, torch.zeros(8, dtype=torch.uint8, device=dev),
                              torch.zeros(nseg, dtype=torch.int32, device=dev), pc)
    else:
        cap = B + nseg * reserve + 8
        caches = [kv.Cache.empty(nseg, D, cap, dev) for _ in range(2)]
        caches[0].seg_start.copy_(torch.arange(nseg, dtype=torch.int64) * reserve)
        ctx = kv.Context(S, w.n_layers, w.n_kv_heads, w.n_q_heads, D, cap)
    score = torch.zeros(cap, dtype=torch.float32, device=dev)
    keep = torch.zeros(cap, dtype=torch.uint8, device=dev)
    kept = torch.zeros(nseg, dtype=torch.int32, device=dev)
    thr = torch.zeros(S, dtype=torch.int32, device=dev)
    budget = torch.tensor(list(w.budget), dtype=torch.int64, device=dev)
    t0 = time.time()
    inp = ki.chunk_inputs(w, chunk, dev)                            # the same K / V / log beta rows every step; positions move on
    torch.cuda.synchronize()
    log(f"[bench] chunk of {chunk} tokens x {nseg} segments: {2 * nseg * chunk * D * 2 / 1e9:.2f} GB of new K/V, "
        f"generated in {time.time() - t0:.1f}s")
    ar = torch.arange(chunk, dtype=torch.int32, device=dev)
    pos_news = [(ar + s * chunk).repeat(nseg, 1).contiguous() for s in range(W + K)]
    nows = [torch.full((S,), (s + 1) * chunk - 1, dtype=torch.int32, device=dev) for s in range(W + K)]
    state = {"cur": 0}

    def step(s):
        if paged:
            kv.kvtrim_paged_append(ctx, pc, inp["k_new"], inp["v_new"], inp["log_beta_new"], pos_news[s], n_new=chunk)
            kv.kvtrim_paged_score(ctx, pc, nows[s], score)
            kv.kvtrim_paged_select(ctx, pc, score, budget, keep, kept, thr)
            kv.kvtrim_paged_evict(ctx, pc, keep)
            return
        cur, dst = caches[state["cur"]], caches[state["cur"] ^ 1]
        if args.one_call:
            kv.kvtrim_append_compact(ctx, cur, inp["k_new"], inp["v_new"], inp["log_beta_new"], pos_news[s], chunk, nows[s],
                                     budget, score, keep, kept, dst, reserve, thr_key_out=thr)
        else:
            kv.kvtrim_append(ctx, cur, inp["k_new"], inp["v_new"], inp["log_beta_new"], pos_news[s], chunk)
            kv.kvtrim_score(ctx, cur, nows[s], score)
            kv.kvtrim_select_global(ctx, cur, score, budget, keep, kept, thr)
            kv.kvtrim_compact(ctx, cur, keep, kept, dst, reserve)
        state["cur"] ^= 1

    for s in range(W):
        step(s)
    torch.cuda.synchronize()
    assert kv.kvtrim_poll_error(ctx) == 0, "device-side error while the caches filled up"
    n_ret = int(kept.sum().item())
    n_cand = n_ret + nseg * chunk
    kv.kvtrim_profile_begin(ctx, (1 << kv.binding.N_KERNELS) - 1)
    torch.cuda.synchronize()
    t_begin = time.perf_counter()
    for s in range(W, W + K):
        step(s)
    torch.cuda.synchronize()
    t_end = time.perf_counter()
    prof = kv.kvtrim_profile_end(ctx)
    assert kv.kvtrim_poll_error(ctx) == 0, "device-side error in the timed region"
    assert int(kept.sum().item()) == n_ret == B
    ms = (t_end - t_begin) * 1e3 / K
    for name, (t, n) in sorted(prof.items(), key=lambda kvp: -kvp[1][0]):
        log(f"[bench]   {name:16s} {t / n * 1e3:8.1f} us x {n}")
    R = 4 * D + 8
    # (kvtrim_append_compact appends 8 B of metadata per new token instead of the whole row; the byte model is
    # kept as the four stages state it, so the figures of the two ways stay comparable)
    stage = {"append": 2 * R * nseg * chunk, "score": 8 * n_cand, "select": 5 * n_cand,
             "compact": 0 if paged else 2 * R * n_ret}              # pages: eviction frees slots, nothing moves
    total = sum(stage.values())
    dom = "k_pg_append" if paged else "k_cmp_copy"
    dom_bytes = stage["append"] if paged else stage["compact"]
    d_ms = prof[dom][0] / prof[dom][1]
    log(f"[bench] chunk step{' on pages' if paged else ''}: {ms:.3f} ms ({total / (ms * 1e-3) / 1e9:.0f} GB/s algorithmic end "
        f"to end); {dom} {d_ms:.3f} ms ({dom_bytes / (d_ms * 1e-3) / 1e9:.0f} GB/s)")
    print(json.dumps({
        "metric": "chunked-prefill steps/sec (append a chunk, rescore, select, compact), 16 sequences", "value": 1e3 / ms,
        "unit": "steps/s", "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": ms, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"multiturn chunk step: S{S} L{w.n_layers} Hkv{w.n_kv_heads} D{D}, {chunk} new tokens per "
                               f"segment, {n_cand} candidates -> {n_ret} retained per step",
                   "layout": "paged" if paged else "ragged",
                   "stages": ("paged_append, paged_score, paged_select, paged_evict" if paged else
                              ("append_compact (one call: metadata appended, rows moved once)" if args.one_call else
                               "append, score, select_global, compact")) + " (no attention in a chunk step)"},
        "end_to_end": {"algorithmic_bytes_per_step": total, "achieved_GBps": total / (ms * 1e-3) / 1e9,
                       "frac_of_hbm_peak": total / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "bytes_by_stage": stage},
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": dom_bytes / (d_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": dom_bytes / (d_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "traffic": None,
                     "algorithmic_bytes_per_launch": dom_bytes, "avg_launch_ms": d_ms},
    }), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default="long", choices=["long", "llama", "vlm", "tiny", "multiturn"])
    ap.add_argument("--prefill", type=int, default=None, help="override the prefilled length (scaled-down run)")
    ap.add_argument("--horizon", type=int, default=1,
                    help="lookahead horizon of the score: 1 = the metric's form, 2 = the paper's inference default, 0 = infinite")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy, the known-size reference for rocprofv3 --pmc counters")
    ap.add_argument("--unfused", action="store_true",
                    help="run stages 3 and 4 as two calls (kvtrim_compact, kvtrim_decode_attn) instead of the fused one")
    ap.add_argument("--paged", action="store_true",
                    help="steady state on the paged layout: eviction frees slots of fixed-size pages and moves no K/V "
                         "(paged_append, paged_score, paged_select, paged_evict, paged_attn)")
    ap.add_argument("--defrag-every", type=int, default=0, metavar="N",
                    help="with --paged: defragment the pages every N steps (kvtrim_paged_defrag), inside the timed region")
    ap.add_argument("--kernel-times", action="store_true",
                    help="bracket every kernel with HIP events and print the per-kernel averages to stderr "
                         "(the events add a little to ms_per_step)")
    ap.add_argument("--graph", action="store_true",
                    help="capture the K timed steps into one HIP graph and time its replay (the per-kernel figures "
                         "then come from 20 eager steps run just before)")
    ap.add_argument("--gate", type=int, default=0, metavar="N_TOK",
                    help="time the retention-gate forward alone (the metric model's shape: 32 layers x 8 KV heads, "
                         "d_model 4096, hidden width 512, projection width 128) for N_TOK tokens per call")
    ap.add_argument("--prepared", action="store_true",
                    help="with --gate: fold the readout and re-tile W1 once before the timed calls (kvtrim_gate_prepare) "
                         "and time kvtrim_gate_forward_prepared - weights that do not change between calls")
    ap.add_argument("--chunk", type=int, default=0, metavar="N_TOK",
                    help="time the chunked-prefill step of the multi-turn workload instead of decode steps: N_TOK new "
                         "tokens per segment, then rescore, select, compact (the paper-shaped chunk is 4096)")
    ap.add_argument("--inplace", type=int, default=0, metavar="ROOM",
                    help="compact inside the cache (kvtrim_compact_attn_inplace: rows move only behind an eviction) with ROOM "
                         "free slots behind every segment; every ROOM-th step is an out-of-place step that evens the room out")
    ap.add_argument("--separate-score-select", action="store_true",
                    help="run stages 1 and 2 as two calls (kvtrim_score, kvtrim_select_global) instead of kvtrim_score_select")
    ap.add_argument("--one-call", action="store_true",
                    help="with --chunk (ragged layout): the chunk step through kvtrim_append_compact, which moves the new rows "
                         "once, from the caller's buffers to the compacted cache")
    args = ap.parse_args()
    if args.one_call and (not args.chunk or args.paged):
        ap.error("--one-call needs --chunk and the ragged layout")
    if args.chunk:
        if args.gpus != 1:
            print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
            sys.exit(2)
        if not 1 <= args.chunk <= 4096:
            ap.error("--chunk takes 1 .. 4096 tokens")
        return bench_chunk(args)
    if args.gate:
        if args.gpus != 1:
            print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
            sys.exit(2)
        return bench_gate(args)
    if args.paged and args.unfused:
        ap.error("--paged and --unfused exclude each other")
    if args.inplace and (args.paged or args.inplace < 2):
        ap.error("--inplace takes a room of at least 2 slots and excludes --paged")
    if args.defrag_every and not args.paged:
        ap.error("--defrag-every needs --paged")
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import kvtrim_inputs as ki
    import paper_2605_09649_amd as kv

    dev = "cuda:0"
    torch.cuda.set_device(0)
    w = ki.workload(args.workload, prefill=args.prefill)
    reserve = args.inplace if args.inplace else 1                 # free slots behind every segment after an out-of-place step
    K, W = args.steps, max(args.warmup, 1)
    G_STEPS = 20 if args.graph else 0         # eager, profiled steps before a captured region
    n_steps = K + W + G_STEPS + CPU_STEPS + 1 # + the extra steps that are replayed on the CPU oracle, + one that is looked at

    t0 = time.time()
    pre = ki.with_horizon(ki.prefill_cache(w, reserve=reserve, device=dev), args.horizon)
    torch.cuda.synchronize()
    total0 = sum(w.prefill) * w.n_layers * w.n_kv_heads
    log(f"[bench] prefill cache: {total0} entries, {2 * total0 * w.head_dim * 2 / 1e9:.2f} GB K/V, "
        f"generated in {time.time() - t0:.1f}s")

    B = sum(w.budget)
    dst_cap = min(B, total0 + n_steps * w.nseg) + w.nseg * reserve + 8
    src = kv.Cache.from_dict(pre, dev)
    spare, pc = [], None
    if args.paged:
        # room for the budget, one partly filled page per segment, and the pages that segments take while
        # their own still hold scattered free slots elsewhere
        n_pages = (min(B, total0 + n_steps * w.nseg) + kv.PAGE_SIZE - 1) // kv.PAGE_SIZE + 3 * w.nseg + 64
        pc = kv.PagedCache(w.nseg, w.head_dim, n_pages, n_pages, dev, with_tail=args.horizon != 1)
        dst_cap = n_pages * kv.PAGE_SIZE
    else:
        spare = [kv.Cache.empty(w.nseg, w.head_dim, dst_cap, dev, with_tail=args.horizon != 1) for _ in range(2)]
    cap = max(src.cap, dst_cap)
    ctx = kv.Context(w.n_seq, w.n_layers, w.n_kv_heads, w.n_q_heads, w.head_dim, cap)
    score = torch.zeros(cap, dtype=torch.float32, device=dev)
    keep = torch.zeros(cap, dtype=torch.uint8, device=dev)
    kept = torch.zeros(w.nseg, dtype=torch.int32, device=dev)
    thr = torch.zeros(w.n_seq, dtype=torch.int32, device=dev)
    budget = torch.tensor(list(w.budget), dtype=torch.int64, device=dev)
    out = torch.zeros(w.n_seq, w.n_layers, w.n_q_heads, w.head_dim, dtype=torch.float32, device=dev)
    lse = torch.zeros(w.n_seq, w.n_layers, w.n_q_heads, dtype=torch.float32, device=dev)
    scale = 1.0 / math.sqrt(w.head_dim)
    per_seq = w.n_layers * w.n_kv_heads

    # every step's inputs are generated before the timed region and stay resident in HBM
    inputs, nows, pos_news = [], [], []
    now0 = np.array([t - 1 for t in w.prefill], np.int32)
    for s in range(n_steps):
        inputs.append(ki.decode_inputs(w, s, device=dev, horizon=args.horizon))
        now = now0 + s + 1
        nows.append(torch.from_numpy(now).to(dev))
        pos_news.append(torch.from_numpy(np.repeat(now, per_seq).astype(np.int32)).to(dev))
    torch.cuda.synchronize()

    state = {"src": src, "flip": 0}

    def step(s):
        inp = inputs[s]
        cur = state["src"]
        if args.paged and s > 0:
            kv.kvtrim_paged_append(ctx, pc, inp["k_new"], inp["v_new"], inp["log_beta_new"], pos_news[s],
                                   log_tail_new=inp.get("log_tail_new"))
            kv.kvtrim_paged_score(ctx, pc, nows[s], score)
            kv.kvtrim_paged_select(ctx, pc, score, budget, keep, kept, thr)
            kv.kvtrim_paged_evict(ctx, pc, keep)
            if args.defrag_every and s % args.defrag_every == 0:
                kv.kvtrim_paged_defrag(ctx, pc)
            kv.kvtrim_paged_attn(ctx, pc, inp["q"], 0, w.n_layers, scale, out, lse)
            return
        kv.kvtrim_append(ctx, cur, inp["k_new"], inp["v_new"], inp["log_beta_new"], pos_news[s], 1,
                         log_tail_new=inp.get("log_tail_new"))
        if args.separate_score_select:
            kv.kvtrim_score(ctx, cur, nows[s], score)
            kv.kvtrim_select_global(ctx, cur, score, budget, keep, kept, thr)
        else:                                   # first step: eviction from the whole prefill (hint 0: the radix passes)
            kv.kvtrim_score_select(ctx, cur, nows[s], budget, score, keep, kept, thr, evict_hint=per_seq if s > 0 else 0)
        if args.paged:                          # first step: the survivors of the prefill go into pages
            kv.kvtrim_paged_build(ctx, cur, keep, kept, pc)
            kv.kvtrim_paged_attn(ctx, pc, inp["q"], 0, w.n_layers, scale, out, lse)
            state["src"] = None
            return
        dst = spare[state["flip"]]
        if args.inplace and s > 0 and s % args.inplace:
            # the other cache lends its arrays as parking space; the segments stay where they are
            if args.unfused:                   # stage 3 alone in place, then the stand-alone attention on the same cache
                kv.kvtrim_compact_inplace(ctx, cur, keep, kept, dst)
                kv.kvtrim_decode_attn(ctx, cur, inp["q"], 0, w.n_layers, scale, out, lse)
            else:
                kv.kvtrim_compact_attn_inplace(ctx, cur, keep, kept, dst, inp["q"], 0, w.n_layers, scale, out, lse)
            return
        if args.unfused:
            kv.kvtrim_compact(ctx, cur, keep, kept, dst, reserve)
            kv.kvtrim_decode_attn(ctx, dst, inp["q"], 0, w.n_layers, scale, out, lse)
        else:
            kv.kvtrim_compact_attn(ctx, cur, keep, kept, dst, reserve, inp["q"], 0, w.n_layers, scale, out, lse)
        state["src"] = dst
        state["flip"] ^= 1

    if args.pmc_calibration:                  # 2^28 floats in, 2^28 floats out, one elementwise copy kernel
        ca = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        cb = torch.empty_like(ca)
        cb.copy_(ca)
        torch.cuda.synchronize()
        del ca, cb
        torch.cuda.empty_cache()

    # ---- warm-up: the first step evicts from the full prefill down to the budget
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    step(0)
    e1.record()
    torch.cuda.synchronize()
    first_ms = e0.elapsed_time(e1)
    assert kv.kvtrim_poll_error(ctx) == 0, "device-side error in the first step"
    del pre, src
    torch.cuda.empty_cache()
    for s in range(1, W):
        step(s)
    torch.cuda.synchronize()
    n_ret = int(kept.sum().item())
    n_cand = n_ret + w.nseg
    log(f"[bench] first step (prefill -> budget): {first_ms:.3f} ms; steady state: {n_cand} candidates, {n_ret} retained")

    # ---- timed region: exactly K steps; the dominant kernels are bracketed by HIP events on the launch stream
    mask = (1 << 8) | (1 << 10) | (1 << 13) | (1 << 30)   # k_cmp_copy, k_att_partial, k_cmp_attn, k_att_fused
    if args.kernel_times:
        mask = (1 << kv.binding.N_KERNELS) - 1   # every kernel (the events then add to the step time)
    kv.kvtrim_profile_begin(ctx, mask)
    torch.cuda.synchronize()
    if args.graph:
        for s in range(W, W + G_STEPS):       # per-kernel durations: events cannot be recorded inside a capture
            step(s)
        torch.cuda.synchronize()
        prof = kv.kvtrim_profile_end(ctx)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):         # the library only enqueues kernels on the current stream
            for s in range(W + G_STEPS, W + G_STEPS + K):
                step(s)
        torch.cuda.synchronize()
        t_begin = time.perf_counter()
        graph.replay()
        torch.cuda.synchronize()
        t_end = time.perf_counter()
    else:
        t_begin = time.perf_counter()
        for s in range(W, W + K):
            step(s)
        torch.cuda.synchronize()
        t_end = time.perf_counter()
        prof = kv.kvtrim_profile_end(ctx)
    assert kv.kvtrim_poll_error(ctx) == 0, "device-side error in the timed region"
    if args.kernel_times:
        for name, (ms, n) in sorted(prof.items(), key=lambda kvp: -kvp[1][0]):
            log(f"[bench]   {name:16s} {ms / n * 1e3:8.1f} us x {n}")
    ms_per_step = (t_end - t_begin) * 1e3 / K
    sel_paths = kv.kvtrim_select_path_counts(ctx)
    log(f"[bench] decode-step selections so far: {sel_paths[0]} from the candidate list, {sel_paths[1]} by the single-block fallback")
    inplace_info = None
    alg = algorithmic_bytes(w, n_cand, n_ret, args.horizon)
    alg_total = sum(alg.values())
    stage_model_bytes = None
    if args.paged:
        # no K/V moves: the step's compulsory bytes are the score (8 B), the selection (4 B score + 1 B mask)
        # and the eviction (1 B mask + 4 B position) per candidate, and the attention's read of K, V and the
        # position of every retained entry
        alg = {"score": alg["score"], "select": alg["select"], "evict": 5 * n_cand,
               "attend": alg["attend"] + 4 * n_ret}
        alg_total = sum(alg.values())
        dom, dom_bytes = "k_att_partial", alg["attend"]
    elif args.unfused and args.inplace:
        # stage 3 alone in place touches only the rows behind an eviction: the attention is the dominant kernel
        dom, dom_bytes = "k_att_partial", alg["attend"]
    elif args.unfused:
        dom, dom_bytes = "k_cmp_copy", alg["compact"]
    else:
        # The fused kernel does the work of stages 3 and 4 but reads K/V once.  Its roofline is priced on
        # the bytes the fused operation cannot avoid: every retained entry read once and written once
        # (2 * (4D + 8) B), the mask (1 B per candidate), q and out (6D B per query head).  The stage-by-stage
        # byte model (1040 + 512 B per retained entry) is reported beside it.
        dom = "k_cmp_attn"
        dom_bytes = alg["compact"] + n_cand + 6 * w.head_dim * w.n_seq * w.n_layers * w.n_q_heads
        stage_model_bytes = alg["compact"] + alg["attend"]
        if args.inplace:
            # In place every retained entry is read once (4D + 8 B) and only the rows behind an eviction are written.
            # How many those are depends on the data: they are counted on one more step after the timed region.
            # One launch in ROOM is out of place.
            s_extra = W + G_STEPS + K                              # the step right after the timed region
            if s_extra % args.inplace == 0:
                step(s_extra)                                      # (an out-of-place step falls here: look at the next one)
                s_extra = None
            moved = None
            if s_extra is not None:
                inp, cur = inputs[s_extra], state["src"]
                kv.kvtrim_append(ctx, cur, inp["k_new"], inp["v_new"], inp["log_beta_new"], pos_news[s_extra], 1,
                                 log_tail_new=inp.get("log_tail_new"))
                kv.kvtrim_score(ctx, cur, nows[s_extra], score)
                kv.kvtrim_select_global(ctx, cur, score, budget, keep, kept, thr)
                torch.cuda.synchronize()
                moved = rows_moved_in_place(cur, keep)
                kv.kvtrim_compact_attn_inplace(ctx, cur, keep, kept, spare[state["flip"]], inp["q"], 0, w.n_layers, scale, out, lse)
                torch.cuda.synchronize()
                log(f"[bench] in place: {moved} of {n_ret} retained rows ({100.0 * moved / n_ret:.1f} %) lie behind an eviction "
                    f"and are written; the others are only read")
            row_bytes = alg["compact"] // (2 * n_ret)
            inplace_bytes = (alg["compact"] // 2 + row_bytes * (moved or 0) +
                             6 * w.head_dim * w.n_seq * w.n_layers * w.n_q_heads)
            dom_bytes = ((args.inplace - 1) * inplace_bytes + dom_bytes) // args.inplace
            stage_model_bytes = None
            alg = {"score": alg["score"], "select": alg["select"],
                   "compact+attend (in place: every retained row read, the rows behind an eviction written)": dom_bytes}
            alg_total = sum(alg.values())
            inplace_info = {"room": args.inplace, "rows_written_sampled": moved, "rows_retained": n_ret}
    if dom not in prof and "k_att_fused" in prof:   # large groups of query heads: the loop-shaped fused kernel, same bytes
        dom = "k_att_fused"
    if dom not in prof:                       # the cache is too large for the fused kernel: the library ran the two stages
        dom, dom_bytes, stage_model_bytes = "k_cmp_copy", alg["compact"], None
    dom_ms, dom_n = prof[dom]
    dom_avg_ms = dom_ms / dom_n
    achieved = dom_bytes / (dom_avg_ms * 1e-3) / 1e9
    log(f"[bench] {ms_per_step:.4f} ms/step ({alg_total / (ms_per_step * 1e-3) / 1e9:.0f} GB/s algorithmic end to end); "
        f"{dom} {dom_avg_ms:.4f} ms ({achieved:.0f} GB/s on its compulsory bytes)")
    second = None
    if args.unfused and args.inplace:
        mv_ms, mv_n = prof["k_cmp_copy"]       # (the in-place row mover is bracketed under the row mover's name)
        second = {"kernel": "k_cmp_move_inplace", "avg_launch_ms": mv_ms / mv_n}
        log(f"[bench] in-place row mover (with one out-of-place launch in {args.inplace}) {mv_ms / mv_n:.4f} ms")
    elif args.unfused:
        att_ms, att_n = prof["k_att_partial"]
        second = {"kernel": "k_att_partial", "avg_launch_ms": att_ms / att_n,
                  "achieved": alg["attend"] / (att_ms / att_n * 1e-3) / 1e9}
        log(f"[bench] k_att_partial {att_ms / att_n:.4f} ms ({second['achieved']:.0f} GB/s)")

    result = {
        "metric": "eviction+decode steps/sec and achieved HBM GB/s (% of peak), 32Lx8H 128K ctx",
        "value": 1e3 / ms_per_step,
        "unit": "steps/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {
            "workload": f"{w.name}: S{w.n_seq} L{w.n_layers} Hkv{w.n_kv_heads} Hq{w.n_q_heads} D{w.head_dim}, "
                        f"{w.prefill[0]} prefilled, B={B} ({n_cand} candidates/step, {n_ret} retained), "
                        f"score lookahead horizon {args.horizon if args.horizon > 0 else 'infinite'}",
            "stages": ("paged_append, paged_score, paged_select, paged_evict, paged_attn (paged layout: no K/V moved; "
                       "five C-ABI calls per step)" if args.paged else
                       "append, score, select_global, compact, decode_attn (five C-ABI calls per step)" if args.unfused else
                       f"append, score, select_global, compact_attn_inplace (stages 3+4 fused inside the cache, {args.inplace} free "
                       f"slots per segment; every {args.inplace}th step is an out-of-place compact_attn)" if args.inplace else
                       "append, score, select_global, compact_attn (stages 3+4 fused; four C-ABI calls per step)"),
            "first_step_ms": first_ms,
            "launch": "one HIP graph holding the K timed steps, replayed once" if args.graph else "eager launches",
        },
        "end_to_end": {"algorithmic_bytes_per_step": alg_total, "achieved_GBps": alg_total / (ms_per_step * 1e-3) / 1e9,
                       "frac_of_hbm_peak": alg_total / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
                       "bytes_by_stage": alg},
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": MEASURED_TRAFFIC.get((w.name + ("-paged" if args.paged else "-inplace" if args.inplace else ""), dom)),
                     "algorithmic_bytes_per_launch": dom_bytes, "avg_launch_ms": dom_avg_ms, "launches": dom_n,
                     "stage_model_bytes_per_launch": stage_model_bytes,
                     "stage_model_achieved": (stage_model_bytes / (dom_avg_ms * 1e-3) / 1e9) if stage_model_bytes else None,
                     "second_kernel": second},
    }

    if inplace_info:
        result["config"]["in_place"] = inplace_info
    if args.paged:
        result["config"]["pages"] = {"page_size": kv.PAGE_SIZE, "n_pages": pc.n_pages,
                                     "in_use_after_timed_region": int(pc.seg_pages.sum().item())}
        log(f"[bench] pages in use after the timed region: {result['config']['pages']['in_use_after_timed_region']} of {pc.n_pages}")

    # ---- CPU baseline: the oracle replays CPU_STEPS more steps of the same workload on the host cores, and the
    # GPU's results of those steps are checked against it (selection/compaction bit-exact, attention 5e-3)
    if not args.no_cpu_baseline:
        import oracle
        from harness import attn_error, compare_cache_contents, compare_caches, device_cache_to_host
        from helpers import bf16_bits
        if args.paged:                          # the pages as the oracle's ragged cache: each segment in position order
            from paged_harness import PagedHost
            ph = PagedHost(pc)
            hc = ph.as_ragged(oracle.Shape(w.n_seq, w.n_layers, w.n_kv_heads, w.n_q_heads, w.head_dim), reserve)
            del ph
        else:
            hc = device_cache_to_host(w, state["src"])
        budget_np = np.array(list(w.budget), np.int64)
        cpu_s, ok_sel, err = 0.0, True, 0.0
        first_cpu = W + G_STEPS + K + (1 if args.inplace else 0)   # (in place: one step was spent counting moved rows)
        for s in range(first_cpu, first_cpu + CPU_STEPS):
            inp = {k: v.cpu() for k, v in inputs[s].items()}
            now = now0 + s + 1
            pos_new = np.repeat(now, per_seq).astype(np.int32)
            kb, vb, qb = bf16_bits(inp["k_new"]), bf16_bits(inp["v_new"]), bf16_bits(inp["q"])
            lbn = inp["log_beta_new"].numpy()
            ltn = inp["log_tail_new"].numpy() if args.horizon != 1 else None
            t_cpu = time.perf_counter()
            oracle.append(hc, kb, vb, lbn, pos_new, log_tail_new=ltn)
            score_ref = oracle.score(hc, now)
            keep_ref, kept_ref, thr_ref = oracle.select(hc, score_ref, budget_np)
            hc = oracle.compact(hc, keep_ref, dst_cap, reserve)
            out_ref, _ = oracle.attend(hc, qb, scale)
            cpu_s += time.perf_counter() - t_cpu
            step(s)
            torch.cuda.synchronize()
            ok_sel = ok_sel and bool(np.array_equal(kept.cpu().numpy(), kept_ref))
            err = max(err, attn_error(out.cpu().numpy(), out_ref))
        if args.paged:
            ph = PagedHost(pc)
            ok_cache = ph.structure_problems() == [] and ph.equals(hc)
        elif args.inplace:                      # the segments keep their starts: contents are compared segment by segment
            ok_cache = compare_cache_contents(device_cache_to_host(w, state["src"]), hc)
        else:
            ok_cache = compare_caches(device_cache_to_host(w, state["src"]), hc)
        log(f"[bench] {CPU_STEPS} oracle steps on the host: {cpu_s:.2f} s; GPU vs oracle on those steps: kept equal={ok_sel}, "
            f"final cache equal={ok_cache}, attention err={err:.2e}")
        assert kv.kvtrim_poll_error(ctx) == 0 and ok_sel and ok_cache and err <= 5e-3, "GPU steps disagree with the oracle"
        result["cpu_baseline"] = {"value": CPU_STEPS / cpu_s, "unit": "steps/s", "cores": oracle.threads(), "kind": "oracle",
                                  "sample": f"{CPU_STEPS} full steps of the same workload after the timed region (append, score, "
                                            "full-sort select, compact, fp64 attention); only the attention loop uses all cores "
                                            "(OpenMP over segments), the other stages run on one"}
        result["parity_on_sampled_step"] = {"steps": CPU_STEPS, "select_compact_bit_exact": ok_sel and ok_cache,
                                            "attn_max_norm_rel_err": err}
    # ---- the same steps with stages 3+4 done inside the cache (kvtrim_compact_attn_inplace), timed beside the metric's
    # out-of-place step: ROOM free slots behind every segment, every ROOM-th step out of place to even them out
    ROOM, K2 = 64, min(K, 128)
    cap_room = n_ret + w.nseg * ROOM + 8
    plain = not (args.paged or args.unfused or args.inplace or args.graph or args.kernel_times or args.pmc_calibration)
    if plain and cap_room <= cap:
        s0 = n_steps
        extra, extra_now, extra_pos = [], [], []
        for s in range(s0, s0 + K2 + 1):
            extra.append(ki.decode_inputs(w, s, device=dev, horizon=args.horizon))
            now = now0 + s + 1
            extra_now.append(torch.from_numpy(now).to(dev))
            extra_pos.append(torch.from_numpy(np.repeat(now, per_seq).astype(np.int32)).to(dev))
        big = [kv.Cache.empty(w.nseg, w.head_dim, cap_room, dev, with_tail=args.horizon != 1) for _ in range(2)]
        cur, other = state["src"], big[0]

        def step_room(i, in_place):
            nonlocal cur, other
            inp = extra[i]
            kv.kvtrim_append(ctx, cur, inp["k_new"], inp["v_new"], inp["log_beta_new"], extra_pos[i], 1,
                             log_tail_new=inp.get("log_tail_new"))
            kv.kvtrim_score(ctx, cur, extra_now[i], score)
            kv.kvtrim_select_global(ctx, cur, score, budget, keep, kept, thr)
            if in_place:
                kv.kvtrim_compact_attn_inplace(ctx, cur, keep, kept, other, inp["q"], 0, w.n_layers, scale, out, lse)
            else:
                kv.kvtrim_compact_attn(ctx, cur, keep, kept, other, ROOM, inp["q"], 0, w.n_layers, scale, out, lse)
                cur, other = other, (big[1] if other is big[0] else big[0])

        step_room(0, False)                                        # into a cache with room behind every segment
        torch.cuda.synchronize()
        t_begin = time.perf_counter()
        for i in range(1, K2 + 1):
            step_room(i, i % ROOM != 0)
        torch.cuda.synchronize()
        ms_room = (time.perf_counter() - t_begin) * 1e3 / K2
        assert kv.kvtrim_poll_error(ctx) == 0 and int(kept.sum().item()) == n_ret and bool(torch.isfinite(out).all())
        log(f"[bench] the same steps compacting in place: {ms_room:.4f} ms/step ({1e3 / ms_room:.0f} steps/s)")
        result["in_place_variant"] = {
            "ms_per_step": ms_room, "value": 1e3 / ms_room, "unit": "steps/s", "steps": K2, "room": ROOM,
            "what": "append, score, select_global, compact_attn_inplace: a row moves only if an entry before it in its segment "
                    "was evicted; every 64th step is out of place (inside the timed steps); checked against the oracle by "
                    "bench.py --inplace 64 and tests/test_gpu_inplace.py"}
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
