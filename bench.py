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
CPU_STEPS_ONE_THREAD = 2       # of these, with the oracle's threaded stage held to one thread
WHOLE_CACHE_PARITY_BYTES = 6e9 # live K/V above this: the oracle checks selection and metadata whole, rows and attention on sampled segments


def kernel_sources_sha16():
    """Hash of the kernel sources: a traffic figure from rocprofv3 counters is quoted only while it is unchanged."""
    import hashlib
    d = os.path.join(ROOT, "paper_2605_09649_amd", "csrc")
    h = hashlib.sha256()
    for f in sorted(os.listdir(d)):
        if f.endswith((".hip", ".h")):
            h.update(f.encode())
            h.update(open(os.path.join(d, f), "rb").read())
    return h.hexdigest()[:16]


def measured_traffic(tag, kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary of workload/variant `tag`
    (profiles/<tag>_hbm_traffic_pmc.txt: FETCH_SIZE and WRITE_SIZE, each scaled by what the counter reads for a plain
    copy of known size), or None when there is no such summary or the kernels have changed since it was taken."""
    path = os.path.join(ROOT, "profiles", f"{tag}_hbm_traffic_pmc.txt")
    if not os.path.exists(path):
        return None
    sha, val = None, None
    for line in open(path):
        p = line.split()
        if len(p) >= 3 and p[0] == "#" and p[1] == "kernel_sources_sha16":
            sha = p[2]
        if len(p) >= 4 and p[0] == "#" and p[1] == "traffic_bytes_per_launch" and p[2] == kernel:
            val = float(p[3])
    return val if sha == kernel_sources_sha16() else None


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
        # (prepared weights, up to 16 tokens: the readout rides in the first-layer kernel and there is no second one)
        r_ms = prof[second][0] / prof[second][1] if second in prof else None
        # first layer: W1 once per 64 tokens of a call, x once per 16-row tile group (cached), u written once (one
        # kernel: the folded vectors read, per block its parts of the readout sums written and read once instead)
        alg_hidden = w1_bytes + L * n_tok * dm * 2 + (L * n_tok * dg * 4 if r_ms is not None else L * H * (dg + 1) * 4 + 2 * L * (dg // 16) * H * n_tok * 4)
        if n_tok <= 64:
            roof = {"bound": "hbm", "kernel": first, "achieved": alg_hidden / (h_ms * 1e-3) / 1e9,
                    "peak": HBM_PEAK_GBS, "unit": "GB/s", "traffic": measured_traffic(f"gate_decode_{n_tok}tok", first),
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


METRIC_LONG = "eviction+decode steps/sec and achieved HBM GB/s (% of peak), 32Lx8H 128K ctx"


def metric_name(w):
    if w.name == "long" and w.prefill[0] == 131072:
        return METRIC_LONG
    return (f"eviction+decode steps/sec and achieved HBM GB/s (% of peak), {w.n_seq} x {w.n_layers}Lx{w.n_kv_heads}H, "
            f"{max(w.prefill)} ctx ({w.name})")


class Runner:
    """Device-side state of the decode loop of one workload in one variant (ragged out of place / in place / two
    calls / paged), with all step inputs resident in HBM, and one step of it through the C ABI."""

    def __init__(self, w, args, n_steps, reserve, dev="cuda:0"):
        import numpy as np
        import torch
        import kvtrim_inputs as ki
        import paper_2605_09649_amd as kv
        self.w, self.args, self.kv, self.reserve, self.dev = w, args, kv, reserve, dev
        self.per_seq = w.n_layers * w.n_kv_heads
        pre = ki.with_horizon(ki.prefill_cache(w, reserve=reserve, device=dev), args.horizon)
        self.total0 = sum(w.prefill) * self.per_seq
        B = sum(w.budget)
        tail = args.horizon != 1
        dst_cap = min(B, self.total0 + n_steps * w.nseg) + w.nseg * reserve + 8
        self.src = kv.Cache.from_dict(pre, dev)
        del pre
        self.spare, self.pc = [], None
        if args.paged:
            # room for the budget, one partly filled page per segment, and the pages that segments take while
            # their own still hold scattered free slots elsewhere
            n_pages = (min(B, self.total0 + n_steps * w.nseg) + kv.PAGE_SIZE - 1) // kv.PAGE_SIZE + 3 * w.nseg + 64
            self.pc = kv.PagedCache(w.nseg, w.head_dim, n_pages, n_pages, dev, with_tail=tail)
            dst_cap = n_pages * kv.PAGE_SIZE
        else:
            self.spare = [kv.Cache.empty(w.nseg, w.head_dim, dst_cap, dev, with_tail=tail) for _ in range(2)]
        self.dst_cap = dst_cap
        self.cap = cap = max(self.src.cap, dst_cap)
        self.ctx = kv.Context(w.n_seq, w.n_layers, w.n_kv_heads, w.n_q_heads, w.head_dim, cap)
        self.score = torch.zeros(cap, dtype=torch.float32, device=dev)
        self.keep = torch.zeros(cap, dtype=torch.uint8, device=dev)
        self.kept = torch.zeros(w.nseg, dtype=torch.int32, device=dev)
        self.thr = torch.zeros(w.n_seq, dtype=torch.int32, device=dev)
        self.budget = torch.tensor(list(w.budget), dtype=torch.int64, device=dev)
        self.out = torch.zeros(w.n_seq, w.n_layers, w.n_q_heads, w.head_dim, dtype=torch.float32, device=dev)
        self.lse = torch.zeros(w.n_seq, w.n_layers, w.n_q_heads, dtype=torch.float32, device=dev)
        self.scale = 1.0 / math.sqrt(w.head_dim)
        # every step's inputs are generated before the timed region and stay resident in HBM
        self.inputs, self.nows, self.pos_news = [], [], []
        self.now0 = np.array([t - 1 for t in w.prefill], np.int32)
        for s in range(n_steps):
            self.inputs.append(ki.decode_inputs(w, s, device=dev, horizon=args.horizon))
            now = self.now0 + s + 1
            self.nows.append(torch.from_numpy(now).to(dev))
            self.pos_news.append(torch.from_numpy(np.repeat(now, self.per_seq).astype(np.int32)).to(dev))
        self.cur, self.flip = self.src, 0
        torch.cuda.synchronize()

    def select(self, s, cur):
        kv, a = self.kv, self.args
        if a.separate_score_select:
            kv.kvtrim_score(self.ctx, cur, self.nows[s], self.score)
            kv.kvtrim_select_global(self.ctx, cur, self.score, self.budget, self.keep, self.kept, self.thr)
        else:
            # first step: eviction from the whole prefill (hint 0: the radix passes); decode steps: one entry per
            # segment comes in, so about as many go
            kv.kvtrim_score_select(self.ctx, cur, self.nows[s], self.budget, self.score, self.keep, self.kept, self.thr,
                                   evict_hint=self.per_seq if s > 0 else 0)

    def step(self, s):
        kv, a, w, ctx = self.kv, self.args, self.w, self.ctx
        inp = self.inputs[s]
        out, lse, scale = self.out, self.lse, self.scale
        if a.paged and s > 0:
            pc = self.pc
            if not (a.separate_score_select or a.separate_calls or a.defrag_every):   # the whole step in one call
                kv.kvtrim_paged_decode_step(ctx, pc, inp["k_new"], inp["v_new"], inp["log_beta_new"], self.pos_news[s], self.nows[s],
                                            self.budget, self.score, self.keep, self.kept, inp["q"], 0, w.n_layers, scale, out, lse,
                                            thr_key_out=self.thr, log_tail_new=inp.get("log_tail_new"), evict_hint=self.per_seq)
                return
            kv.kvtrim_paged_append(ctx, pc, inp["k_new"], inp["v_new"], inp["log_beta_new"], self.pos_news[s],
                                   log_tail_new=inp.get("log_tail_new"))
            if a.separate_score_select:
                kv.kvtrim_paged_score(ctx, pc, self.nows[s], self.score)
                kv.kvtrim_paged_select(ctx, pc, self.score, self.budget, self.keep, self.kept, self.thr)
            else:
                kv.kvtrim_paged_score_select(ctx, pc, self.nows[s], self.budget, self.score, self.keep, self.kept, self.thr,
                                             evict_hint=self.per_seq)
            kv.kvtrim_paged_evict(ctx, pc, self.keep)
            if a.defrag_every and s % a.defrag_every == 0:
                kv.kvtrim_paged_defrag(ctx, pc)
            kv.kvtrim_paged_attn(ctx, pc, inp["q"], 0, w.n_layers, scale, out, lse)
            return
        cur = self.cur
        if a.inplace and not (a.unfused or a.separate_score_select or a.separate_calls) and s > 0:
            # the whole step in one call, inside the cache (three kernels) or - every ROOM-th step - out of place
            new = (inp["k_new"], inp["v_new"], inp["log_beta_new"], self.pos_news[s], 1, self.nows[s], self.budget, self.score,
                   self.keep, self.kept)
            dst = self.spare[self.flip]
            if s % a.inplace:
                kv.kvtrim_decode_step_inplace(ctx, cur, *new, dst, inp["q"], 0, w.n_layers, scale, out, lse, thr_key_out=self.thr,
                                              log_tail_new=inp.get("log_tail_new"), evict_hint=self.per_seq)
            else:
                kv.kvtrim_decode_step(ctx, cur, *new, dst, self.reserve, inp["q"], 0, w.n_layers, scale, out, lse,
                                      thr_key_out=self.thr, log_tail_new=inp.get("log_tail_new"), evict_hint=self.per_seq)
                self.cur = dst
                self.flip ^= 1
            return
        if not (a.paged or a.inplace or a.unfused or a.separate_score_select or a.separate_calls):
            # the whole step in one call (three kernels for a decode step; the first step, with hint 0, runs the
            # calls it stands for one after the other)
            dst = self.spare[self.flip]
            kv.kvtrim_decode_step(ctx, cur, inp["k_new"], inp["v_new"], inp["log_beta_new"], self.pos_news[s], 1, self.nows[s],
                                  self.budget, self.score, self.keep, self.kept, dst, self.reserve, inp["q"], 0, w.n_layers,
                                  scale, out, lse, thr_key_out=self.thr, log_tail_new=inp.get("log_tail_new"),
                                  evict_hint=self.per_seq if s > 0 else 0)
            self.cur = dst
            self.src = None
            self.flip ^= 1
            return
        kv.kvtrim_append(ctx, cur, inp["k_new"], inp["v_new"], inp["log_beta_new"], self.pos_news[s], 1,
                         log_tail_new=inp.get("log_tail_new"))
        self.select(s, cur)
        if a.paged:                             # first step: the survivors of the prefill go into pages
            kv.kvtrim_paged_build(ctx, cur, self.keep, self.kept, self.pc)
            kv.kvtrim_paged_attn(ctx, self.pc, inp["q"], 0, w.n_layers, scale, out, lse)
            self.cur = self.src = None
            return
        dst = self.spare[self.flip]
        if a.inplace and s > 0 and s % a.inplace:
            # the other cache lends its arrays as parking space; the segments stay where they are
            if a.unfused:                      # stage 3 alone in place, then the stand-alone attention on the same cache
                kv.kvtrim_compact_inplace(ctx, cur, self.keep, self.kept, dst)
                kv.kvtrim_decode_attn(ctx, cur, inp["q"], 0, w.n_layers, scale, out, lse)
            else:
                kv.kvtrim_compact_attn_inplace(ctx, cur, self.keep, self.kept, dst, inp["q"], 0, w.n_layers, scale, out, lse)
            return
        if a.unfused:
            kv.kvtrim_compact(ctx, cur, self.keep, self.kept, dst, self.reserve)
            kv.kvtrim_decode_attn(ctx, dst, inp["q"], 0, w.n_layers, scale, out, lse)
        else:
            kv.kvtrim_compact_attn(ctx, cur, self.keep, self.kept, dst, self.reserve, inp["q"], 0, w.n_layers, scale, out, lse)
        self.cur = dst
        self.src = None                         # (drops the prefill cache after the first step)
        self.flip ^= 1


def moved_bytes(w, a, n_cand, n_ret, rows_written_in_place=None):
    """Compulsory HBM bytes of the calls a step actually makes (every array counted once per kernel that has to
    read or write it) - unlike the stage-by-stage model, which charges the attention a second read of K/V that the
    fused call does not make."""
    D = w.head_dim
    tail = 0 if a.horizon == 1 else 4
    R = 4 * D + 8 + tail
    nq = w.n_seq * w.n_layers * w.n_q_heads
    one_call = not (a.paged or a.inplace or a.unfused or a.separate_score_select or a.separate_calls)
    m = {"append": 2 * R * w.nseg}
    if a.paged and not a.separate_score_select:
        m["paged_score_select"] = (8 + tail + 4 + 4 + 4 + 1) * n_cand   # scoring pass (score out), mask pass (score and position in, mask out)
    elif a.separate_score_select or a.paged:
        m["score"] = (8 + tail + 4) * n_cand                       # log beta, position (, tail) in; score out
        m["select"] = (3 * 4 + 4 + 1) * n_cand                     # three histogram passes and the mask pass read the score; mask out
    elif one_call:
        m["score + select (inside decode_step)"] = (8 + tail + 4 + 1) * n_cand   # one scoring pass (score out); the mask is written by the row mover
    else:
        m["score_select"] = (8 + tail + 4 + 4 + 1) * n_cand        # one scoring pass (score out), one mask pass (score in, mask out)
    if a.paged:
        if a.separate_score_select or a.separate_calls or a.defrag_every:
            m["evict"] = 5 * n_cand                                # mask and position in (the few freed slots out)
        # (in the one call the eviction rides in the mask kernel, which reads the positions anyway)
        m["attend"] = (4 * D + 4) * n_ret + 6 * D * nq             # K, V and position of every live slot; q in, out out
    elif a.inplace:
        moved = rows_written_in_place or 0
        if a.unfused:
            # stage 3 alone in place touches only the rows that move (read and written once); the attention reads all
            per_ip = n_cand + 2 * R * moved
            per_oop = n_cand + 2 * R * n_ret
            m["compact (in place; one step in %d out of place)" % a.inplace] = ((a.inplace - 1) * per_ip + per_oop) // a.inplace
            m["decode_attn"] = 4 * D * n_ret + 6 * D * nq
        else:
            per_ip = n_cand + R * n_ret + R * moved + 6 * D * nq
            per_oop = n_cand + 2 * R * n_ret + 6 * D * nq
            m["compact_attn (in place; one step in %d out of place)" % a.inplace] = ((a.inplace - 1) * per_ip + per_oop) // a.inplace
    elif a.unfused:
        m["compact"] = n_cand + 2 * R * n_ret
        m["decode_attn"] = 4 * D * n_ret + 6 * D * nq
    elif one_call:
        m["compact + attend (inside decode_step)"] = 2 * R * n_ret + 6 * D * nq   # every retained entry in and out once; q in, out out
    else:
        m["compact_attn"] = n_cand + 2 * R * n_ret + 6 * D * nq    # mask in; every retained entry in and out once; q in, out out
    return m


def run_decode(args, brief=False):
    """Decode steps of one workload in one variant; returns the result (what a stand-alone run prints as its JSON line).
    brief: a side measurement of the default run - no in-place leg and no extra runs behind it."""
    import gc
    import numpy as np
    import torch
    import kvtrim_inputs as ki
    import paper_2605_09649_amd as kv

    dev = "cuda:0"
    torch.cuda.set_device(0)
    w = ki.workload(args.workload, prefill=args.prefill, seed_index=args.seed)
    reserve = args.inplace if args.inplace else 1                 # free slots behind every segment after an out-of-place step
    K, W = args.steps, max(args.warmup, 1)
    cpu_steps = 0 if args.no_cpu_baseline else args.cpu_steps
    cpu_steps_1t = min(CPU_STEPS_ONE_THREAD, cpu_steps // 2)
    G_STEPS = 20 if args.graph else 0         # eager, profiled steps before a captured region
    n_steps = K + W + G_STEPS + cpu_steps + 2 # + the steps that are replayed on the CPU oracle, + two that are looked at
    per_seq = w.n_layers * w.n_kv_heads

    # ---- the library's code objects are loaded by a throw-away run of the same calls on a small context of the same
    # shape, so that the first step below times the eviction and not the loading
    t0 = time.time()
    # (paged: long enough for the page pool, with its spare pages per segment, to stay under a quarter of the prefill -
    # the sparse first eviction then runs the same kernels as at full size)
    small = ki.workload(args.workload, prefill=min(4096 if args.paged else 512, min(w.prefill)))
    warm = Runner(small, args, 4, reserve, dev)
    for s in range(4):
        warm.step(s)
    torch.cuda.synchronize()
    assert kv.kvtrim_poll_error(warm.ctx) == 0
    del warm
    gc.collect()
    torch.cuda.empty_cache()

    r = Runner(w, args, n_steps, reserve, dev)
    ctx, total0, B = r.ctx, r.total0, sum(w.budget)
    log(f"[bench] {w.name}: prefill cache of {total0} entries, {2 * total0 * w.head_dim * 2 / 1e9:.2f} GB K/V; "
        f"set up (with the code-object warm-up) in {time.time() - t0:.1f}s")

    if args.pmc_calibration:                  # 2^28 floats in, 2^28 floats out, one elementwise copy kernel
        ca = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        cb = torch.empty_like(ca)
        cb.copy_(ca)
        torch.cuda.synchronize()
        del ca, cb
        torch.cuda.empty_cache()

    # ---- the first step evicts from the full prefill down to the budget: wall time between two events, and the
    # sum of its kernels' own durations
    all_kernels = (1 << kv.binding.N_KERNELS) - 1
    kv.kvtrim_profile_begin(ctx, all_kernels)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    r.step(0)
    e1.record()
    torch.cuda.synchronize()
    first_ms = e0.elapsed_time(e1)
    prof0 = kv.kvtrim_profile_end(ctx)
    first_kernels_ms = sum(ms for ms, _ in prof0.values())
    assert kv.kvtrim_poll_error(ctx) == 0, "device-side error in the first step"
    gc.collect()
    torch.cuda.empty_cache()
    for s in range(1, W):
        r.step(s)
    torch.cuda.synchronize()
    n_ret = int(r.kept.sum().item())
    n_cand = n_ret + w.nseg
    log(f"[bench] first step (prefill -> budget): {first_ms:.3f} ms ({first_kernels_ms:.3f} ms in its "
        f"{sum(n for _, n in prof0.values())} kernels); steady state: {n_cand} candidates, {n_ret} retained")
    if args.kernel_times:
        for name, (kms, n) in sorted(prof0.items(), key=lambda kvp: -kvp[1][0]):
            log(f"[bench]   first step: {name:<18s} {1e3 * kms / n:7.1f} us x {n}")

    # ---- timed region: exactly K steps; the dominant kernels are bracketed by HIP events on the launch stream
    mask = (1 << 8) | (1 << 10) | (1 << 13)   # k_cmp_copy, k_att_partial, k_cmp_attn
    if args.kernel_times:
        mask = all_kernels                    # every kernel (the events then add to the step time)
    kv.kvtrim_profile_begin(ctx, mask)
    torch.cuda.synchronize()
    if args.graph:
        for s in range(W, W + G_STEPS):       # per-kernel durations: events cannot be recorded inside a capture
            r.step(s)
        torch.cuda.synchronize()
        prof = kv.kvtrim_profile_end(ctx)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):         # the library only enqueues kernels on the current stream
            for s in range(W + G_STEPS, W + G_STEPS + K):
                r.step(s)
        torch.cuda.synchronize()
        t_begin = time.perf_counter()
        graph.replay()
        torch.cuda.synchronize()
        t_end = time.perf_counter()
    else:
        t_begin = time.perf_counter()
        for s in range(W, W + K):
            r.step(s)
        torch.cuda.synchronize()
        t_end = time.perf_counter()
        prof = kv.kvtrim_profile_end(ctx)
    assert kv.kvtrim_poll_error(ctx) == 0, "device-side error in the timed region"
    if args.kernel_times:
        for name, (ms, n) in sorted(prof.items(), key=lambda kvp: -kvp[1][0]):
            log(f"[bench]   {name:16s} {ms / n * 1e3:8.1f} us x {n}")
    ms_per_step = (t_end - t_begin) * 1e3 / K
    sel_paths = kv.kvtrim_select_path_counts(ctx)
    next_step = W + G_STEPS + K               # first step after the timed region

    # ---- byte models.  stage model: what the four stages move when each runs on its own (the benchmark's figure);
    # moved: the compulsory bytes of the calls this run makes.
    alg = algorithmic_bytes(w, n_cand, n_ret, args.horizon)
    moved_rows = None
    if args.inplace and not args.paged:
        # how many rows an in-place step writes depends on the data: counted on the step after the timed region
        s_extra = next_step
        if s_extra % args.inplace == 0:
            r.step(s_extra)
            s_extra += 1
        inp = r.inputs[s_extra]
        kv.kvtrim_append(ctx, r.cur, inp["k_new"], inp["v_new"], inp["log_beta_new"], r.pos_news[s_extra], 1,
                         log_tail_new=inp.get("log_tail_new"))
        r.select(s_extra, r.cur)
        torch.cuda.synchronize()
        moved_rows = rows_moved_in_place(r.cur, r.keep)
        kv.kvtrim_compact_attn_inplace(ctx, r.cur, r.keep, r.kept, r.spare[r.flip], inp["q"], 0, w.n_layers, r.scale, r.out, r.lse)
        torch.cuda.synchronize()
        next_step = s_extra + 1
        log(f"[bench] in place: {moved_rows} of {n_ret} retained rows ({100.0 * moved_rows / n_ret:.1f} %) lie behind an eviction "
            f"and are written; the others are only read")
    moved = moved_bytes(w, args, n_cand, n_ret, moved_rows)
    moved_total = sum(moved.values())
    stage_model_bytes = None
    nq_bytes = 6 * w.head_dim * w.n_seq * w.n_layers * w.n_q_heads
    if args.paged:
        dom, dom_bytes = "k_att_partial", moved["attend"]
    elif args.unfused and args.inplace:
        dom, dom_bytes = "k_att_partial", alg["attend"]
    elif args.unfused:
        dom, dom_bytes = "k_cmp_copy", alg["compact"]
    else:
        # The fused kernel does the work of stages 3 and 4 but reads K/V once.  Its roofline is priced on the bytes the
        # fused operation cannot avoid: every retained entry read once and written once, the mask, q and out.
        dom = "k_cmp_attn"                      # (the one-call step's row mover is bracketed under the same name)
        dom_bytes = alg["compact"] + n_cand + nq_bytes   # mask in (separate calls) / out (one call)
        stage_model_bytes = alg["compact"] + alg["attend"]
        if args.inplace:
            dom_bytes = [v for k, v in moved.items() if k.startswith("compact_attn")][0]
            stage_model_bytes = None
    if dom not in prof:                       # the cache is too large for the fused kernel: the library ran the two stages
        dom, dom_bytes, stage_model_bytes = "k_cmp_copy", alg["compact"], None
    dom_ms, dom_n = prof[dom]
    dom_avg_ms = dom_ms / dom_n
    achieved = dom_bytes / (dom_avg_ms * 1e-3) / 1e9
    alg_total = sum(alg.values())
    log(f"[bench] {ms_per_step:.4f} ms/step: {moved_total / (ms_per_step * 1e-3) / 1e9:.0f} GB/s on the {moved_total / 1e9:.3f} GB the "
        f"calls move ({100 * moved_total / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS:.1f} % of peak); stage model "
        f"{alg_total / 1e9:.3f} GB -> {alg_total / (ms_per_step * 1e-3) / 1e9:.0f} GB/s; {dom} {dom_avg_ms:.4f} ms "
        f"({achieved:.0f} GB/s on its compulsory bytes)")
    if not args.separate_score_select:
        log(f"[bench] decode-step selections: {sel_paths[0]} from the candidate list, {sel_paths[1]} by the single-block fallback")
    second = None
    if args.unfused and args.inplace:
        mv_ms, mv_n = prof["k_cmp_copy"]       # (the in-place row mover is bracketed under the row mover's name)
        second = {"kernel": "k_cmp_move_inplace", "avg_launch_ms": mv_ms / mv_n}
    elif args.unfused:
        att_ms, att_n = prof["k_att_partial"]
        second = {"kernel": "k_att_partial", "avg_launch_ms": att_ms / att_n,
                  "achieved": alg["attend"] / (att_ms / att_n * 1e-3) / 1e9}

    variant = "paged" if args.paged else "inplace" if args.inplace else "unfused" if args.unfused else "fused"
    tag = {"long": "long_128k", "llama": "llama_32k", "vlm": "vlm", "tiny": "tiny", "multiturn": "multiturn"}[w.name] + \
          {"fused": "", "paged": "_paged", "inplace": "_inplace", "unfused": "_unfused"}[variant]
    one_call = not (args.paged or args.inplace or args.unfused or args.separate_score_select or args.separate_calls)
    calls = ("decode_step (append, stages 1-4 in one call; three kernels per decode step where the shape allows)" if one_call else
             ("paged_decode_step (append, score_select, evict, attn in one call; paged layout: no K/V moved)"
              if not (args.separate_score_select or args.separate_calls or args.defrag_every) else
              "paged_append, " + ("paged_score, paged_select" if args.separate_score_select else "paged_score_select") +
              ", paged_evict, paged_attn (paged layout: no K/V moved)") if args.paged else
             ("append, " + ("score, select_global" if args.separate_score_select else "score_select") + ", " +
              ("compact, decode_attn" if args.unfused and not args.inplace else
               "compact_inplace, decode_attn" if args.unfused else
               f"compact_attn_inplace (stages 3+4 fused inside the cache, {args.inplace} free slots per segment; every "
               f"{args.inplace}th step an out-of-place compact_attn)" if args.inplace else
               "compact_attn (stages 3+4 fused)")))
    if args.inplace and not (args.paged or args.unfused or args.separate_score_select or args.separate_calls):
        calls = (f"decode_step_inplace (append, stages 1-4 in one call, stages 3+4 inside the cache: three kernels per decode step; "
                 f"{args.inplace} free slots per segment, every {args.inplace}th step an out-of-place decode_step)")
    result = {
        "metric": metric_name(w),
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
                        f"{w.prefill[0] if w.n_seq == 1 else 'lengths ' + str(min(w.prefill)) + '..' + str(max(w.prefill))} prefilled, "
                        f"B={B} ({n_cand} candidates/step, {n_ret} retained), "
                        f"score lookahead horizon {args.horizon if args.horizon > 0 else 'infinite'}",
            "seed_index": args.seed,
            "stages": calls,
            "first_step_ms": first_ms,
            "first_step_kernels_ms": first_kernels_ms,
            "first_step_note": "eviction from the whole prefill down to the budget, timed after a throw-away run of the same "
                               "calls on a small context (code objects loaded); kernels_ms = sum of its kernels' durations",
            "launch": "one HIP graph holding the K timed steps, replayed once" if args.graph else "eager launches",
        },
        "end_to_end": {
            "moved_bytes_per_step": moved_total,
            "moved_GBps": moved_total / (ms_per_step * 1e-3) / 1e9,
            "frac_of_hbm_peak_on_moved_bytes": moved_total / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "moved_bytes_by_call": moved,
            "moved_note": "compulsory HBM bytes of the calls this run makes (every array once per kernel that reads or writes it)",
            "stage_model_bytes_per_step": alg_total,
            "stage_model_GBps": alg_total / (ms_per_step * 1e-3) / 1e9,
            "frac_of_hbm_peak_on_stage_model": alg_total / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "stage_model_bytes_by_stage": alg,
            "stage_model_note": "a MODEL, not traffic: the bytes of the four stages run one by one (score 8 B, select 5 B per "
                                "candidate; compact 2(4D+8) B, attend 4D B per retained entry); a fused call moves fewer",
        },
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": measured_traffic(tag, dom),
                     "algorithmic_bytes_per_launch": dom_bytes, "avg_launch_ms": dom_avg_ms, "launches": dom_n,
                     "stage_model_bytes_per_launch": stage_model_bytes,
                     "stage_model_achieved": (stage_model_bytes / (dom_avg_ms * 1e-3) / 1e9) if stage_model_bytes else None,
                     "second_kernel": second},
    }
    if not args.separate_score_select:
        result["config"]["decode_step_selection"] = {"from_candidate_list": sel_paths[0], "single_block_fallback": sel_paths[1]}
    if moved_rows is not None:
        result["config"]["in_place"] = {"room": args.inplace, "rows_written_sampled": moved_rows, "rows_retained": n_ret}
    if args.paged:
        result["config"]["pages"] = {"page_size": kv.PAGE_SIZE, "n_pages": r.pc.n_pages,
                                     "in_use_after_timed_region": int(r.pc.seg_pages.sum().item())}

    # ---- CPU baseline: the oracle replays more steps of the same workload on the host cores, and the GPU's results of
    # those steps are checked against it (selection / compaction bit-exact, attention 5e-3)
    if cpu_steps:
        import oracle
        from harness import attn_error, compare_cache_contents, compare_caches, device_cache_to_host, sampled_step_check
        from helpers import bf16_bits
        budget_np = np.array(list(w.budget), np.int64)
        live_bytes = 2 * n_ret * w.head_dim * 2
        if live_bytes <= WHOLE_CACHE_PARITY_BYTES:
            if args.paged:                      # the pages as the oracle's ragged cache: each segment in position order
                from paged_harness import PagedHost
                ph = PagedHost(r.pc)
                hc = ph.as_ragged(oracle.Shape(w.n_seq, w.n_layers, w.n_kv_heads, w.n_q_heads, w.head_dim), reserve)
                del ph
            else:
                hc = device_cache_to_host(w, r.cur)
            t_all, t_one, ok_sel, err = 0.0, 0.0, True, 0.0
            n_all = cpu_steps - cpu_steps_1t
            threads_all = oracle.threads()
            for i, s in enumerate(range(next_step, next_step + cpu_steps)):
                one = i >= n_all
                oracle.set_threads(1 if one else threads_all)
                inp = {k: v.cpu() for k, v in r.inputs[s].items()}
                now = r.now0 + s + 1
                pos_new = np.repeat(now, per_seq).astype(np.int32)
                kb, vb, qb = bf16_bits(inp["k_new"]), bf16_bits(inp["v_new"]), bf16_bits(inp["q"])
                lbn = inp["log_beta_new"].numpy()
                ltn = inp["log_tail_new"].numpy() if args.horizon != 1 else None
                t_cpu = time.perf_counter()
                oracle.append(hc, kb, vb, lbn, pos_new, log_tail_new=ltn)
                score_ref = oracle.score(hc, now)
                keep_ref, kept_ref, thr_ref = oracle.select(hc, score_ref, budget_np)
                hc = oracle.compact(hc, keep_ref, r.dst_cap, reserve)
                out_ref, _ = oracle.attend(hc, qb, r.scale)
                dt = time.perf_counter() - t_cpu
                t_one, t_all = (t_one + dt, t_all) if one else (t_one, t_all + dt)
                r.step(s)
                torch.cuda.synchronize()
                ok_sel = ok_sel and bool(np.array_equal(r.kept.cpu().numpy(), kept_ref)) \
                    and bool(np.array_equal(r.thr.cpu().numpy().view(np.uint32), thr_ref))
                err = max(err, attn_error(r.out.cpu().numpy(), out_ref))
            oracle.set_threads(threads_all)
            if args.paged:
                ph = PagedHost(r.pc)
                ok_cache = ph.structure_problems() == [] and ph.equals(hc)
            elif args.inplace:                  # the segments keep their starts: contents are compared segment by segment
                ok_cache = compare_cache_contents(device_cache_to_host(w, r.cur), hc)
            else:
                ok_cache = compare_caches(device_cache_to_host(w, r.cur), hc)
            del hc
            log(f"[bench] oracle on the host: {n_all} steps with {threads_all} threads in {t_all:.2f} s, {cpu_steps_1t} steps with one "
                f"thread in {t_one:.2f} s; GPU vs oracle on those steps: selection equal={ok_sel}, final cache equal={ok_cache}, "
                f"attention err={err:.2e}")
            assert kv.kvtrim_poll_error(ctx) == 0 and ok_sel and ok_cache and err <= 5e-3, "GPU steps disagree with the oracle"
            result["cpu_baseline"] = {
                "value": n_all / t_all, "unit": "steps/s", "cores": threads_all, "kind": "oracle",
                "sample": f"{n_all} full steps of the same workload after the timed region (append, score, full-sort select, "
                          f"compact, fp64 attention); the attention loop runs on {threads_all} threads (OpenMP over segments), "
                          "the other stages on one",
                "single_thread": None if not cpu_steps_1t else {
                    "value": cpu_steps_1t / t_one, "unit": "steps/s", "cores": 1,
                    "sample": f"{cpu_steps_1t} further steps with every stage on one thread"}}
            result["parity_on_sampled_step"] = {"steps": cpu_steps, "mode": "whole cache, every step",
                                                "select_compact_bit_exact": ok_sel and ok_cache, "attn_max_norm_rel_err": err}
        else:
            # too large to replay whole on the host: one more step, selection and metadata whole, rows and attention sampled
            assert not (args.paged or args.inplace), "sampled parity covers the out-of-place ragged step"
            s = next_step
            src = r.cur
            t_cpu = time.perf_counter()
            r.step(s)
            torch.cuda.synchronize()
            chk = sampled_step_check(w, src, r.now0 + s + 1, budget_np, reserve,
                                     {"score": r.score, "keep": r.keep, "kept": r.kept, "thr": r.thr, "dst": r.cur, "out": r.out, "lse": r.lse},
                                     q=r.inputs[s]["q"], scale=r.scale)
            ok = all(chk[k] for k in ("score_equal", "keep_equal", "kept_equal", "thr_equal", "tables_equal", "metadata_equal", "rows_equal"))
            log(f"[bench] sampled parity of one step ({time.perf_counter() - t_cpu:.1f} s): selection and metadata whole equal={ok}, "
                f"rows and attention on {len(chk['sampled_segments'])} segments: err={chk['attn_err']:.2e}")
            assert kv.kvtrim_poll_error(ctx) == 0 and ok and chk["attn_err"] <= 5e-3, "GPU step disagrees with the oracle"
            result["parity_on_sampled_step"] = {"steps": 1, "mode": f"selection, counts, thresholds and compaction metadata whole; K/V rows "
                                                f"and attention on {len(chk['sampled_segments'])} segments",
                                                "select_compact_bit_exact": ok, "attn_max_norm_rel_err": chk["attn_err"]}
        next_step += cpu_steps

    # ---- the same steps with stages 3+4 done inside the cache (kvtrim_decode_step_inplace), timed beside the metric's
    # out-of-place step: ROOM free slots behind every segment, every ROOM-th step out of place to even them out (at
    # least one such step falls inside the timed steps); the last step is checked against the oracle
    K2 = min(K, 128)
    ROOM = max(2, min(64, K2 // 2))
    cap_room = n_ret + w.nseg * ROOM + 8
    plain = not (brief or args.no_inplace_leg or args.paged or args.unfused or args.inplace or args.graph or args.kernel_times or args.pmc_calibration
                 or args.separate_score_select or args.separate_calls)
    if plain and cap_room <= r.cap:
        s0 = n_steps
        extra, extra_now, extra_pos = [], [], []
        for s in range(s0, s0 + K2 + 1):
            extra.append(ki.decode_inputs(w, s, device=dev, horizon=args.horizon))
            now = r.now0 + s + 1
            extra_now.append(torch.from_numpy(now).to(dev))
            extra_pos.append(torch.from_numpy(np.repeat(now, per_seq).astype(np.int32)).to(dev))
        big = [kv.Cache.empty(w.nseg, w.head_dim, cap_room, dev, with_tail=args.horizon != 1) for _ in range(2)]
        cur, other = r.cur, big[0]

        def step_room(i, in_place):
            nonlocal cur, other
            inp = extra[i]
            new = (inp["k_new"], inp["v_new"], inp["log_beta_new"], extra_pos[i], 1, extra_now[i], r.budget, r.score, r.keep, r.kept)
            if in_place:
                kv.kvtrim_decode_step_inplace(ctx, cur, *new, other, inp["q"], 0, w.n_layers, r.scale, r.out, r.lse,
                                              thr_key_out=r.thr, log_tail_new=inp.get("log_tail_new"), evict_hint=per_seq)
            else:
                kv.kvtrim_decode_step(ctx, cur, *new, other, ROOM, inp["q"], 0, w.n_layers, r.scale, r.out, r.lse,
                                      thr_key_out=r.thr, log_tail_new=inp.get("log_tail_new"), evict_hint=per_seq)
                cur, other = other, (big[1] if other is big[0] else big[0])

        step_room(0, False)                                        # into a cache with room behind every segment
        torch.cuda.synchronize()
        t_begin = time.perf_counter()
        for i in range(1, K2):
            step_room(i, i % ROOM != 0)
        torch.cuda.synchronize()
        ms_room = (time.perf_counter() - t_begin) * 1e3 / (K2 - 1)
        n_oop = sum(1 for i in range(1, K2) if i % ROOM == 0)
        parity_ip = None
        if cpu_steps:                                              # the last step, in place, against the oracle
            hc = device_cache_to_host(w, cur)
            i = K2
            inp = {k: v.cpu() for k, v in extra[i].items()}
            now = r.now0 + s0 + i + 1
            pos_new = np.repeat(now, per_seq).astype(np.int32)
            oracle.append(hc, bf16_bits(inp["k_new"]), bf16_bits(inp["v_new"]), inp["log_beta_new"].numpy(), pos_new,
                          log_tail_new=inp["log_tail_new"].numpy() if args.horizon != 1 else None)
            keep_ref, kept_ref, thr_ref = oracle.select(hc, oracle.score(hc, now), budget_np)
            hc = oracle.compact(hc, keep_ref, cap_room, 1)
            out_ref, _ = oracle.attend(hc, bf16_bits(inp["q"]), r.scale)
            step_room(i, i % ROOM != 0)
            torch.cuda.synchronize()
            ok = bool(np.array_equal(r.kept.cpu().numpy(), kept_ref)) and compare_cache_contents(device_cache_to_host(w, cur), hc)
            err_ip = attn_error(r.out.cpu().numpy(), out_ref)
            assert ok and err_ip <= 5e-3, "in-place step disagrees with the oracle"
            parity_ip = {"select_compact_bit_exact": ok, "attn_max_norm_rel_err": err_ip, "in_place": i % ROOM != 0}
            del hc
        assert kv.kvtrim_poll_error(ctx) == 0 and int(r.kept.sum().item()) == n_ret and bool(torch.isfinite(r.out).all())
        log(f"[bench] the same steps compacting in place: {ms_room:.4f} ms/step ({1e3 / ms_room:.0f} steps/s), "
            f"{n_oop} of the {K2 - 1} timed steps out of place")
        result["in_place_variant"] = {
            "ms_per_step": ms_room, "value": 1e3 / ms_room, "unit": "steps/s", "steps": K2 - 1, "room": ROOM,
            "out_of_place_steps_in_timed_region": n_oop, "parity_on_last_step": parity_ip,
            "what": "kvtrim_decode_step_inplace (three kernels per decode step): a row moves only if an entry before it in its "
                    f"segment was evicted; every {ROOM}th step is an out-of-place kvtrim_decode_step that evens the free slots out"}
        del big, extra
    del r
    gc.collect()
    torch.cuda.empty_cache()
    return result


def summary_of(res):
    """The figures of a side measurement that go into the main line."""
    e = res["end_to_end"]
    return {"workload": res["config"]["workload"], "calls": res["config"]["stages"], "steps": res["steps"],
            "ms_per_step": res["ms_per_step"], "value": res["value"], "unit": res["unit"],
            "first_step_ms": res["config"]["first_step_ms"], "first_step_kernels_ms": res["config"]["first_step_kernels_ms"],
            "moved_bytes_per_step": e["moved_bytes_per_step"], "frac_of_hbm_peak_on_moved_bytes": e["frac_of_hbm_peak_on_moved_bytes"],
            "stage_model_bytes_per_step": e["stage_model_bytes_per_step"],
            "frac_of_hbm_peak_on_stage_model": e["frac_of_hbm_peak_on_stage_model"],
            "dominant_kernel": {k: res["roofline"][k] for k in ("kernel", "avg_launch_ms", "achieved", "frac")},
            "parity": res.get("parity_on_sampled_step"),
            "decode_step_selection": res["config"].get("decode_step_selection")}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default="long", choices=["long", "llama", "vlm", "tiny", "multiturn"])
    ap.add_argument("--prefill", type=int, default=None, help="override the prefilled length (scaled-down run)")
    ap.add_argument("--seed", type=int, default=0, metavar="I",
                    help="another seeded draw of every random input of the workload's recipe (0: the default inputs)")
    ap.add_argument("--horizon", type=int, default=1,
                    help="lookahead horizon of the score: 1 = the metric's form, 2 = the paper's inference default, 0 = infinite")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-steps", type=int, default=CPU_STEPS,
                    help="steps the CPU oracle replays (and the GPU is checked on) after the timed region")
    ap.add_argument("--only", action="store_true",
                    help="time the named workload and variant only: no paged / other-workload side measurements behind the default run")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy, the known-size reference for rocprofv3 --pmc counters")
    ap.add_argument("--unfused", action="store_true",
                    help="run stages 3 and 4 as two calls (kvtrim_compact, kvtrim_decode_attn) instead of the fused one")
    ap.add_argument("--separate-calls", action="store_true",
                    help="run the step as append, score_select, compact_attn instead of the one call kvtrim_decode_step")
    ap.add_argument("--separate-score-select", action="store_true",
                    help="run stages 1 and 2 as two calls (kvtrim_score, kvtrim_select_global) instead of kvtrim_score_select")
    ap.add_argument("--paged", action="store_true",
                    help="steady state on the paged layout: eviction frees slots of fixed-size pages and moves no K/V "
                         "(paged_append, paged_score_select, paged_evict, paged_attn)")
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
    ap.add_argument("--no-inplace-leg", action="store_true",
                    help="do not time the in-place variant behind the metric's steps (for profiles: its launches of the scoring and "
                         "merge kernels would mix into the per-kernel means)")
    ap.add_argument("--inplace", type=int, default=0, metavar="ROOM",
                    help="compact inside the cache (kvtrim_compact_attn_inplace: rows move only behind an eviction) with ROOM "
                         "free slots behind every segment; every ROOM-th step is an out-of-place step that evens the room out")
    ap.add_argument("--one-call", action="store_true",
                    help="with --chunk (ragged layout): the chunk step through kvtrim_append_compact, which moves the new rows "
                         "once, from the caller's buffers to the compacted cache")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    if args.one_call and (not args.chunk or args.paged):
        ap.error("--one-call needs --chunk and the ragged layout")
    if args.chunk:
        if not 1 <= args.chunk <= 4096:
            ap.error("--chunk takes 1 .. 4096 tokens")
        return bench_chunk(args)
    if args.gate:
        return bench_gate(args)
    if args.paged and args.unfused:
        ap.error("--paged and --unfused exclude each other")
    if args.inplace and (args.paged or args.inplace < 2):
        ap.error("--inplace takes a room of at least 2 slots and excludes --paged")
    if args.defrag_every and not args.paged:
        ap.error("--defrag-every needs --paged")

    result = run_decode(args)
    default_run = not (args.only or args.paged or args.unfused or args.inplace or args.graph or args.kernel_times or
                       args.pmc_calibration or args.separate_score_select or args.separate_calls or args.prefill or args.horizon != 1 or
                       args.workload != "long")
    if default_run:
        # side measurements of the default run (each a short run of its own, after the metric's): the same workload on
        # the paged layout, and the decode step of the other workloads; each with a parity check against the oracle
        import copy
        side = copy.copy(args)
        side.steps, side.warmup, side.cpu_steps = min(args.steps, 50), 3, 0 if args.no_cpu_baseline else 4
        side.paged = True
        t0 = time.time()
        result["paged_variant"] = summary_of(run_decode(side, brief=True))
        log(f"[bench] paged variant: {result['paged_variant']['ms_per_step']:.4f} ms/step ({time.time() - t0:.0f} s)")
        side.paged = False
        result["other_workloads"] = {}
        for name in ("tiny", "llama", "vlm", "multiturn"):
            side.workload = name
            side.steps = min(args.steps, 20 if name == "multiturn" else 50)
            t0 = time.time()
            result["other_workloads"][name] = summary_of(run_decode(side, brief=True))
            log(f"[bench] {name}: {result['other_workloads'][name]['ms_per_step']:.4f} ms/step ({time.time() - t0:.0f} s)")
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
