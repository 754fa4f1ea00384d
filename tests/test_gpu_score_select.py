"""GPU parity of kvtrim_score_select (stages 1 + 2 in one call) against the oracle's score + full sort:
scores, mask, per-segment counts and threshold key bit for bit, in both of its forms - the radix passes with the
score fused into the first (evict_hint 0) and the decode-step form (candidate list + ranking, with its single-block
fallback) - through whole decode loops (the rest of the step runs too, so a wrong mask would also show in the
compacted cache and the attention)."""
import numpy as np
import pytest
import torch

import kvtrim_inputs as ki
import oracle
import paper_2605_09649_amd as kv
from harness import run_steps_both
from helpers import host_cache, live_mask

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
ATTN_TOL = 5e-3


def check(results, what=""):
    for i, r in enumerate(results):
        assert r["status"] == 0, (what, i, r)
        assert r["score_equal"], (what, i, "score bits differ")
        assert r["keep_equal"], (what, i, "selection differs")
        assert r["cache_equal"], (what, i, "compacted cache differs")
        assert r["attn_err"] <= ATTN_TOL and r["lse_err"] <= 2e-3 and r["lse_inf_equal"], (what, i, r)


def wl(S, L, H, G, D):
    return ki.Workload("t", 0, S, L, H, G * H, D, (0,) * S, (0,) * S, 1, 3.0, 1.5)


@pytest.mark.parametrize("hint", [0, 16])
def test_tiny_workload_full_loop(hint):
    w = ki.workload("tiny")                                       # 16 segments: 16 evictions per step once at the budget
    res = run_steps_both(w, steps=16, budget=w.budget, device=DEV, fused=True, hint=hint)
    check(res, hint)
    listed, fallback = res[-1]["path_counts"]
    if hint:
        # the first call has no bound yet (single-block select), the second starts from the bound that one left;
        # from then on the candidate list must carry every step: scores only decay and 16 entries go per step
        assert fallback <= 2 and listed >= 14, (listed, fallback)
    else:
        assert listed == 0 and fallback == 0


@pytest.mark.parametrize("name,prefill,steps", [("llama", 700, 6), ("long", 900, 6), ("vlm", 640, 6), ("multiturn", 600, 4)])
def test_scaled_down_workloads_decode_step_form(name, prefill, steps):
    w = ki.workload(name, prefill=prefill)
    res = run_steps_both(w, steps=steps, budget=w.budget, device=DEV, fused=True, hint=w.n_layers * w.n_kv_heads)
    check(res, name)
    listed, fallback = res[-1]["path_counts"]
    assert listed >= (steps - 2) * w.n_seq - fallback and fallback <= 2 * w.n_seq, (listed, fallback)


def test_radix_passes_leave_the_bound_the_decode_step_form_starts_from():
    # first eviction from the prefill through the radix passes (hint 0), decode steps after it with a hint: the
    # first of them already finds its candidates listed, no sequence ever takes the single-block fallback
    for name, prefill in (("long", 2000), ("vlm", 900)):
        w = ki.workload(name, prefill=prefill)
        per_seq = w.n_layers * w.n_kv_heads
        res = run_steps_both(w, steps=6, budget=w.budget, device=DEV, fused=True, hint=[0, per_seq])
        check(res, name)
        listed, fallback = res[-1]["path_counts"]
        assert fallback == 0 and listed == 5 * w.n_seq, (name, listed, fallback)


@pytest.mark.parametrize("horizon", [2, 0])
def test_lookahead_horizon_tail_enters_the_fused_score(horizon):
    w = ki.workload("tiny", prefill=500)
    for hint in (0, 16):
        check(run_steps_both(w, steps=5, budget=w.budget, device=DEV, fused=True, hint=hint, horizon=horizon), (horizon, hint))


@pytest.mark.parametrize("hint", [0, 4, 60])
@pytest.mark.parametrize("S,L,H,G,D", [(1, 2, 2, 1, 128), (2, 2, 1, 7, 128), (3, 1, 2, 3, 64), (1, 2, 1, 4, 128)])
def test_ragged_segments_spanning_several_blocks(S, L, H, G, D, hint):
    w = wl(S, L, H, G, D)
    rng = np.random.default_rng(S * 1000 + G * 10 + D)
    seg_len = rng.integers(0, 20000, w.nseg)                      # more than one 8192-entry share per segment
    seg_len[rng.integers(0, w.nseg)] = 0
    seg_len[rng.integers(0, w.nseg)] = 8192 * 2 + 1
    c, now = ki.ragged_cache(w, seg_len, reserve=1, salt=G)
    per_seq = [int(seg_len[s * L * H:(s + 1) * L * H].sum()) for s in range(S)]
    budget = [max(1, n // 3) for n in per_seq]
    check(run_steps_both(w, steps=4, budget=budget, device=DEV, cache_dict=c, now0=now.numpy(), fused=True, hint=hint))


def test_budget_changes_from_step_to_step_and_nothing_to_evict():
    # budget far above the count (nothing evicted, the threshold is the lowest key), then at the count, then a
    # drop to a third (many evictions: the list cannot hold them, the fallback runs), then steady, then zero
    w = wl(2, 2, 2, 2, 64)
    rng = np.random.default_rng(8)
    seg_len = rng.integers(50, 900, w.nseg)
    c, now = ki.ragged_cache(w, seg_len, reserve=1, salt=3)
    n0 = [int(seg_len[:4].sum()), int(seg_len[4:].sum())]
    steps = [[10 ** 9, 10 ** 9], [n0[0] + 8, n0[1]], [n0[0] // 3, n0[1] - 5], [n0[0] // 3, n0[1] - 5], [n0[0] // 3, n0[1] - 5],
             [n0[0] // 3 + 2, n0[1] - 9], [0, n0[1] - 9], [5, 0]]
    res = run_steps_both(w, steps=len(steps), budget=[10 ** 9, 10 ** 9], device=DEV, cache_dict=c, now0=now.numpy(), fused=True,
                         hint=8, budget_per_step=steps)
    check(res)


@pytest.mark.parametrize("levels", [1, 2, 5])
def test_quantised_retention_gives_ties_at_the_threshold_every_step(levels):
    # few distinct log beta values: whole groups of entries share a score, the threshold falls inside a group in
    # every step and (segment, position) decides - one level: pure recency, every segment ties with every other
    w = wl(2, 2, 3, 2, 64)
    rng = np.random.default_rng(40 + levels)
    seg_len = rng.integers(100, 1500, w.nseg)
    c, now = ki.ragged_cache(w, seg_len, reserve=1, salt=levels, pos_stride_max=1)
    g = torch.Generator().manual_seed(levels)
    c["log_beta"] = -(torch.randint(0, levels, c["log_beta"].shape, generator=g).to(torch.float32) + 1.0) * 0.125
    budget = [int(seg_len[:6].sum()) // 2, int(seg_len[6:].sum()) - 7]
    for hint in (0, 6, 200):
        clone = {k: (v.clone() if torch.is_tensor(v) else v) for k, v in c.items()}
        check(run_steps_both(w, steps=5, budget=budget, device=DEV, cache_dict=clone, now0=now.numpy(), fused=True, hint=hint),
              (levels, hint))


@pytest.mark.parametrize("seed,long_segments", [(s, False) for s in range(24)] + [(s, True) for s in range(12)])
def test_random_configuration(seed, long_segments):
    from test_gpu_random_sweep import random_case
    w, c, now, budgets = random_case(seed, long_segments=long_segments)
    for hint in (0, 1 + seed % 7, 900):
        clone = {k: (v.clone() if torch.is_tensor(v) else v) for k, v in c.items()}
        res = run_steps_both(w, steps=len(budgets), budget=[max(b[s] for b in budgets) for s in range(w.n_seq)], device=DEV,
                             cache_dict=clone, now0=now.numpy(), fused=True, hint=hint, budget_per_step=budgets)
        check(res, (seed, hint))


@pytest.mark.parametrize("S,L,H", [(600, 1, 2), (1100, 1, 1)])
def test_many_short_sequences(S, L, H):
    rng = np.random.default_rng(77 + S)
    w = ki.Workload("m", 0, S, L, H, 2 * H, 64, (0,) * S, (0,) * S, 1, 3.0, 1.5)
    seg_len = rng.integers(0, 41, w.nseg)
    seg_len[rng.random(w.nseg) < 0.1] = 0
    c, now = ki.ragged_cache(w, seg_len, reserve=1, salt=S, pos_stride_max=2)
    g = torch.Generator().manual_seed(S)
    c["log_beta"] = -(torch.randint(0, 3, c["log_beta"].shape, generator=g).to(torch.float32)) * 0.25
    per_seq = [int(seg_len[s * L * H:(s + 1) * L * H].sum()) for s in range(S)]
    budget = [0 if rng.random() < 0.05 else int(rng.integers(1, max(2, n + 3))) for n in per_seq]
    for hint in (0, 2):
        clone = {k: (v.clone() if torch.is_tensor(v) else v) for k, v in c.items()}
        check(run_steps_both(w, steps=3, budget=budget, device=DEV, cache_dict=clone, now0=now.numpy(), fused=True, hint=hint), (S, hint))


def test_the_context_is_shared_by_unrelated_caches():
    # the carried bound belongs to the context, not to a cache: alternating two unrelated caches on one context makes
    # the bound useless (too low or far too high) - results must not depend on it
    w = wl(1, 2, 2, 2, 64)
    caches = []
    for salt, scale in ((1, 1.0), (2, 30.0)):
        c, now = ki.ragged_cache(w, [3000, 10, 5000, 2222], reserve=1, salt=salt)
        c["log_beta"] = c["log_beta"] * scale
        caches.append((c, now))
    cap = max(c["cap"] for c, _ in caches)
    ctx = kv.Context(1, 2, 2, 4, 64, cap)
    score = torch.zeros(cap, dtype=torch.float32, device=DEV)
    keep = torch.zeros(cap, dtype=torch.uint8, device=DEV)
    kept = torch.zeros(w.nseg, dtype=torch.int32, device=DEV)
    thr = torch.zeros(1, dtype=torch.int32, device=DEV)
    for rnd in range(3):
        for c, now in caches:
            hc = host_cache(w, c)
            n = int(hc.seg_len.sum())
            budget = np.array([n - 4 - rnd], np.int64)
            now_np = now.numpy() + rnd
            s_ref = oracle.score(hc, now_np)
            keep_ref, kept_ref, thr_ref = oracle.select(hc, s_ref, budget)
            dc = kv.Cache.from_dict(c, DEV)
            kv.kvtrim_score_select(ctx, dc, torch.from_numpy(now_np).to(DEV), torch.from_numpy(budget).to(DEV), score, keep,
                                   kept, thr, evict_hint=4)
            assert kv.kvtrim_poll_error(ctx) == 0
            live = live_mask(hc)
            assert np.array_equal(score[:hc.cap].cpu().numpy()[live].view(np.uint32), s_ref[live].view(np.uint32))
            assert np.array_equal(keep[:hc.cap].cpu().numpy()[live], keep_ref[live])
            assert np.array_equal(kept.cpu().numpy(), kept_ref)
            assert np.array_equal(thr.cpu().numpy().view(np.uint32), thr_ref)


def test_bad_segment_table_is_reported():
    w = wl(1, 1, 2, 2, 64)
    c, now = ki.ragged_cache(w, [100, 100], reserve=1, salt=1)
    c["seg_len"][0] = 150                                         # runs into the next segment
    dc = kv.Cache.from_dict(c, DEV)
    ctx = kv.Context(1, 1, 2, 4, 64, dc.cap)
    score = torch.zeros(dc.cap, dtype=torch.float32, device=DEV)
    keep = torch.zeros(dc.cap, dtype=torch.uint8, device=DEV)
    kept = torch.zeros(2, dtype=torch.int32, device=DEV)
    bud = torch.tensor([50], dtype=torch.int64, device=DEV)
    for hint in (0, 2):
        kv.kvtrim_score_select(ctx, dc, now.to(DEV), bud, score, keep, kept, None, evict_hint=hint)
        assert kv.kvtrim_poll_error(ctx) == -6
