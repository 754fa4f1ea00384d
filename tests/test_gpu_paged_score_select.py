"""GPU parity of kvtrim_paged_score_select (stages 1 + 2 on the paged layout in one call) against the oracle's
ragged loop, in both of its forms - the two existing calls' kernels (evict_hint 0) and the decode-step form
(candidate list + ranking through the block tables, with its single-block fallback) - through whole paged decode
loops: scores, mask, per-segment counts and threshold key bit for bit, page bookkeeping consistent, attention
within tolerance."""
import numpy as np
import pytest
import torch

import kvtrim_inputs as ki
from paged_harness import P, run_paged_both
from test_gpu_paged import check, wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("hint", [0, 16])
def test_tiny_workload_paged_loop(hint):
    w = ki.workload("tiny")                                       # 16 segments: 16 evictions per step once at the budget
    res = run_paged_both(w, [w.budget] * 14, device=DEV, hint=hint)
    check(res)
    listed, fallback = res[-1]["path_counts"]
    if hint:
        # step 0 builds the pages through the ragged radix passes, which leave the bound the first paged step starts
        # from: every paged step must find its candidates listed
        assert fallback == 0 and listed == 13, (listed, fallback)
    else:
        assert listed == 0 and fallback == 0


@pytest.mark.parametrize("name,prefill,steps", [("llama", 700, 5), ("long", 900, 5), ("vlm", 640, 5), ("multiturn", 600, 4)])
def test_scaled_down_workloads_paged_decode_step_form(name, prefill, steps):
    w = ki.workload(name, prefill=prefill)
    res = run_paged_both(w, [w.budget] * steps, device=DEV, hint=w.n_layers * w.n_kv_heads)
    check(res)
    listed, fallback = res[-1]["path_counts"]
    # (a sequence still below its budget evicts nothing and counts as neither)
    assert 0 < listed + fallback <= (steps - 1) * w.n_seq and fallback <= w.n_seq, (listed, fallback)


@pytest.mark.parametrize("hint", [0, 4, 60])
@pytest.mark.parametrize("S,L,H,G,D", [(1, 2, 2, 1, 128), (2, 2, 1, 7, 128), (3, 1, 2, 3, 64), (1, 1, 2, 6, 128)])
def test_ragged_segments_with_empty_ones_paged(S, L, H, G, D, hint):
    w = wl(S, L, H, G, D)
    rng = np.random.default_rng(S * 1000 + G * 10 + D)
    seg_len = rng.integers(0, 20000, w.nseg)                      # more than one 8192-slot share per segment
    seg_len[rng.integers(0, w.nseg)] = 0
    seg_len[rng.integers(0, w.nseg)] = 5 * P                      # ends exactly on a page boundary
    c, now = ki.ragged_cache(w, seg_len, reserve=1, salt=G)
    per_seq = [int(seg_len[s * L * H:(s + 1) * L * H].sum()) for s in range(S)]
    budget = [max(1, n // 3) for n in per_seq]
    check(run_paged_both(w, [budget] * 5, device=DEV, cache_dict=c, now0=now.numpy(), hint=hint))


@pytest.mark.parametrize("hint", [3, 500])
def test_pages_are_freed_and_taken_again(hint):
    # the budget shrinks (many evictions: the list cannot hold them, the single-block select runs; pages empty out
    # and holes appear in the others), then grows past the cache size (nothing is evicted)
    w = wl(1, 2, 3, 2, 64)
    seg_len = [700, 130, 0, 1024, 255, 256]
    c, now = ki.ragged_cache(w, seg_len, reserve=1, salt=11)
    total = sum(seg_len)
    budgets = [[total], [total // 2], [total // 8], [40], [10 ** 6], [10 ** 6], [10 ** 6], [50], [10 ** 6]]
    budgets += [[10 ** 6]] * 20 + [[60]] * 6 + [[3], [0], [10 ** 6], [10 ** 6]]
    res = run_paged_both(w, budgets, device=DEV, cache_dict=c, now0=now.numpy(), n_pages=40, hint=hint)
    check(res)
    listed, fallback = res[-1]["path_counts"]
    assert fallback >= 2 and listed >= 4, (listed, fallback)


@pytest.mark.parametrize("horizon", [2, 0])
def test_lookahead_horizon_paged(horizon):
    w = ki.workload("tiny", prefill=700)
    check(run_paged_both(w, [w.budget] * 5, device=DEV, horizon=horizon, hint=16))


@pytest.mark.parametrize("hint", [0, 2, 400])
def test_ties_at_the_threshold_are_ranked_by_layer_head_position(hint):
    # beta = 1 (log beta = 0) for most entries: their scores are all 0, the maximum, and the budget cuts through them,
    # so the tie rule decides - whole segments first, in one segment by position.  After the first eviction the slots
    # of a segment are no longer in position order: the position bound has to come from a selection over the ties.
    w = wl(2, 2, 2, 2, 64)
    seg_len = [600, 300, 257, 900, 128, 0, 640, 1000]
    c, now = ki.ragged_cache(w, seg_len, reserve=1, salt=5)
    g = torch.Generator().manual_seed(1)
    lb = c["log_beta"]
    lb[torch.rand(lb.shape, generator=g) < 0.8] = 0.0

    def plant(step, inp):
        if step % 2 == 0:
            inp["log_beta_new"][:] = 0.0

    budgets = [[1500, 1200], [900, 1100], [901, 600], [450, 601], [451, 100], [100, 99], [7, 98], [7, 98], [6, 97]]
    res = run_paged_both(w, budgets, device=DEV, cache_dict=c, now0=now.numpy(), tweak_new=plant, hint=hint)
    check(res)
    assert sum(r["ties_overflow"] for r in res[1:]) >= 5


@pytest.mark.parametrize("levels", [1, 2, 5])
def test_quantised_retention_gives_ties_at_the_threshold_every_step(levels):
    # few distinct log beta values: whole groups of entries share a score and the threshold falls inside a group in
    # every step - with the steady trickle of a decode loop, so the candidate list carries the steps and its direct
    # ranking meets the ties (one level: pure recency, every segment ties with every other)
    w = wl(2, 2, 3, 2, 64)
    rng = np.random.default_rng(40 + levels)
    seg_len = rng.integers(100, 1500, w.nseg)
    c, now = ki.ragged_cache(w, seg_len, reserve=1, salt=levels, pos_stride_max=1)
    g = torch.Generator().manual_seed(levels)
    c["log_beta"] = -(torch.randint(0, levels, c["log_beta"].shape, generator=g).to(torch.float32) + 1.0) * 0.125
    budget = [int(seg_len[:6].sum()) // 2, int(seg_len[6:].sum()) - 7]
    for hint in (6, 200):
        clone = {k: (v.clone() if torch.is_tensor(v) else v) for k, v in c.items()}
        check(run_paged_both(w, [budget] * 6, device=DEV, cache_dict=clone, now0=now.numpy(), hint=hint))


def test_budget_zero_and_above_full_per_sequence():
    w = wl(3, 1, 2, 2, 128)
    seg_len = [300, 200, 500, 1, 129, 640]
    c, now = ki.ragged_cache(w, seg_len, reserve=1, salt=2)
    budgets = [[400, 10 ** 6, 600], [0, 10 ** 6, 300], [5, 0, 10 ** 6], [10 ** 6, 10 ** 6, 0], [10 ** 6, 3, 2]]
    check(run_paged_both(w, budgets, device=DEV, cache_dict=c, now0=now.numpy(), hint=4))


def test_bad_page_tables_are_reported():
    import paper_2605_09649_amd as kv
    from test_gpu_paged import _small_setup
    w, ctx, src, pc, keep, kept = _small_setup(n_pages=16, max_pps=8)
    kv.kvtrim_paged_build(ctx, src, keep, kept, pc)
    assert kv.kvtrim_poll_error(ctx) == 0
    pc.seg_pages[0] = 9                                           # more pages than the block table has columns
    slots = 16 * P
    score = torch.zeros(slots, dtype=torch.float32, device=DEV)
    mask = torch.zeros(slots, dtype=torch.uint8, device=DEV)
    now = torch.tensor([400], dtype=torch.int32, device=DEV)
    budget = torch.tensor([100], dtype=torch.int64, device=DEV)
    for hint in (0, 2):
        kv.kvtrim_paged_score_select(ctx, pc, now, budget, score, mask, kept, None, evict_hint=hint)
        assert kv.kvtrim_poll_error(ctx) == -6, hint


# ---------------------------------------------------------------------------------- the paged step in one call

@pytest.mark.parametrize("hint", [0, 16])
def test_one_call_tiny_workload_paged_loop(hint):
    w = ki.workload("tiny")
    res = run_paged_both(w, [w.budget] * 14, device=DEV, hint=hint, one_call=True)
    check(res)
    listed, fallback = res[-1]["path_counts"]
    assert (listed, fallback) == ((13, 0) if hint else (0, 0))


@pytest.mark.parametrize("name,prefill,steps", [("llama", 700, 5), ("long", 900, 5), ("vlm", 640, 5), ("multiturn", 600, 4)])
def test_one_call_scaled_down_workloads_paged(name, prefill, steps):
    w = ki.workload(name, prefill=prefill)
    check(run_paged_both(w, [w.budget] * steps, device=DEV, hint=w.n_layers * w.n_kv_heads, one_call=True))


@pytest.mark.parametrize("hint", [4, 60])
@pytest.mark.parametrize("S,L,H,G,D", [(1, 2, 2, 1, 128), (2, 2, 1, 7, 128), (3, 1, 2, 3, 64)])
def test_one_call_ragged_segments_with_empty_ones_paged(S, L, H, G, D, hint):
    w = wl(S, L, H, G, D)
    rng = np.random.default_rng(S * 1000 + G * 10 + D)
    seg_len = rng.integers(0, 20000, w.nseg)
    seg_len[rng.integers(0, w.nseg)] = 0
    seg_len[rng.integers(0, w.nseg)] = 5 * P
    c, now = ki.ragged_cache(w, seg_len, reserve=1, salt=G)
    per_seq = [int(seg_len[s * L * H:(s + 1) * L * H].sum()) for s in range(S)]
    budget = [max(1, n // 3) for n in per_seq]
    check(run_paged_both(w, [budget] * 5, device=DEV, cache_dict=c, now0=now.numpy(), hint=hint, one_call=True))


def test_one_call_pages_are_freed_and_taken_again():
    # whole pages empty out under the eviction that rides in the mask kernel, leave the block tables and are taken again
    w = wl(1, 2, 3, 2, 64)
    seg_len = [700, 130, 0, 1024, 255, 256]
    c, now = ki.ragged_cache(w, seg_len, reserve=1, salt=11)
    total = sum(seg_len)
    budgets = [[total], [total - 6], [total - 12], [total - 18]] + [[total - 18 - 40 * i] for i in range(1, 40)]
    budgets += [[10 ** 6]] * 10 + [[400]] * 6 + [[3], [0], [10 ** 6], [10 ** 6]]
    res = run_paged_both(w, budgets, device=DEV, cache_dict=c, now0=now.numpy(), n_pages=40, hint=60, one_call=True)
    check(res)
    pages = [r["pages_in_use"] for r in res]
    listed, fallback = res[-1]["path_counts"]
    # (pages empty out - entirely at the budget of zero - and every segment takes one again afterwards)
    assert min(pages) == 0 and pages[-1] == w.nseg and max(pages[:44]) > min(pages[44:60]) and listed >= 30, (pages, listed, fallback)


@pytest.mark.parametrize("layer_range", [(1, 2), (0, 2), (2, 3)])
def test_one_call_layer_range_paged(layer_range):
    # the step's scoring kernel builds the attention's chunk table for the layers asked for only: their rows of `out`
    # equal the oracle's, the other rows stay as they were, and every segment is scored, evicted and tidied all the same
    w = wl(2, 3, 2, 4, 128)
    seg_len = [400, 130, 700, 5, 256, 300, 0, 128, 129, 640, 50, 900]
    c, now = ki.ragged_cache(w, seg_len, reserve=1, salt=8)
    budget = [sum(seg_len[:6]) - 30, sum(seg_len[6:]) - 200]
    res = run_paged_both(w, [budget] * 5, device=DEV, cache_dict=c, now0=now.numpy(), hint=12, one_call=True,
                         layer_range=layer_range)
    check(res)
    assert all(r["untouched_outside_range"] for r in res[1:]), res


@pytest.mark.parametrize("horizon", [2, 0])
def test_one_call_lookahead_horizon_paged(horizon):
    w = ki.workload("tiny", prefill=700)
    check(run_paged_both(w, [w.budget] * 5, device=DEV, horizon=horizon, hint=16, one_call=True))


def test_one_call_ties_at_the_threshold():
    w = wl(2, 2, 2, 2, 64)
    seg_len = [600, 300, 257, 900, 128, 0, 640, 1000]
    c, now = ki.ragged_cache(w, seg_len, reserve=1, salt=5)
    g = torch.Generator().manual_seed(1)
    lb = c["log_beta"]
    lb[torch.rand(lb.shape, generator=g) < 0.8] = 0.0

    def plant(step, inp):
        if step % 2 == 0:
            inp["log_beta_new"][:] = 0.0

    budgets = [[1500, 1200], [1490, 1190], [1480, 1180], [901, 600], [890, 590], [451, 100], [445, 99], [7, 98], [7, 98]]
    res = run_paged_both(w, budgets, device=DEV, cache_dict=c, now0=now.numpy(), tweak_new=plant, hint=12, one_call=True)
    check(res)
    assert sum(r["ties_overflow"] for r in res[1:]) >= 5


def test_one_call_budget_zero_and_above_full_per_sequence():
    w = wl(3, 1, 2, 2, 128)
    seg_len = [300, 200, 500, 1, 129, 640]
    c, now = ki.ragged_cache(w, seg_len, reserve=1, salt=2)
    budgets = [[400, 10 ** 6, 600], [0, 10 ** 6, 300], [5, 0, 10 ** 6], [10 ** 6, 10 ** 6, 0], [10 ** 6, 3, 2]]
    check(run_paged_both(w, budgets, device=DEV, cache_dict=c, now0=now.numpy(), hint=4, one_call=True))
