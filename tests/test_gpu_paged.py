"""GPU parity of the paged layout (Sec. 4.2, implementation details: pages, block tables, per-head
variable lengths, eviction without moving K/V) against the CPU oracle's ragged loop.

Scores, the keep mask, the survivors of every segment and the threshold are compared bit for bit
(entries matched through their positions); attention within 5e-3; and the page bookkeeping must
be consistent after every call.
"""
import numpy as np
import pytest
import torch

import kvtrim_inputs as ki
import paper_2605_09649_amd as kv
from paged_harness import P, PagedHost, run_paged_both

pytestmark = pytest.mark.gpu
ATTN_TOL = 5e-3
DEV = "cuda:0"


def check(results):
    for r in results:
        assert r["status"] == 0 and r.get("status_select", 0) == 0, r
        assert r["structure"] == [] and r.get("structure_pre", []) == [], r
        assert r["score_equal"], (r["step"], "score bits differ")
        assert r["keep_equal"] and r["kept_equal"], (r["step"], "selection differs")
        assert r["cache_equal"], (r["step"], "surviving entries differ")
        assert r["attn_err"] <= ATTN_TOL, r
        assert r["lse_err"] <= 2e-3 and r["lse_inf_equal"], r


def wl(S, L, H, G, D):
    return ki.Workload("t", 0, S, L, H, G * H, D, (0,) * S, (0,) * S, 1, 3.0, 1.5)


def test_tiny_workload_paged_loop():
    w = ki.workload("tiny")                       # L4 H4 G2 D64, 2048 prefilled, B = 1024
    check(run_paged_both(w, [w.budget] * 12, device=DEV))


@pytest.mark.parametrize("name,prefill,steps", [("llama", 700, 4), ("long", 900, 4), ("vlm", 640, 4),
                                                ("multiturn", 600, 3)])
def test_scaled_down_workloads_paged(name, prefill, steps):
    w = ki.workload(name, prefill=prefill)
    check(run_paged_both(w, [w.budget] * steps, device=DEV))


@pytest.mark.parametrize("S,L,H,G,D", [(1, 2, 2, 1, 128), (2, 2, 1, 7, 128), (1, 1, 3, 8, 64), (3, 1, 2, 3, 64),
                                       (1, 2, 2, 5, 128), (1, 1, 2, 6, 128)])
def test_ragged_segments_with_empty_ones_paged(S, L, H, G, D):
    w = wl(S, L, H, G, D)
    rng = np.random.default_rng(S * 1000 + G * 10 + D)
    seg_len = rng.integers(0, 3000, w.nseg)
    seg_len[rng.integers(0, w.nseg)] = 0
    seg_len[rng.integers(0, w.nseg)] = 5 * P                      # ends exactly on a page boundary
    c, now = ki.ragged_cache(w, seg_len, reserve=1, salt=G)
    per_seq = [int(seg_len[s * L * H:(s + 1) * L * H].sum()) for s in range(S)]
    budget = [max(1, n // 3) for n in per_seq]
    check(run_paged_both(w, [budget] * 4, device=DEV, cache_dict=c, now0=now.numpy()))


@pytest.mark.parametrize("blocks", [1, 3, 10, 100000])
def test_paged_attention_for_any_size_of_the_fixed_grid(blocks, monkeypatch):
    # as in the ragged path: whatever the number of blocks of the attention kernel, the merge finds their partial results
    monkeypatch.setenv("KVTRIM_ATT_BLOCKS", str(blocks))
    w = wl(1, 2, 3, 2, 64)
    seg_len = [2900, 130, 0, 1024, 255, 3000]
    c, now = ki.ragged_cache(w, seg_len, reserve=1, salt=12)
    total = sum(seg_len)
    check(run_paged_both(w, [[total - 100], [total - 300], [total - 301]], device=DEV, cache_dict=c, now0=now.numpy()))
    check(run_paged_both(w, [[total - 100], [total - 300], [total - 301]], device=DEV, cache_dict=c, now0=now.numpy(), hint=60,
                         one_call=True))


def test_pages_are_freed_and_taken_again():
    # the budget shrinks (pages empty out and return to the free list), then grows past the cache
    # size (nothing is evicted, every full segment takes a page from the free list)
    w = wl(1, 2, 3, 2, 64)
    seg_len = [700, 130, 0, 1024, 255, 256]
    c, now = ki.ragged_cache(w, seg_len, reserve=1, salt=11)
    total = sum(seg_len)
    budgets = [[total], [total // 2], [total // 8], [40], [10 ** 6], [10 ** 6], [10 ** 6], [50], [10 ** 6]]
    budgets += [[10 ** 6]] * 130 + [[3], [0], [10 ** 6], [10 ** 6]]
    res = run_paged_both(w, budgets, device=DEV, cache_dict=c, now0=now.numpy(), n_pages=40)
    check(res)
    pages = [r["pages_in_use"] for r in res]
    assert min(pages[:9]) < pages[0] and pages[-3] == 0 and pages[-1] == w.nseg
    assert max(pages) > pages[8]                                   # pages were taken from the free list again


@pytest.mark.parametrize("horizon", [2, 0])
def test_lookahead_horizon_paged(horizon):
    w = ki.workload("tiny", prefill=700)
    check(run_paged_both(w, [w.budget] * 4, device=DEV, horizon=horizon))


def test_ties_at_the_threshold_are_ranked_by_layer_head_position():
    # beta = 1 (log beta = 0) for most entries: their scores are all 0, the maximum, and the budget
    # cuts through them, so the tie rule decides - whole segments first, in one segment by position.
    # After the first eviction the slots of a segment are no longer in position order.
    w = wl(2, 2, 2, 2, 64)
    seg_len = [600, 300, 257, 900, 128, 0, 640, 1000]
    c, now = ki.ragged_cache(w, seg_len, reserve=1, salt=5)
    g = torch.Generator().manual_seed(1)
    lb = c["log_beta"]
    lb[torch.rand(lb.shape, generator=g) < 0.8] = 0.0

    def plant(step, inp):
        if step % 2 == 0:
            inp["log_beta_new"][:] = 0.0

    budgets = [[1500, 1200], [900, 1100], [901, 600], [450, 601], [451, 100], [100, 99], [7, 98]]
    res = run_paged_both(w, budgets, device=DEV, cache_dict=c, now0=now.numpy(), tweak_new=plant)
    check(res)
    assert sum(r["ties_overflow"] for r in res[1:]) >= 5


def test_budget_zero_and_above_full_per_sequence():
    w = wl(3, 1, 2, 2, 128)
    seg_len = [300, 200, 500, 1, 129, 640]
    c, now = ki.ragged_cache(w, seg_len, reserve=1, salt=2)
    budgets = [[400, 10 ** 6, 600], [0, 10 ** 6, 300], [5, 0, 10 ** 6], [10 ** 6, 10 ** 6, 0]]
    check(run_paged_both(w, budgets, device=DEV, cache_dict=c, now0=now.numpy()))


def _small_setup(n_pages, max_pps, seg_len=(300, 200)):
    w = wl(1, 1, 2, 2, 64)
    c, now = ki.ragged_cache(w, list(seg_len), reserve=1, salt=9)
    src = kv.Cache.from_dict(c, DEV)
    ctx = kv.Context(w.n_seq, w.n_layers, w.n_kv_heads, w.n_q_heads, w.head_dim, max(src.cap, n_pages * P))
    pc = kv.PagedCache(w.nseg, w.head_dim, n_pages, max_pps, DEV)
    keep = torch.ones(src.cap, dtype=torch.uint8, device=DEV)
    kept = torch.tensor(list(seg_len), dtype=torch.int32, device=DEV)
    return w, ctx, src, pc, keep, kept


def test_device_side_errors_of_the_paged_calls():
    # not enough pages for the build
    w, ctx, src, pc, keep, kept = _small_setup(n_pages=4, max_pps=8)
    kv.kvtrim_paged_build(ctx, src, keep, kept, pc)
    assert kv.kvtrim_poll_error(ctx) == -4
    # a segment needs more pages than its block table holds
    w, ctx, src, pc, keep, kept = _small_setup(n_pages=8, max_pps=2)
    kv.kvtrim_paged_build(ctx, src, keep, kept, pc)
    assert kv.kvtrim_poll_error(ctx) == -4
    # kept that disagrees with the mask
    w, ctx, src, pc, keep, kept = _small_setup(n_pages=8, max_pps=8)
    kept[0] = 299
    kv.kvtrim_paged_build(ctx, src, keep, kept, pc)
    assert kv.kvtrim_poll_error(ctx) == -5
    # append with every page full and none free: the cache stays as it was
    w, ctx, src, pc, keep, kept = _small_setup(n_pages=3, max_pps=8, seg_len=(256, 128))
    kv.kvtrim_paged_build(ctx, src, keep, kept, pc)
    assert kv.kvtrim_poll_error(ctx) == 0
    before = PagedHost(pc)
    assert before.structure_problems() == [] and before.n_free == 0
    inp = {k: v.to(DEV) for k, v in ki.decode_inputs(w, 0).items()}
    pos_new = torch.full((w.nseg,), 5000, dtype=torch.int32, device=DEV)
    kv.kvtrim_paged_append(ctx, pc, inp["k_new"], inp["v_new"], inp["log_beta_new"], pos_new)
    assert kv.kvtrim_poll_error(ctx) == -4
    after = PagedHost(pc)
    assert after.structure_problems() == [] and np.array_equal(after.pos, before.pos)
    # a block table that is full
    w, ctx, src, pc, keep, kept = _small_setup(n_pages=6, max_pps=2, seg_len=(256, 100))
    kv.kvtrim_paged_build(ctx, src, keep, kept, pc)
    assert kv.kvtrim_poll_error(ctx) == 0
    kv.kvtrim_paged_append(ctx, pc, inp["k_new"], inp["v_new"], inp["log_beta_new"], pos_new)
    assert kv.kvtrim_poll_error(ctx) == -4
    after = PagedHost(pc)
    assert after.structure_problems() == []
    assert list(after.seg_live) == [256, 101]                     # the other segment took its token


def test_host_side_argument_checks_of_the_paged_calls():
    w, ctx, src, pc, keep, kept = _small_setup(n_pages=8, max_pps=8)
    score = torch.zeros(pc.slots, dtype=torch.float32, device=DEV)
    now = torch.zeros(1, dtype=torch.int32, device=DEV)
    with pytest.raises(kv.KvtrimError):
        kv.kvtrim_paged_score(ctx, pc, None, score)
    with pytest.raises(kv.KvtrimError):
        kv.kvtrim_paged_build(ctx, src, None, kept, pc)
    big = kv.PagedCache(w.nseg, w.head_dim, 64, 8, DEV)           # more slots than the context was made for
    with pytest.raises(kv.KvtrimError):
        kv.kvtrim_paged_score(ctx, big, now, score)
    tail = kv.PagedCache(w.nseg, w.head_dim, 8, 8, DEV, with_tail=True)
    with pytest.raises(kv.KvtrimError):
        kv.kvtrim_paged_build(ctx, src, keep, kept, tail)         # horizon constant on one side only
    q = torch.zeros(1, 1, 4, 64, dtype=torch.bfloat16, device=DEV)
    out = torch.zeros(1, 1, 4, 64, dtype=torch.float32, device=DEV)
    with pytest.raises(kv.KvtrimError):
        kv.kvtrim_paged_attn(ctx, pc, q, 0, 2, 0.125, out)        # layer range beyond the model
    assert kv.kvtrim_poll_error(ctx) == 0


def test_paged_append_skips_segments_whose_position_is_negative():
    # one sequence of the batch brings a token, the other does not (its rows are padding)
    w = wl(2, 1, 2, 2, 64)
    seg_len = (300, 200, 128, 77)
    c, now = ki.ragged_cache(w, list(seg_len), reserve=1, salt=4)
    src = kv.Cache.from_dict(c, DEV)
    ctx = kv.Context(w.n_seq, w.n_layers, w.n_kv_heads, w.n_q_heads, w.head_dim, max(src.cap, 16 * P))
    pc = kv.PagedCache(w.nseg, w.head_dim, 16, 8, DEV)
    keep = torch.ones(src.cap, dtype=torch.uint8, device=DEV)
    kept = torch.tensor(list(seg_len), dtype=torch.int32, device=DEV)
    kv.kvtrim_paged_build(ctx, src, keep, kept, pc)
    inp = {k: v.to(DEV) for k, v in ki.decode_inputs(w, 0).items()}
    pos_new = torch.tensor([-1, -1, 9000, 9000], dtype=torch.int32, device=DEV)
    kv.kvtrim_paged_append(ctx, pc, inp["k_new"], inp["v_new"], inp["log_beta_new"], pos_new)
    assert kv.kvtrim_poll_error(ctx) == 0
    ph = PagedHost(pc)
    assert ph.structure_problems() == []
    assert list(ph.seg_live) == [300, 200, 129, 78]
    assert list(ph.seg_pages) == [3, 2, 2, 1]                      # the full page of segment 2 made it take a new one
    idx, counts = ph.ordered_slots()
    assert ph.pos[idx[300 + 200 + 128]] == 9000 and ph.pos[idx[-1]] == 9000


def check_flow(results):
    for r in results:
        assert r["status"] == 0 and r["status_select"] == 0, r
        assert r["structure"] == [] and r["structure_pre"] == [], r
        assert r["score_equal"] and r["keep_equal"] and r["kept_equal"] and r["cache_equal"], r
        if "attn_err" in r:
            assert r["attn_err"] <= ATTN_TOL and r["lse_err"] <= 2e-3 and r["lse_inf_equal"], r


def test_multi_turn_chunked_prefill_into_pages():
    # pages start empty; chunks of 200 tokens (more than a page) fill holes first, then take new pages; sequences of
    # different lengths (ragged last chunks), per-sequence budgets, four turns with decode steps in between
    from paged_harness import run_multiturn_paged
    w = wl(3, 2, 2, 2, 64)
    res = run_multiturn_paged(w, [1500, 380, 811], chunk=200, decode_per_turn=3, budget=[300, 10 ** 6, 170], device=DEV)
    assert len(res) >= 20
    check_flow(res)
    pages = [r["pages_in_use"] for r in res]
    assert max(pages) > pages[-1] or max(pages) > min(pages[5:])     # pages were given back along the way


def test_multi_turn_chunked_sixteen_sequences_into_pages():
    from paged_harness import run_multiturn_paged
    w = ki.workload("multiturn", prefill=1024)                   # S16 L32 Hkv8 Hq32 D128, lengths in [64, 1024]
    check_flow(run_multiturn_paged(w, list(w.prefill), chunk=256, decode_per_turn=2, budget=[96 * 32 * 8] * 16, device=DEV,
                                   turns=2))


def test_chunk_append_without_pages_leaves_the_segment_unchanged():
    w, ctx, src, pc, keep, kept = _small_setup(n_pages=5, max_pps=8, seg_len=(250, 100))
    kv.kvtrim_paged_build(ctx, src, keep, kept, pc)
    assert kv.kvtrim_poll_error(ctx) == 0
    before = PagedHost(pc)
    assert before.n_free == 2
    inp = {k: v.to(DEV) for k, v in ki.chunk_inputs(w, 300, "cpu", 1).items()}
    pos = torch.arange(5000, 5300, dtype=torch.int32).repeat(w.nseg, 1)
    pos[1, 40:] = -1                                             # segment 1 brings 40 tokens, segment 0 all 300
    kv.kvtrim_paged_append(ctx, pc, inp["k_new"], inp["v_new"], inp["log_beta_new"], pos.to(DEV), n_new=300)
    assert kv.kvtrim_poll_error(ctx) == -4                       # segment 0 needs 3 more pages, 2 are free
    after = PagedHost(pc)
    assert after.structure_problems() == []
    assert list(after.seg_live) == [250, 140] and after.n_free == 1   # segment 1 filled its hole and took one page
    with pytest.raises(kv.KvtrimError):
        kv.kvtrim_paged_append(ctx, pc, inp["k_new"], inp["v_new"], inp["log_beta_new"], pos.to(DEV), n_new=5000)


def check_defrag(results, steps_with_defrag, must_free=True):
    for r in results:
        if r["step"] in steps_with_defrag:
            d = r["defrag"]
            assert d["tight"] and d["live_unchanged"], d
            assert d["free_gain"] == d["pages_before"] - d["pages_after"] >= 0, d
            if must_free:
                assert d["pages_after"] < d["pages_before"], d


def test_defragmentation_packs_every_segment_into_the_fewest_pages():
    # the budget drops to a third after the pages were built with everything kept: holes all over the pages; the
    # defragmented pool holds ceil(live / 128) pages per segment, the entries of every segment are the oracle's
    # (the checks of every step run after the call), and the loop goes on from the packed pages
    w = ki.workload("tiny", prefill=1500)
    full = [1500 * w.n_layers * w.n_kv_heads + 64]
    third = [full[0] // 3]
    results = run_paged_both(w, [full, third, third, third, [third[0] // 2], [third[0] // 2]], device=DEV,
                             defrag_at=(1, 2, 4))
    check(results)
    check_defrag(results, (1, 4))
    assert results[2]["defrag"]["pages_before"] - results[2]["defrag"]["pages_after"] <= w.nseg   # little to do one step later


def test_defragmentation_in_several_passes_with_empty_and_tight_segments():
    # segments of up to 9000 entries shrink to a quarter: more than 1024 entries move in one segment (two passes
    # of the move list); one segment is empty, one ends exactly on a page boundary; lookahead tail constants travel too
    w = wl(1, 2, 2, 2, 128)
    seg_len = np.array([9000, 0, 5 * P, 4100])
    c, now = ki.ragged_cache(w, seg_len, reserve=1, salt=11)
    n = int(seg_len.sum())
    results = run_paged_both(w, [[n + 8], [n // 4], [n // 4], [8], [0]], device=DEV, cache_dict=c, now0=now.numpy(), horizon=2,
                             defrag_at=(1, 3, 4))
    check(results)
    check_defrag(results, (1,), must_free=True)
    check_defrag(results, (3, 4), must_free=False)                # a handful of entries, then none: nothing to pack
    assert results[1]["defrag"]["pages_before"] - results[1]["defrag"]["pages_after"] > 2 * 1024 // P


def test_defragmentation_of_a_tight_pool_changes_nothing():
    w = ki.workload("tiny")
    results = run_paged_both(w, [w.budget] * 3, device=DEV, defrag_at=(0,))
    check(results)
    d = results[0]["defrag"]                                      # right after the build every segment is packed
    assert d["tight"] and d["pages_before"] == d["pages_after"] and d["free_gain"] == 0
