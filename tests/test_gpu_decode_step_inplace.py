"""GPU parity of kvtrim_decode_step_inplace (append + stages 1-4 in one call, stages 3 + 4 inside the cache: four
kernels for a decode step) against the oracle's five operations, through whole decode loops: in its list form (few
evictions), its mask form (ties at the threshold, budget drops: the single-block select), and the shapes and hints that
make it run the calls it stands for one after the other."""
import numpy as np
import pytest
import torch

import kvtrim_inputs as ki
import paper_2605_09649_amd as kv
from harness import run_steps_inplace_both

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
ATTN_TOL = 5e-3


def check(res, what=""):
    for i, r in enumerate(res):
        assert r["status"] == 0 and r["score_equal"] and r["keep_equal"] and r["cache_equal"], (what, i, r)
        assert r["attn_err"] <= ATTN_TOL and r["lse_err"] <= 2e-3 and r["lse_inf_equal"], (what, i, r)


def wl(S, L, H, G, D):
    return ki.Workload("t", 0, S, L, H, G * H, D, (0,) * S, (0,) * S, 1, 3.0, 1.5)


@pytest.mark.parametrize("G,D", [(1, 64), (2, 128), (4, 128), (4, 64), (6, 128), (7, 128), (8, 64), (8, 128)])
def test_decode_steps_in_place_in_one_call(G, D):
    # segments of many chunks, ragged tails, an empty segment and one of exactly three chunks; a budget that evicts a
    # few entries per step (most chunks lose nothing, some only shift; the evicted entries come as lists), then one
    # that evicts half in its first step (more than the hint: the single-block select, mask and table instead of lists)
    w = wl(2, 2, 3, G, D)
    rng = np.random.default_rng(G * 10 + D)
    seg_len = rng.integers(1, 1500, w.nseg)
    seg_len[4] = 0
    seg_len[7] = 3 * 128
    per_seq = [int(seg_len[:6].sum()), int(seg_len[6:].sum())]
    c, now = ki.ragged_cache(w, seg_len, reserve=6, salt=G)
    check(run_steps_inplace_both(w, 6, [per_seq[0] - 7, per_seq[1] - 2], 6, c, now.numpy(), device=DEV, one_call=True, hint=6))
    c, now = ki.ragged_cache(w, seg_len, reserve=3, salt=G + 1)
    check(run_steps_inplace_both(w, 3, [per_seq[0] // 2, per_seq[1] // 3], 3, c, now.numpy(), device=DEV, one_call=True, hint=6))


def test_path_counts_and_the_list_form():
    # steady decode steps: after the first step (no bound yet: the general select) every selection comes from the
    # candidate list, i.e. the four-kernel form ran
    w = ki.workload("tiny", prefill=900)
    pre = {k: (v.cpu() if torch.is_tensor(v) else v) for k, v in ki.prefill_cache(w, reserve=12, device=DEV).items()}
    n = sum(w.prefill) * w.n_layers * w.n_kv_heads // w.n_seq
    res = run_steps_inplace_both(w, 12, [n - 40] * w.n_seq, 12, pre, [t - 1 for t in w.prefill], device=DEV, one_call=True,
                                 hint=w.n_layers * w.n_kv_heads)
    check(res)


@pytest.mark.parametrize("horizon", [2, 0])
def test_lookahead_horizon(horizon):
    w = wl(1, 2, 2, 4, 128)
    seg_len = [700, 130, 128, 1]
    c, now = ki.ragged_cache(w, seg_len, reserve=5, salt=3)
    check(run_steps_inplace_both(w, 5, [sum(seg_len) - 9], 5, c, now.numpy(), device=DEV, horizon=horizon, one_call=True, hint=4))


def test_edge_budgets_and_ties():
    # budget 0 empties every segment, a budget above the count moves nothing, ties everywhere (quantised log beta)
    w = wl(2, 1, 2, 2, 64)
    seg_len = [300, 257, 5, 640]
    c, now = ki.ragged_cache(w, seg_len, reserve=3, salt=8)
    g = torch.Generator().manual_seed(4)
    c["log_beta"] = -(torch.randint(0, 2, c["log_beta"].shape, generator=g).to(torch.float32)) * 0.25
    check(run_steps_inplace_both(w, 3, [10 ** 6, 0], 3, c, now.numpy(), device=DEV, one_call=True, hint=2))
    c2, now2 = ki.ragged_cache(w, seg_len, reserve=3, salt=9)
    c2["log_beta"] = c["log_beta"].clone()
    check(run_steps_inplace_both(w, 3, [333, 400], 3, c2, now2.numpy(), device=DEV, one_call=True, hint=2))


def test_out_of_place_steps_between_and_hints():
    # the free slots behind the segments are evened out by an out-of-place step (kvtrim_decode_step) now and then; a
    # hint of 0 (the general select: the separate calls) and a large one give the same results
    w = wl(2, 2, 2, 4, 128)
    rng = np.random.default_rng(12)
    seg_len = rng.integers(100, 900, w.nseg)
    per_seq = [int(seg_len[:4].sum()), int(seg_len[4:].sum())]
    for hint in (0, 4, 500):
        c, now = ki.ragged_cache(w, seg_len, reserve=3, salt=5)
        res = run_steps_inplace_both(w, 9, [per_seq[0] - 11, per_seq[1] - 30], 3, c, now.numpy(), device=DEV, rebalance_at=(2, 5, 8),
                                     one_call=True, hint=hint)
        assert [r["in_place"] for r in res] == [True, True, False] * 3
        check(res, hint)


def test_many_evictions_in_a_segment_overflow_the_record():
    # more evictions in one segment than its record holds (12): the block reads the rest from the list
    w = wl(1, 1, 2, 2, 128)
    seg_len = [2000, 300]
    c, now = ki.ragged_cache(w, seg_len, reserve=8, salt=21)
    check(run_steps_inplace_both(w, 8, [sum(seg_len) - 60], 8, c, now.numpy(), device=DEV, one_call=True, hint=40))


def test_many_segments_and_sequences():
    w = wl(5, 16, 16, 2, 64)                                     # 1280 segments, 256 per sequence
    rng = np.random.default_rng(3)
    seg_len = rng.integers(0, 300, w.nseg)
    per = w.n_layers * w.n_kv_heads
    per_seq = [int(seg_len[s * per:(s + 1) * per].sum()) for s in range(5)]
    c, now = ki.ragged_cache(w, seg_len, reserve=3, salt=6)
    check(run_steps_inplace_both(w, 3, [n - 300 for n in per_seq], 3, c, now.numpy(), device=DEV, one_call=True, hint=per))


@pytest.mark.parametrize("G", [4, 8])
def test_layer_range(G):
    # a layer range attends only its layers (the other rows of `out` stay as they were) while every segment is
    # compacted; the attended rows, the mask, the counts and the cache equal those of a full-range call on a copy of
    # the cache, in the four-kernel form (second step: the bound is there) as in the separate calls (first step)
    from harness import compare_cache_contents, device_cache_to_host
    w = wl(1, 3, 2, G, 128)
    seg_len = [400, 130, 700, 5, 256, 300]
    c, now = ki.ragged_cache(w, seg_len, reserve=3, salt=11)
    cap = c["cap"]
    spare = kv.Cache.empty(w.nseg, 128, cap, DEV)
    budget = torch.tensor([sum(seg_len) - 40], dtype=torch.int64, device=DEV)
    res = []
    for rng in ((0, 3), (1, 2)):
        ctx = kv.Context(1, 3, 2, 2 * G, 128, cap)
        cache = kv.Cache.from_dict({k: (v.clone() if torch.is_tensor(v) else v) for k, v in c.items()}, DEV)
        score, keep = torch.zeros(cap, dtype=torch.float32, device=DEV), torch.zeros(cap, dtype=torch.uint8, device=DEV)
        kept = torch.zeros(w.nseg, dtype=torch.int32, device=DEV)
        outs = []
        for step in range(3):
            inp = {k: v.to(DEV) for k, v in ki.decode_inputs(w, step).items()}
            t = int(now[0]) + 1 + step
            out = torch.full((1, 3, 2 * G, 128), 7.0, dtype=torch.float32, device=DEV)
            kv.kvtrim_decode_step_inplace(ctx, cache, inp["k_new"], inp["v_new"], inp["log_beta_new"],
                                          torch.full((w.nseg,), t, dtype=torch.int32, device=DEV), 1,
                                          torch.tensor([t], dtype=torch.int32, device=DEV), budget, score, keep, kept, spare,
                                          inp["q"], rng[0], rng[1], 0.0884, out, evict_hint=w.nseg)
            assert kv.kvtrim_poll_error(ctx) == 0
            outs.append(out.cpu())
        assert kv.kvtrim_select_path_counts(ctx)[0] >= 1          # (the candidate list carried a step: the four kernels ran)
        res.append((outs, keep.cpu(), kept.cpu(), device_cache_to_host(w, cache)))
    (full, keep_a, kept_a, cache_a), (part, keep_b, kept_b, cache_b) = res
    for step in range(3):
        assert torch.equal(part[step][:, 1], full[step][:, 1])
        assert bool((part[step][:, 0] == 7.0).all()) and bool((part[step][:, 2] == 7.0).all())
    assert torch.equal(keep_a, keep_b) and torch.equal(kept_a, kept_b)
    assert compare_cache_contents(cache_b, cache_a)


def test_no_room_for_the_new_token_is_reported():
    w = wl(1, 1, 2, 2, 64)
    seg_len = [100, 50]
    c, now = ki.ragged_cache(w, seg_len, reserve=0, salt=2)       # no free slot behind the first segment
    cur = kv.Cache.from_dict(c, DEV)
    other = kv.Cache.empty(w.nseg, 64, cur.cap, DEV)
    ctx = kv.Context(1, 1, 2, 4, 64, cur.cap)
    inp = {k: v.to(DEV) for k, v in ki.decode_inputs(w, 0).items()}
    z = lambda *s, dt=torch.float32: torch.zeros(*s, dtype=dt, device=DEV)
    t = int(now[0]) + 1
    for hint in (0, 2):                                            # the separate calls and the four kernels
        kv.kvtrim_decode_step_inplace(ctx, cur, inp["k_new"], inp["v_new"], inp["log_beta_new"],
                                      torch.full((w.nseg, 1), t, dtype=torch.int32, device=DEV), 1,
                                      torch.tensor([t], dtype=torch.int32, device=DEV), torch.tensor([10 ** 6], device=DEV),
                                      z(cur.cap), z(cur.cap, dt=torch.uint8), z(w.nseg, dt=torch.int32), other, inp["q"], 0, 1, 0.125,
                                      z(1, 1, 4, 64), evict_hint=hint)
        assert kv.kvtrim_poll_error(ctx) == -4                     # KVTRIM_ECAP
        assert cur.seg_len.cpu().tolist() == seg_len               # nothing was appended


def test_argument_checks():
    cap = 256
    ctx = kv.Context(1, 1, 1, 1, 64, cap)
    a, b = kv.Cache.empty(1, 64, cap, DEV), kv.Cache.empty(1, 64, cap, DEV)
    small = kv.Cache.empty(1, 64, 128, DEV)
    z = lambda *s, dt=torch.float32: torch.zeros(*s, dtype=dt, device=DEV)
    new = (z(1, 1, 64, dt=torch.bfloat16), z(1, 1, 64, dt=torch.bfloat16), z(1, 1), z(1, 1, dt=torch.int32), 1,
           z(1, dt=torch.int32), torch.ones(1, dtype=torch.int64, device=DEV), z(cap), z(cap, dt=torch.uint8), z(1, dt=torch.int32))
    q, out = z(1, 1, 1, 64, dt=torch.bfloat16), z(1, 1, 1, 64)
    with pytest.raises(kv.KvtrimError):                           # the cache as its own parking space
        kv.kvtrim_decode_step_inplace(ctx, a, *new, a, q, 0, 1, 0.125, out)
    with pytest.raises(kv.KvtrimError):                           # parking space smaller than the cache
        kv.kvtrim_decode_step_inplace(ctx, a, *new, small, q, 0, 1, 0.125, out)
    with pytest.raises(kv.KvtrimError):                           # empty layer range
        kv.kvtrim_decode_step_inplace(ctx, a, *new, b, q, 1, 1, 0.125, out)
    with pytest.raises(kv.KvtrimError):                           # a tail for a cache that carries none
        kv.kvtrim_decode_step_inplace(ctx, a, *new, b, q, 0, 1, 0.125, out, log_tail_new=z(1, 1))
    kv.kvtrim_decode_step_inplace(ctx, a, *new, b, q, 0, 1, 0.125, out, evict_hint=1)
    assert kv.kvtrim_poll_error(ctx) == 0
    assert int(a.seg_len.cpu()[0]) == 1
