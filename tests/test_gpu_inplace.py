"""Stages 3 + 4 inside the cache (kvtrim_compact_attn_inplace) against the oracle's four stages: same scores, mask,
counts and threshold, the same entries in every segment afterwards (the segment starts stay where they were), the
same attention."""
import numpy as np
import pytest
import torch

import kvtrim_inputs as ki
import paper_2605_09649_amd as kv
from harness import run_steps_inplace_both

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
ATTN_TOL = 5e-3


def check(res):
    for i, r in enumerate(res):
        assert r["status"] == 0 and r["score_equal"] and r["keep_equal"] and r["cache_equal"], (i, r)
        assert r["attn_err"] <= ATTN_TOL and r["lse_err"] <= 2e-3 and r["lse_inf_equal"], (i, r)


def wl(S, L, H, G, D):
    return ki.Workload("t", 0, S, L, H, G * H, D, (0,) * S, (0,) * S, 1, 3.0, 1.5)


@pytest.mark.parametrize("G,D", [(1, 64), (2, 128), (4, 128), (4, 64), (6, 128), (7, 128), (8, 64), (8, 128)])
def test_decode_steps_in_place(G, D):
    # segments of many chunks, ragged tails, an empty segment and one of exactly three chunks; a budget that evicts a
    # few entries per step (most chunks lose nothing, some only shift), then one that evicts half
    w = wl(2, 2, 3, G, D)
    rng = np.random.default_rng(G * 10 + D)
    seg_len = rng.integers(1, 1500, w.nseg)
    seg_len[4] = 0
    seg_len[7] = 3 * 128
    per_seq = [int(seg_len[:6].sum()), int(seg_len[6:].sum())]
    c, now = ki.ragged_cache(w, seg_len, reserve=6, salt=G)
    check(run_steps_inplace_both(w, 5, [per_seq[0] - 7, per_seq[1] - 2], 6, c, now.numpy(), device=DEV))
    c, now = ki.ragged_cache(w, seg_len, reserve=3, salt=G + 1)
    check(run_steps_inplace_both(w, 3, [per_seq[0] // 2, per_seq[1] // 3], 3, c, now.numpy(), device=DEV))


@pytest.mark.parametrize("horizon", [2, 0])
def test_in_place_with_a_lookahead_horizon(horizon):
    w = wl(1, 2, 2, 4, 128)
    seg_len = [700, 130, 128, 1]
    c, now = ki.ragged_cache(w, seg_len, reserve=4, salt=3)
    check(run_steps_inplace_both(w, 4, [sum(seg_len) - 9], 4, c, now.numpy(), device=DEV, horizon=horizon))


@pytest.mark.parametrize("G,D", [(4, 128), (3, 64), (8, 128)])
def test_stage_three_alone_in_place(G, D):
    # kvtrim_compact_inplace followed by the stand-alone attention on the same cache
    w = wl(2, 2, 3, G, D)
    rng = np.random.default_rng(G + D)
    seg_len = rng.integers(1, 1500, w.nseg)
    seg_len[1] = 0
    seg_len[9] = 2 * 128
    per_seq = [int(seg_len[:6].sum()), int(seg_len[6:].sum())]
    c, now = ki.ragged_cache(w, seg_len, reserve=5, salt=G)
    check(run_steps_inplace_both(w, 5, [per_seq[0] - 5, per_seq[1] // 2], 5, c, now.numpy(), device=DEV, two_call=True,
                                 rebalance_at=(3,)))
    c, now = ki.ragged_cache(w, seg_len, reserve=2, salt=G + 1)
    check(run_steps_inplace_both(w, 2, [10 ** 6, 0], 2, c, now.numpy(), device=DEV, two_call=True))


def test_in_place_edge_budgets():
    # budget 0 empties every segment, a budget above the count moves nothing, ties everywhere (quantised log beta)
    w = wl(2, 1, 2, 2, 64)
    seg_len = [300, 257, 5, 640]
    c, now = ki.ragged_cache(w, seg_len, reserve=3, salt=8)
    g = torch.Generator().manual_seed(4)
    c["log_beta"] = -(torch.randint(0, 2, c["log_beta"].shape, generator=g).to(torch.float32)) * 0.25
    check(run_steps_inplace_both(w, 3, [10 ** 6, 0], 3, c, now.numpy(), device=DEV))
    c2, now2 = ki.ragged_cache(w, seg_len, reserve=3, salt=9)
    c2["log_beta"] = c["log_beta"].clone()
    check(run_steps_inplace_both(w, 3, [333, 400], 3, c2, now2.numpy(), device=DEV))


def test_in_place_steps_with_out_of_place_steps_between():
    # the free slots behind the segments are evened out by an out-of-place step now and then
    w = wl(2, 2, 2, 4, 128)
    rng = np.random.default_rng(12)
    seg_len = rng.integers(100, 900, w.nseg)
    per_seq = [int(seg_len[:4].sum()), int(seg_len[4:].sum())]
    c, now = ki.ragged_cache(w, seg_len, reserve=3, salt=5)
    res = run_steps_inplace_both(w, 9, [per_seq[0] - 11, per_seq[1] - 30], 3, c, now.numpy(), device=DEV, rebalance_at=(2, 5, 8))
    assert [r["in_place"] for r in res] == [True, True, False] * 3
    check(res)


def test_in_place_many_segments():
    # more than 1024 segments: the segment prefixes come from the one-block pass
    w = wl(5, 16, 16, 2, 64)
    rng = np.random.default_rng(3)
    seg_len = rng.integers(0, 300, w.nseg)
    per = w.n_layers * w.n_kv_heads
    per_seq = [int(seg_len[s * per:(s + 1) * per].sum()) for s in range(5)]
    c, now = ki.ragged_cache(w, seg_len, reserve=2, salt=6)
    check(run_steps_inplace_both(w, 2, [n - 300 for n in per_seq], 2, c, now.numpy(), device=DEV))


def test_in_place_argument_checks():
    w = wl(1, 1, 1, 1, 64)
    cap = 256
    ctx = kv.Context(1, 1, 1, 1, 64, cap)
    a, b = kv.Cache.empty(1, 64, cap, DEV), kv.Cache.empty(1, 64, cap, DEV)
    small = kv.Cache.empty(1, 64, 128, DEV)
    keep, kept = torch.zeros(cap, dtype=torch.uint8, device=DEV), torch.zeros(1, dtype=torch.int32, device=DEV)
    q = torch.zeros(1, 1, 1, 64, dtype=torch.bfloat16, device=DEV)
    out = torch.zeros(1, 1, 1, 64, dtype=torch.float32, device=DEV)
    with pytest.raises(kv.KvtrimError):                           # the cache as its own parking space
        kv.kvtrim_compact_attn_inplace(ctx, a, keep, kept, a, q, 0, 1, 0.125, out)
    with pytest.raises(kv.KvtrimError):                           # parking space smaller than the cache
        kv.kvtrim_compact_attn_inplace(ctx, a, keep, kept, small, q, 0, 1, 0.125, out)
    with pytest.raises(kv.KvtrimError):                           # empty layer range
        kv.kvtrim_compact_attn_inplace(ctx, a, keep, kept, b, q, 1, 1, 0.125, out)
    kv.kvtrim_compact_attn_inplace(ctx, a, keep, kept, b, q, 0, 1, 0.125, out)   # an empty cache is fine
    assert kv.kvtrim_poll_error(ctx) == 0


@pytest.mark.parametrize("G", [4, 7])
def test_in_place_layer_range(G):
    # a layer range attends only its layers (the other rows of `out` stay as they were) while every segment is
    # compacted; the attended rows and the cache equal those of a full-range call on a copy of the cache
    w = wl(1, 3, 2, G, 128)
    seg_len = [400, 130, 700, 5, 256, 300]
    c, now = ki.ragged_cache(w, seg_len, reserve=2, salt=11)
    cap = c["cap"]
    ctx = kv.Context(1, 3, 2, 2 * G, 128, cap)
    a, b = kv.Cache.from_dict(c, DEV), kv.Cache.from_dict({k: (v.clone() if torch.is_tensor(v) else v) for k, v in c.items()}, DEV)
    spare = kv.Cache.empty(w.nseg, 128, cap, DEV)
    inp = {k: v.to(DEV) for k, v in ki.decode_inputs(w, 0).items()}
    now_dev = (now + 1).to(DEV)
    pos = torch.full((w.nseg,), int(now[0]) + 1, dtype=torch.int32, device=DEV)
    score, keep = torch.zeros(cap, dtype=torch.float32, device=DEV), torch.zeros(cap, dtype=torch.uint8, device=DEV)
    kept, budget = torch.zeros(w.nseg, dtype=torch.int32, device=DEV), torch.tensor([sum(seg_len) - 40], dtype=torch.int64, device=DEV)
    outs = []
    for cache, rng in ((a, (0, 3)), (b, (1, 2))):
        kv.kvtrim_append(ctx, cache, inp["k_new"], inp["v_new"], inp["log_beta_new"], pos, 1)
        kv.kvtrim_score(ctx, cache, now_dev, score)
        kv.kvtrim_select_global(ctx, cache, score, budget, keep, kept)
        out = torch.full((1, 3, 2 * G, 128), 7.0, dtype=torch.float32, device=DEV)
        kv.kvtrim_compact_attn_inplace(ctx, cache, keep, kept, spare, inp["q"], rng[0], rng[1], 0.0884, out)
        assert kv.kvtrim_poll_error(ctx) == 0
        outs.append(out.cpu())
    assert torch.equal(outs[1][:, 1], outs[0][:, 1])
    assert bool((outs[1][:, 0] == 7.0).all()) and bool((outs[1][:, 2] == 7.0).all())
    from harness import compare_cache_contents, device_cache_to_host
    assert compare_cache_contents(device_cache_to_host(w, b), device_cache_to_host(w, a))


def test_min_room_follows_the_segments():
    # free slots behind the tightest segment: after an out-of-place step with a reserve, after appends, after an
    # in-place step that evicts from every segment
    w = wl(1, 2, 2, 2, 64)
    seg_len = [300, 10, 129, 77]
    c, now = ki.ragged_cache(w, seg_len, reserve=5, salt=4)
    cap = c["cap"]
    ctx = kv.Context(1, 2, 2, 4, 64, cap)
    cache, spare = kv.Cache.from_dict(c, DEV), kv.Cache.empty(w.nseg, 64, cap, DEV)
    room = torch.zeros(1, dtype=torch.int32, device=DEV)
    kv.kvtrim_min_room(ctx, cache, room)
    assert int(room.item()) == 5
    inp = {k: v.to(DEV) for k, v in ki.decode_inputs(w, 0).items()}
    pos = torch.full((w.nseg,), int(now[0]) + 1, dtype=torch.int32, device=DEV)
    kv.kvtrim_append(ctx, cache, inp["k_new"], inp["v_new"], inp["log_beta_new"], pos, 1)
    kv.kvtrim_min_room(ctx, cache, room)
    assert int(room.item()) == 4
    score, keep = torch.zeros(cap, dtype=torch.float32, device=DEV), torch.zeros(cap, dtype=torch.uint8, device=DEV)
    kept = torch.zeros(w.nseg, dtype=torch.int32, device=DEV)
    kv.kvtrim_score(ctx, cache, (now + 1).to(DEV), score)
    kv.kvtrim_select_global(ctx, cache, score, torch.tensor([0], dtype=torch.int64, device=DEV), keep, kept)
    kv.kvtrim_compact_inplace(ctx, cache, keep, kept, spare)          # budget 0: every segment is emptied where it stands
    kv.kvtrim_min_room(ctx, cache, room)
    assert kv.kvtrim_poll_error(ctx) == 0
    assert int(room.item()) == min(seg_len) + 5 and int(cache.seg_len.sum().item()) == 0
