"""Pins of the oracle's score and selection (CPU only).

Everything here checks the oracle against something other than itself: direct
summation of the geometric series the score is defined by (Sec. 4.2,
Eq. global_score), numpy's own fp32 multiply, Python's tuple sort as a brute
force of the eviction rule, and closed forms / invariants of the rule
(Sec. 2.1, Eq. reform and Eq. problem; Sec. 4.2).
"""
import math
import struct
from fractions import Fraction

import numpy as np
import pytest
import torch

import kvtrim_inputs as ki
import oracle
from helpers import host_cache, live_mask, shape_of


def small_cache(seg_len, n_seq=1, n_layers=2, n_kv_heads=2, reserve=1, salt=0):
    w = ki.Workload("t", 0, n_seq, n_layers, n_kv_heads, 2 * n_kv_heads, 64, (0,) * n_seq, (0,) * n_seq, 1, 3.0, 1.5)
    c, now = ki.ragged_cache(w, seg_len, reserve=reserve, salt=salt)
    return w, host_cache(w, c), now.numpy()


# ----------------------------------------------------------------------------- score

def test_score_is_log_of_direct_geometric_sum_at_horizon_one():
    # Eq. global_score with T = t+1: the sum has the single term beta^(t+1-i).
    w, hc, now = small_cache([5, 0, 17, 3])
    s = oracle.score(hc, now)
    for e in hc.entry_index():
        beta = math.exp(float(hc.log_beta[e]))
        t, i = int(now[0]), int(hc.pos[e])
        direct = sum(beta ** (sidx - i) for sidx in range(t + 1, t + 2))
        assert math.isclose(math.exp(float(s[e])), direct, rel_tol=2e-6), (e, s[e], direct)


@pytest.mark.parametrize("H", [1, 2, 5, 40])
def test_horizon_score_matches_direct_sum_and_printed_closed_form(H):
    w, hc, now = small_cache([9, 4, 0, 30], salt=H)
    s = oracle.score_horizon(hc, now, H)
    for e in hc.entry_index():
        beta = math.exp(float(hc.log_beta[e]))
        t, i = int(now[0]), int(hc.pos[e])
        T = t + H
        direct = math.fsum(beta ** (sidx - i) for sidx in range(t + 1, T + 1))
        closed = beta ** (t + 1 - i) * (1 - beta ** (T - t)) / (1 - beta)
        assert math.isclose(math.exp(s[e]), direct, rel_tol=1e-11)
        assert math.isclose(math.exp(s[e]), closed, rel_tol=1e-9)


def test_infinite_horizon_is_limit_of_long_horizons():
    w, hc, now = small_cache([12, 7, 1, 2], salt=3)
    s_inf = oracle.score_horizon(hc, now, 0)
    for e in hc.entry_index():
        beta = math.exp(float(hc.log_beta[e]))
        i, t = int(hc.pos[e]), int(now[0])
        assert math.isclose(math.exp(s_inf[e]), beta ** (t + 1 - i) / (1 - beta), rel_tol=1e-9)


def test_horizon_one_fp64_agrees_with_fp32_hot_path_score():
    w, hc, now = small_cache([40, 40, 40, 40], salt=4)
    s32 = oracle.score(hc, now)
    s64 = oracle.score_horizon(hc, now, 1)
    idx = hc.entry_index()
    np.testing.assert_allclose(s32[idx], s64[idx], rtol=1e-6)


def test_score_is_one_fp32_multiply_and_newest_token_has_elapsed_one():
    w, hc, now = small_cache([33, 8, 1, 64], salt=5)
    s = oracle.score(hc, now)
    idx = hc.entry_index()
    elapsed = (now[0] + 1 - hc.pos[idx]).astype(np.float32)
    expect = elapsed * hc.log_beta[idx]            # numpy's own binary32 multiply
    assert expect.dtype == np.float32
    np.testing.assert_array_equal(s[idx].view(np.uint32), expect.view(np.uint32))
    # a token appended now (pos == now) has elapsed 1: its score is log(beta) itself
    hc.pos[idx[-1]] = now[0]
    s2 = oracle.score(hc, now)
    assert s2[idx[-1]] == hc.log_beta[idx[-1]]


def nearest_f32(x):
    """Correct rounding of an exact rational to binary32 (no double rounding)."""
    c = np.float32(float(x))
    cands = [c, np.nextafter(c, np.float32(np.inf)), np.nextafter(c, np.float32(-np.inf))]
    return min(cands, key=lambda v: abs(Fraction(float(v)) - x))


@pytest.mark.parametrize("H", [2, 5, 0])
def test_cached_horizon_tail_gives_the_log_of_the_series_with_one_fused_multiply_add(H):
    w, hc, now = small_cache([25, 3, 0, 40], salt=20 + H)
    import torch
    hc.log_tail = ki.log_tail_of(torch.from_numpy(hc.log_beta), H).numpy()
    s = oracle.score(hc, now)
    s64 = oracle.score_horizon(hc, now, H)
    for e in hc.entry_index():
        beta = math.exp(float(hc.log_beta[e]))
        t, i = int(now[0]), int(hc.pos[e])
        if H > 0:
            direct = math.fsum(beta ** (sidx - i) for sidx in range(t + 1, t + H + 1))
        else:
            direct = beta ** (t + 1 - i) / (1 - beta)
        assert math.isclose(math.exp(float(s[e])), direct, rel_tol=3e-6)
        assert math.isclose(float(s[e]), s64[e], rel_tol=2e-6, abs_tol=1e-6)
        # exactly one rounding: the exact value of elapsed * log_beta + log_tail, rounded once to binary32
        exact = Fraction(t + 1 - i) * Fraction(float(hc.log_beta[e])) + Fraction(float(hc.log_tail[e]))
        assert s[e] == nearest_f32(exact), e


def test_a_long_horizon_prefers_the_slowly_decaying_old_token():
    # two entries: A fresh with beta 0.9, B ten steps old with beta 0.985.  One-step score: A 0.9 > B 0.8597;
    # infinite horizon: A 0.9/0.1 = 9 < B 0.8597/0.015 = 57.3 (Sec. 4.2: longer horizons favour larger beta).
    w = ki.Workload("t", 0, 1, 1, 2, 2, 64, (0,), (0,), 1, 3.0, 1.5)
    c, _ = ki.ragged_cache(w, [1, 1], reserve=0)
    hc = host_cache(w, c)
    hc.log_beta[:] = np.log(np.array([0.9, 0.985])).astype(np.float32)
    hc.pos[:] = [9, 0]
    now = np.array([9], np.int32)
    keep1, _, _ = oracle.select(hc, oracle.score(hc, now), np.array([1], np.int64))
    assert keep1[:2].tolist() == [1, 0]
    import torch
    hc.log_tail = ki.log_tail_of(torch.from_numpy(hc.log_beta), 0).numpy()
    keep_inf, _, _ = oracle.select(hc, oracle.score(hc, now), np.array([1], np.int64))
    assert keep_inf[:2].tolist() == [0, 1]


def test_score_decays_monotonically_for_beta_below_one():
    w, hc, now = small_cache([50, 50, 50, 50], salt=6)
    idx = hc.entry_index()
    prev = oracle.score(hc, now)[idx]
    for step in range(1, 6):
        cur = oracle.score(hc, now + step)[idx]
        assert np.all(cur < prev)            # log(beta) < 0 strictly for every generated entry
        prev = cur
    hc.log_beta[idx] = 0.0                   # beta = 1: no decay
    assert np.all(oracle.score(hc, now + 7)[idx] == 0.0)


def test_gaps_between_segments_are_not_written():
    w, hc, now = small_cache([3, 3, 3, 3], reserve=2)
    s = oracle.score(hc, now)
    assert np.all(s[~live_mask(hc)] == 0.0)


# ----------------------------------------------------------------------------- key order

def test_key_is_monotone_in_float_order_and_orders_signed_zero():
    vals = [-math.inf, -3.0e38, -1e5, -1.0000001, -1.0, -1e-30, -1e-45, -0.0, 0.0, 1e-45, 2.5, math.inf]
    keys = [oracle.key_of_score(v) for v in vals]
    assert keys == sorted(keys)
    assert len(set(keys)) == len(keys)                      # -0.0 and +0.0 differ, -0.0 lower
    rng = np.random.default_rng(0)
    x = rng.standard_normal(2000).astype(np.float32) * np.float32(1e3)
    k = np.array([oracle.key_of_score(v) for v in x], dtype=np.uint64)
    order = np.argsort(x, kind="stable")
    assert np.all(np.diff(k[order].astype(np.int64)) >= 0)


# ----------------------------------------------------------------------------- selection

def brute_force_keep(w, hc, score, budget):
    """Eviction rule by exhaustive sorting with Python tuples; float order by value, and
    the sign bit only to separate -0.0 from +0.0."""
    keep = np.zeros(hc.cap, np.uint8)
    per_seq = w.n_layers * w.n_kv_heads
    for seq in range(w.n_seq):
        cand = []
        for g in range(seq * per_seq, (seq + 1) * per_seq):
            layer, head = divmod(g - seq * per_seq, w.n_kv_heads)
            for j in range(hc.seg_len[g]):
                e = int(hc.seg_start[g] + j)
                sc = float(score[e])
                neg_zero = sc == 0.0 and struct.pack("<f", sc)[3] & 0x80
                cand.append((-sc, 1 if neg_zero else 0, layer, head, int(hc.pos[e]), e))
        cand.sort()
        for t in cand[:max(0, int(budget[seq]))]:
            keep[t[-1]] = 1
    return keep


@pytest.mark.parametrize("seed", range(6))
def test_select_equals_brute_force_sort_on_small_inputs(seed):
    rng = np.random.default_rng(seed)
    S, L, H = [(1, 2, 2), (2, 3, 2), (1, 4, 4), (3, 1, 2), (2, 2, 3), (1, 1, 1)][seed]
    seg_len = rng.integers(0, 40, S * L * H)
    seg_len[rng.integers(0, len(seg_len))] = 0
    w, hc, now = small_cache(seg_len, S, L, H, reserve=int(rng.integers(0, 3)), salt=seed)
    score = oracle.score(hc, now)
    idx = hc.entry_index()
    # plant ties, signed zeros and -inf
    if len(idx) > 10:
        pick = rng.choice(idx, size=len(idx) // 3, replace=False)
        score[pick] = rng.choice(np.array([-2.5, -0.0, 0.0, -np.inf, -1e-3], np.float32), size=len(pick))
    per_seq_n = [int(hc.seg_len[s * L * H:(s + 1) * L * H].sum()) for s in range(S)]
    for frac in (0.0, 0.3, 0.5, 1.0, 1.5):
        budget = np.array([int(frac * n) for n in per_seq_n], np.int64)
        keep, kept, thr = oracle.select(hc, score, budget)
        ref = brute_force_keep(w, hc, score, budget)
        np.testing.assert_array_equal(keep, ref)
        for g in range(w.nseg):
            s0, n = int(hc.seg_start[g]), int(hc.seg_len[g])
            assert kept[g] == keep[s0:s0 + n].sum()
        for s in range(S):
            assert kept[s * L * H:(s + 1) * L * H].sum() == min(budget[s], per_seq_n[s])


def test_select_all_equal_scores_keeps_first_in_layer_head_position_order():
    w, hc, now = small_cache([6, 6, 6, 6])
    score = np.full(hc.cap, -1.25, np.float32)
    keep, kept, thr = oracle.select(hc, score, np.array([15], np.int64))
    assert kept.tolist() == [6, 6, 3, 0]
    s2 = int(hc.seg_start[2])
    assert keep[s2:s2 + 6].tolist() == [1, 1, 1, 0, 0, 0]     # lowest positions first
    assert thr[0] == oracle.key_of_score(-1.25)


def test_negative_zero_ranks_below_positive_zero():
    w, hc, now = small_cache([2, 0, 0, 0])
    score = np.zeros(hc.cap, np.float32)
    s0 = int(hc.seg_start[0])
    score[s0] = -0.0
    score[s0 + 1] = 0.0
    keep, kept, thr = oracle.select(hc, score, np.array([1], np.int64))
    assert keep[s0:s0 + 2].tolist() == [0, 1]


def test_equal_beta_reduces_to_a_sliding_window_per_segment():
    # All beta equal: the score depends on elapsed steps only, so the kept set is the B most
    # recent entries; with equal-length segments holding the same positions that is a window of
    # floor(B/nseg) per segment, plus one more for the first B mod nseg segments.
    L, H, T = 3, 2, 50
    w = ki.Workload("t", 0, 1, L, H, 2 * H, 64, (T,), (0,), 1, 3.0, 1.5)
    c = ki.prefill_cache(w, reserve=1)
    c["log_beta"][:] = -0.125
    hc = host_cache(w, c)
    now = np.array([T - 1], np.int32)
    B = 6 * 7 + 4
    keep, kept, _ = oracle.select(hc, oracle.score(hc, now), np.array([B], np.int64))
    assert kept.tolist() == [8, 8, 8, 8, 7, 7]
    for g in range(6):
        s0 = int(hc.seg_start[g])
        expect = np.zeros(T, np.uint8)
        expect[T - kept[g]:] = 1
        np.testing.assert_array_equal(keep[s0:s0 + T], expect)


def test_budget_at_least_count_keeps_everything_and_zero_budget_nothing():
    w, hc, now = small_cache([11, 0, 5, 9])
    score = oracle.score(hc, now)
    live = live_mask(hc)
    keep, kept, thr = oracle.select(hc, score, np.array([25], np.int64))
    assert keep[live].all() and kept.tolist() == [11, 0, 5, 9]
    keep, kept, thr = oracle.select(hc, score, np.array([10 ** 12], np.int64))
    assert keep[live].all()
    keep, kept, thr = oracle.select(hc, score, np.array([0], np.int64))
    assert not keep.any() and kept.sum() == 0 and thr[0] == 0xFFFFFFFF


def test_kept_scores_dominate_evicted_scores_and_budgets_are_per_sequence():
    w, hc, now = small_cache(np.arange(12) * 3, n_seq=3, n_layers=2, n_kv_heads=2, salt=9)
    score = oracle.score(hc, now)
    budget = np.array([7, 0, 40], np.int64)
    keep, kept, thr = oracle.select(hc, score, budget)
    for s in range(3):
        segs = range(s * 4, (s + 1) * 4)
        idx = np.concatenate([np.arange(hc.seg_start[g], hc.seg_start[g] + hc.seg_len[g]) for g in segs])
        k, sc = keep[idx].astype(bool), score[idx]
        assert k.sum() == min(budget[s], len(idx))
        if k.any() and (~k).any():
            assert sc[k].min() >= sc[~k].max()
            assert thr[s] == oracle.key_of_score(sc[k].min())


def test_multi_step_loop_never_exceeds_budget_and_never_readmits():
    # Eq. reform: r_{t,i} >= r_{t+1,i}; Eq. problem: sum r <= M.  Run the whole loop on the oracle.
    w = ki.workload("tiny", prefill=96)
    B = 200
    c = ki.prefill_cache(w, reserve=1)
    hc = host_cache(w, c)
    now = np.array([w.prefill[0] - 1], np.int32)
    ever_evicted = set()
    for step in range(12):
        inp = ki.decode_inputs(w, step)
        now = now + 1
        from helpers import bf16_bits
        oracle.append(hc, bf16_bits(inp["k_new"]), bf16_bits(inp["v_new"]), inp["log_beta_new"].numpy(),
                      np.full(w.nseg, now[0], np.int32))
        score = oracle.score(hc, now)
        keep, kept, _ = oracle.select(hc, score, np.array([B], np.int64))
        before = {(g, int(hc.pos[hc.seg_start[g] + j])) for g in range(w.nseg) for j in range(hc.seg_len[g])}
        hc = oracle.compact(hc, keep, B + w.nseg, reserve=1)
        after = {(g, int(hc.pos[hc.seg_start[g] + j])) for g in range(w.nseg) for j in range(hc.seg_len[g])}
        assert len(after) == min(B, len(before)) and after <= before
        assert not (after & ever_evicted)
        ever_evicted |= before - after
