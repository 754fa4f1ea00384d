"""Seeded sweep over random configurations: shapes, ragged and empty segments (small ones, and segments of up to
40,000 entries beside tiny ones), budgets from 0 to above the entry count, quantised log beta (exact score ties
everywhere) - the ragged loop (two-call and fused) and the paged loop against the oracle, every stage compared as
in the other parity tests."""
import numpy as np
import pytest
import torch

import kvtrim_inputs as ki
from harness import run_steps_both, run_steps_inplace_both
from paged_harness import run_paged_both

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
ATTN_TOL = 5e-3


def random_case(seed, reserve=1, long_segments=False):
    """long_segments: segments of up to 40,000 entries (several blocks of the scoring kernel and many chunks of the
    row mover and the attention per segment) beside empty and tiny ones; budgets mostly a few hundred under the count."""
    rng = np.random.default_rng((5000 if long_segments else 1000) + seed)
    S = int(rng.integers(1, 4))
    L = int(rng.integers(1, 4))
    H = int(rng.integers(1, 4))
    G = int(rng.integers(1, 9))
    D = int(rng.choice([64, 128]))
    w = ki.Workload("r", 0, S, L, H, G * H, D, (0,) * S, (0,) * S, 1, 3.0, 1.5)
    hi = int(rng.choice([4000, 9000, 20000, 40000] if long_segments else [5, 150, 700, 2600]))
    seg_len = rng.integers(0, hi + 1, w.nseg)
    seg_len[rng.random(w.nseg) < 0.2] = 0
    if long_segments:
        seg_len[rng.random(w.nseg) < 0.2] = rng.integers(1, 130)
    c, now = ki.ragged_cache(w, seg_len, reserve=reserve, salt=seed, pos_stride_max=int(rng.integers(1, 5)))
    if rng.random() < 0.5:                                         # few distinct retention values: ties at the threshold
        g = torch.Generator().manual_seed(seed)
        levels = int(rng.choice([1, 2, 7]))
        q = torch.randint(0, levels, c["log_beta"].shape, generator=g)
        c["log_beta"] = -(q.to(torch.float32)) * 0.25
    per_seq = [int(seg_len[s * L * H:(s + 1) * L * H].sum()) for s in range(S)]
    steps = int(rng.integers(2, 5))
    budgets = []
    for _ in range(steps):
        b = []
        for n in per_seq:
            kind = rng.random()
            if long_segments and 0.2 <= kind < 0.6:
                b.append(max(1, n - int(rng.integers(0, 400))))
            else:
                b.append(0 if kind < 0.1 else (10 ** 7 if kind < 0.2 else int(rng.integers(1, max(2, n + 10)))))
        budgets.append(b)
    return w, c, now, budgets


@pytest.mark.parametrize("seed", range(48))
def test_random_configuration(seed):
    check_case(seed, False)


@pytest.mark.parametrize("seed", range(24))
def test_random_configuration_with_long_segments(seed):
    check_case(seed, True)


def check_case(seed, long_segments):
    w, c, now, budgets = random_case(seed, long_segments=long_segments)
    clone = lambda: {k: (v.clone() if torch.is_tensor(v) else v) for k, v in c.items()}
    for fused in (False, True):
        # the ragged harness takes one budget for all steps: the first of the list
        res = run_steps_both(w, steps=len(budgets), budget=budgets[0], device=DEV, cache_dict=clone(), now0=now.numpy(),
                             fused=fused)
        for i, r in enumerate(res):
            assert r["status"] == 0 and r["score_equal"] and r["keep_equal"] and r["cache_equal"], (seed, fused, i, r)
            assert r["attn_err"] <= ATTN_TOL and r["lse_err"] <= 2e-3 and r["lse_inf_equal"], (seed, fused, i, r)
    # the same configuration compacted inside the cache (fused for even seeds, stage 3 alone + attention for odd ones),
    # with an out-of-place step in between where there are at least three steps
    w2, c2, now2, budgets2 = random_case(seed, reserve=len(budgets) + 1, long_segments=long_segments)
    res = run_steps_inplace_both(w2, len(budgets2), budgets2[0], len(budgets2) + 1, c2, now2.numpy(), device=DEV,
                                 two_call=bool(seed % 2), rebalance_at=(1,) if len(budgets2) > 2 else (),
                                 rebalance_room=lambda step: len(budgets2) - step - 1)   # budgets above the count evict nothing
    for i, r in enumerate(res):
        assert r["status"] == 0 and r["score_equal"] and r["keep_equal"] and r["cache_equal"], (seed, "in place", i, r)
        assert r["attn_err"] <= ATTN_TOL and r["lse_err"] <= 2e-3 and r["lse_inf_equal"], (seed, "in place", i, r)
    # every other seed also packs the pages after each eviction from the second step on
    defrag_at = tuple(range(1, len(budgets))) if seed % 2 else ()
    res = run_paged_both(w, budgets, device=DEV, cache_dict=clone(), now0=now.numpy(), defrag_at=defrag_at)
    for r in res:
        if "defrag" in r:
            assert r["defrag"]["tight"] and r["defrag"]["live_unchanged"], (seed, r)
        assert r["status"] == 0 and r.get("status_select", 0) == 0, (seed, r)
        assert r["structure"] == [] and r.get("structure_pre", []) == [], (seed, r)
        assert r["score_equal"] and r["keep_equal"] and r["kept_equal"] and r["cache_equal"], (seed, r)
        assert r["attn_err"] <= ATTN_TOL and r["lse_err"] <= 2e-3 and r["lse_inf_equal"], (seed, r)


@pytest.mark.parametrize("S,L,H", [(600, 1, 2), (1100, 1, 1)])
def test_many_short_sequences(S, L, H):
    """Hundreds of sequences of a few dozen entries: a histogram block then holds several whole sequences, a
    sequence's last block is found per sequence, and ties at the threshold (quantised log beta) have to be ranked
    in many sequences of the same call."""
    rng = np.random.default_rng(77 + S)
    w = ki.Workload("m", 0, S, L, H, 2 * H, 64, (0,) * S, (0,) * S, 1, 3.0, 1.5)
    seg_len = rng.integers(0, 41, w.nseg)
    seg_len[rng.random(w.nseg) < 0.1] = 0
    c, now = ki.ragged_cache(w, seg_len, reserve=1, salt=S, pos_stride_max=2)
    g = torch.Generator().manual_seed(S)
    c["log_beta"] = -(torch.randint(0, 3, c["log_beta"].shape, generator=g).to(torch.float32)) * 0.25
    per_seq = [int(seg_len[s * L * H:(s + 1) * L * H].sum()) for s in range(S)]
    budgets = [[0 if rng.random() < 0.05 else int(rng.integers(1, max(2, n + 3))) for n in per_seq] for _ in range(2)]
    clone = lambda: {k: (v.clone() if torch.is_tensor(v) else v) for k, v in c.items()}
    res = run_steps_both(w, steps=2, budget=budgets[0], device=DEV, cache_dict=clone(), now0=now.numpy(), fused=True)
    for i, r in enumerate(res):
        assert r["status"] == 0 and r["score_equal"] and r["keep_equal"] and r["cache_equal"], (S, i, r)
        assert r["attn_err"] <= ATTN_TOL and r["lse_err"] <= 2e-3 and r["lse_inf_equal"], (S, i, r)
    res = run_paged_both(w, budgets, device=DEV, cache_dict=clone(), now0=now.numpy())
    for r in res:
        assert r["status"] == 0 and r.get("status_select", 0) == 0, (S, r)
        assert r["structure"] == [] and r.get("structure_pre", []) == [], (S, r)
        assert r["score_equal"] and r["keep_equal"] and r["kept_equal"] and r["cache_equal"], (S, r)
        assert r["attn_err"] <= ATTN_TOL and r["lse_err"] <= 2e-3 and r["lse_inf_equal"], (S, r)
