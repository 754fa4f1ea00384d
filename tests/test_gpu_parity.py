"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Selection and compaction must match bit for bit; attention within
max|o_gpu - o_ref| / max|o_ref| <= 5e-3 (bf16 inputs, fp32 accumulation).
"""
import math

import numpy as np
import pytest
import torch

import kvtrim_inputs as ki
import oracle
import paper_2605_09649_amd as kv
from harness import attn_error, compare_caches, device_cache_to_host, run_multiturn_both, run_steps_both
from helpers import bf16_bits, host_cache, live_mask

pytestmark = pytest.mark.gpu
ATTN_TOL = 5e-3
DEV = "cuda:0"


def check(results):
    for i, r in enumerate(results):
        assert r["status"] == 0, (i, r)
        assert r["score_equal"], (i, "score bits differ")
        assert r["keep_equal"], (i, "selection differs")
        assert r["cache_equal"], (i, "compacted cache differs")
        assert r["attn_err"] <= ATTN_TOL, (i, r["attn_err"])
        assert r["lse_err"] <= 2e-3 and r["lse_inf_equal"], (i, r)


def wl(S, L, H, G, D, name="t"):
    return ki.Workload(name, 0, S, L, H, G * H, D, (0,) * S, (0,) * S, 1, 3.0, 1.5)


# ---------------------------------------------------------------------------------- whole loop

@pytest.mark.parametrize("fused", [False, True])
def test_tiny_workload_full_loop(fused):
    w = ki.workload("tiny")                       # L4 H4 G2 D64, 2048 prefilled, B = 1024, 16 steps
    check(run_steps_both(w, steps=16, budget=w.budget, device=DEV, fused=fused))


@pytest.mark.parametrize("fused", [False, True])
@pytest.mark.parametrize("name,prefill,steps", [("llama", 700, 3), ("long", 900, 3), ("vlm", 640, 3),
                                                ("multiturn", 600, 2)])
def test_scaled_down_workloads(name, prefill, steps, fused):
    w = ki.workload(name, prefill=prefill)
    check(run_steps_both(w, steps=steps, budget=w.budget, device=DEV, fused=fused))


@pytest.mark.parametrize("fused", [False, True])
@pytest.mark.parametrize("S,L,H,G,D", [(1, 2, 2, 1, 128), (2, 2, 1, 7, 128), (1, 1, 3, 8, 64), (3, 1, 2, 3, 64),
                                       (1, 2, 2, 5, 128), (1, 1, 2, 6, 128), (1, 2, 1, 4, 128), (1, 1, 2, 2, 64)])
def test_ragged_segments_spanning_several_chunks(S, L, H, G, D, fused):
    w = wl(S, L, H, G, D)
    rng = np.random.default_rng(S * 1000 + G * 10 + D)
    seg_len = rng.integers(0, 6000, w.nseg)
    seg_len[rng.integers(0, w.nseg)] = 0          # an empty segment
    seg_len[rng.integers(0, w.nseg)] = 2048 * 2 + 1
    c, now = ki.ragged_cache(w, seg_len, reserve=1, salt=G)
    per_seq = [int(seg_len[s * L * H:(s + 1) * L * H].sum()) for s in range(S)]
    budget = [max(1, n // 3) for n in per_seq]
    check(run_steps_both(w, steps=2, budget=budget, device=DEV, cache_dict=c, now0=now.numpy(), fused=fused))


@pytest.mark.parametrize("fused", [False, True])
def test_multi_turn_chunked_prefill_then_decode(fused):
    # the multi-turn configuration scaled down: sequences of different lengths grow by prefill chunks (ragged last
    # chunks are padded with negative positions), the cache is rescored, selected and compacted after every chunk,
    # then a few tokens are decoded; four turns, per-sequence budgets
    w = wl(3, 2, 2, 2, 64)
    lengths = [700, 180, 411]
    res = run_multiturn_both(w, lengths, chunk=64, decode_per_turn=3, budget=[160, 10 ** 6, 96], device=DEV, fused=fused)
    assert len(res) > 20 and any("decode" in r["what"] for r in res)
    for r in res:
        assert r["status"] == 0 and r["score_equal"] and r["keep_equal"] and r["cache_equal"], r
        if "attn_err" in r:
            assert r["attn_err"] <= ATTN_TOL and r["lse_err"] <= 2e-3, r


@pytest.mark.parametrize("D", [64, 128])
def test_multi_turn_chunks_in_one_call(D):
    # the same flow with every chunk step done by kvtrim_append_compact (metadata appended, rows moved once, from
    # the caller's buffers to the compacted cache): scores, mask, counts, threshold and cache as the oracle's four stages
    w = wl(3, 2, 2, 2, D)
    res = run_multiturn_both(w, [700, 180, 411], chunk=64, decode_per_turn=2, budget=[160, 10 ** 6, 96], device=DEV,
                             one_call_chunks=True)
    assert sum("chunk" in r["what"] for r in res) > 10
    for r in res:
        assert r["status"] == 0 and r["score_equal"] and r["keep_equal"] and r["cache_equal"], r
        if "attn_err" in r:
            assert r["attn_err"] <= ATTN_TOL and r["lse_err"] <= 2e-3, r


def test_multi_turn_chunks_in_one_call_sixteen_sequences():
    w = ki.workload("multiturn", prefill=1024)                   # S16 L32 Hkv8 Hq32 D128, lengths in [64, 1024]
    res = run_multiturn_both(w, list(w.prefill), chunk=256, decode_per_turn=1, budget=[96 * 32 * 8] * 16, device=DEV,
                             turns=2, one_call_chunks=True)
    for r in res:
        assert r["status"] == 0 and r["score_equal"] and r["keep_equal"] and r["cache_equal"], r


@pytest.mark.parametrize("horizon", [1, 2, 0])
def test_append_compact_on_a_ragged_cache(horizon):
    # one call on a cache with gapped positions and an empty segment: sequence 0 brings a full chunk, sequence 1 a
    # ragged one (padding rows behind its 11 tokens); with a lookahead horizon the new tokens bring their tail constant
    w = wl(2, 2, 3, 2, 128)
    rng = np.random.default_rng(5 + horizon)
    seg_len = rng.integers(1, 300, w.nseg)
    seg_len[3] = 0
    n_new, per_seq = 37, w.n_layers * w.n_kv_heads
    c, now = ki.ragged_cache(w, seg_len, reserve=n_new, salt=9)
    c = ki.with_horizon(c, horizon)
    inp = ki.chunk_inputs(w, n_new, "cpu", 3)
    lt_new = None if horizon == 1 else ki.log_tail_of(inp["log_beta_new"], horizon)
    take = [n_new, 11]
    pos_new = np.full((w.nseg, n_new), -1, np.int32)
    for s in range(2):
        pos_new[s * per_seq:(s + 1) * per_seq, :take[s]] = int(now[s]) + np.arange(take[s])
    now_after = (now.numpy() + np.array(take) - 1).astype(np.int32)
    n_seq_entries = [int(seg_len[s * per_seq:(s + 1) * per_seq].sum()) + take[s] * per_seq for s in range(2)]
    budget = np.array([n_seq_entries[0] // 2, n_seq_entries[1] - 5], np.int64)
    cap = c["cap"]
    # ---- oracle: the four stages
    hc = host_cache(w, c)
    oracle.append(hc, bf16_bits(inp["k_new"]), bf16_bits(inp["v_new"]), inp["log_beta_new"].numpy(), pos_new,
                  log_tail_new=None if lt_new is None else lt_new.numpy())
    s_ref = oracle.score(hc, now_after)
    k_ref, kept_ref, thr_ref = oracle.select(hc, s_ref, budget)
    hc_next = oracle.compact(hc, k_ref, cap, 1)
    # ---- GPU: one call
    ctx = kv.Context(w.n_seq, w.n_layers, w.n_kv_heads, w.n_q_heads, w.head_dim, cap)
    src = kv.Cache.from_dict(c, DEV)
    dst = kv.Cache.empty(w.nseg, w.head_dim, cap, DEV, with_tail=horizon != 1)
    score = torch.zeros(cap, dtype=torch.float32, device=DEV)
    keep = torch.zeros(cap, dtype=torch.uint8, device=DEV)
    kept = torch.zeros(w.nseg, dtype=torch.int32, device=DEV)
    thr = torch.zeros(w.n_seq, dtype=torch.int32, device=DEV)
    kv.kvtrim_append_compact(ctx, src, inp["k_new"].to(DEV), inp["v_new"].to(DEV), inp["log_beta_new"].to(DEV),
                             torch.from_numpy(pos_new).to(DEV), n_new, torch.from_numpy(now_after).to(DEV),
                             torch.from_numpy(budget).to(DEV), score, keep, kept, dst, 1, thr_key_out=thr,
                             log_tail_new=None if lt_new is None else lt_new.to(DEV))
    assert kv.kvtrim_poll_error(ctx) == 0
    live = live_mask(hc)
    assert np.array_equal(score.cpu().numpy()[live].view(np.uint32), s_ref[live].view(np.uint32))
    assert np.array_equal(keep.cpu().numpy()[live], k_ref[live]) and np.array_equal(kept.cpu().numpy(), kept_ref)
    assert np.array_equal(thr.cpu().numpy().view(np.uint32), thr_ref)
    assert compare_caches(device_cache_to_host(w, dst), hc_next)
    assert int(kept_ref.sum()) == int(budget.sum())


def test_append_compact_argument_checks():
    w = wl(1, 1, 1, 1, 64)
    nseg, cap = 1, 64
    ctx = kv.Context(1, 1, 1, 1, 64, cap)
    a, b = kv.Cache.empty(nseg, 64, cap, DEV), kv.Cache.empty(nseg, 64, cap, DEV)
    t = lambda *shape, dt=torch.float32: torch.zeros(*shape, dtype=dt, device=DEV)
    k_new, lb, pos = t(1, 4, 64, dt=torch.bfloat16), t(1, 4), t(1, 4, dt=torch.int32)
    now, budget = t(1, dt=torch.int32), t(1, dt=torch.int64)
    score, keep, kept = t(cap), t(cap, dt=torch.uint8), t(nseg, dt=torch.int32)
    with pytest.raises(kv.KvtrimError):                           # source and destination share buffers
        kv.kvtrim_append_compact(ctx, a, k_new, k_new, lb, pos, 4, now, budget, score, keep, kept, a, 0)
    with pytest.raises(kv.KvtrimError):                           # no tokens
        kv.kvtrim_append_compact(ctx, a, k_new, k_new, lb, pos, 0, now, budget, score, keep, kept, b, 0)
    with pytest.raises(kv.KvtrimError):                           # a missing output
        kv.kvtrim_append_compact(ctx, a, k_new, k_new, lb, pos, 4, now, budget, None, keep, kept, b, 0)
    with pytest.raises(kv.KvtrimError):                           # the tail constant without a cache that carries it
        kv.kvtrim_append_compact(ctx, a, k_new, k_new, lb, pos, 4, now, budget, score, keep, kept, b, 0, log_tail_new=lb)
    assert kv.kvtrim_poll_error(ctx) == 0


def test_multi_turn_chunked_sixteen_sequences():
    w = ki.workload("multiturn", prefill=1024)                   # S16 L32 Hkv8 Hq32 D128, lengths in [64, 1024]
    per_head = 96
    res = run_multiturn_both(w, list(w.prefill), chunk=256, decode_per_turn=2, budget=[per_head * 32 * 8] * 16, device=DEV,
                             turns=2)
    for r in res:
        assert r["status"] == 0 and r["score_equal"] and r["keep_equal"] and r["cache_equal"], r
        if "attn_err" in r:
            assert r["attn_err"] <= ATTN_TOL and r["lse_err"] <= 2e-3, r


@pytest.mark.parametrize("fused", [False, True])
def test_one_giant_segment_and_many_empty_ones(fused):
    w = wl(1, 2, 4, 4, 128)
    seg_len = [0, 0, 0, 70001, 0, 0, 3, 0]
    c, now = ki.ragged_cache(w, seg_len, reserve=1, salt=3)
    check(run_steps_both(w, steps=2, budget=[20011], device=DEV, cache_dict=c, now0=now.numpy(), fused=fused))


@pytest.mark.parametrize("fused", [False, True])
@pytest.mark.parametrize("horizon", [2, 5, 0])
def test_lookahead_horizon_scores_through_the_whole_loop(horizon, fused):
    # Sec. 4.2: horizon T-t = 2 is the paper's inference default, 0 stands for the limit T-t -> infinity
    w = ki.workload("tiny", prefill=700)
    check(run_steps_both(w, steps=6, budget=w.budget, device=DEV, fused=fused, horizon=horizon))
    w = ki.workload("llama", prefill=600)
    check(run_steps_both(w, steps=2, budget=w.budget, device=DEV, fused=fused, horizon=horizon))


def test_horizon_tail_must_be_consistent_between_caches():
    w = wl(1, 1, 2, 2, 64)
    c, now = ki.ragged_cache(w, [10, 10], salt=1)
    ctx = kv.Context(1, 1, 2, 4, 64, 32)
    src = kv.Cache.from_dict(ki.with_horizon(c, 2), DEV)
    dst = kv.Cache.empty(2, 64, 32, DEV)                                  # no tail in the destination
    keep = torch.ones(32, dtype=torch.uint8, device=DEV)
    kept = torch.tensor([10, 10], dtype=torch.int32, device=DEV)
    with pytest.raises(kv.KvtrimError):
        kv.kvtrim_compact(ctx, src, keep, kept, dst, 1)
    new = ki.decode_inputs(w, 0)
    with pytest.raises(kv.KvtrimError):                                   # tail required for this cache
        kv.kvtrim_append(ctx, src, new["k_new"].to(DEV), new["v_new"].to(DEV), new["log_beta_new"].to(DEV),
                         torch.zeros(2, dtype=torch.int32, device=DEV), 1)


@pytest.mark.parametrize("G,D", [(4, 128), (8, 128), (6, 64)])
@pytest.mark.parametrize("roomy", [True, False])
def test_fused_call_with_a_layer_range_and_sparse_mask(roomy, G, D):
    # compaction + attention in one call on a mask that keeps about one entry in five, layers [1, 3) only.  With a
    # destination of at least a quarter of the source the fused kernel works a block per chunk of the source; with a
    # tight one the library expects few survivors and works a block per chunk of the destination - same results
    # either way.
    w = wl(2, 3, 2, G, D)
    rng = np.random.default_rng(21)
    seg_len = rng.integers(0, 2500, w.nseg)
    c, _ = ki.ragged_cache(w, seg_len, salt=21)
    hc = host_cache(w, c)
    keep_np = (rng.random(hc.cap) < 0.2).astype(np.uint8)
    kept_np = np.array([keep_np[s:s + n].sum() for s, n in zip(hc.seg_start, hc.seg_len)], np.int32)
    dst_cap = hc.cap // 2 if roomy else int(kept_np.sum()) + 2 * w.nseg
    assert (dst_cap >= hc.cap // 4) == roomy
    dst_ref = oracle.compact(hc, keep_np, dst_cap, 2)
    q = ki.decode_inputs(w, 3)["q"]
    scale = 1.0 / math.sqrt(D)
    ref, ref_lse = oracle.attend(dst_ref, bf16_bits(q), scale)
    ctx = kv.Context(w.n_seq, w.n_layers, w.n_kv_heads, w.n_q_heads, D, hc.cap)
    dst = kv.Cache.empty(w.nseg, D, dst_cap, DEV)
    out = torch.full(ref.shape, 99.0, dtype=torch.float32, device=DEV)
    lse = torch.full(ref_lse.shape, 99.0, dtype=torch.float32, device=DEV)
    kv.kvtrim_compact_attn(ctx, kv.Cache.from_dict(c, DEV), torch.from_numpy(keep_np).to(DEV),
                           torch.from_numpy(kept_np).to(DEV), dst, 2, q.to(DEV), 1, 3, scale, out, lse)
    assert kv.kvtrim_poll_error(ctx) == 0
    assert compare_caches(device_cache_to_host(w, dst), dst_ref)
    o = out.cpu().numpy()
    assert np.all(o[:, 0] == 99.0)
    assert attn_error(o[:, 1:3], ref[:, 1:3]) <= ATTN_TOL
    fin = np.isfinite(ref_lse[:, 1:3])
    assert np.abs(lse.cpu().numpy()[:, 1:3][fin] - ref_lse[:, 1:3][fin]).max() <= 2e-3


@pytest.mark.parametrize("D,horizon", [(128, 1), (64, 1), (128, 2)])
def test_sparse_selection_in_stage_three_alone_gathers_by_destination_chunk(D, horizon):
    # a destination under a quarter of the source: the row mover works a block per 128-row chunk of the DESTINATION
    # (the fused kernel's gathering instance with no layer to attend).  One entry in sixteen survives on average; some
    # source chunks keep nothing, some keep every entry, segments end in ragged chunks, one segment is empty.
    w = wl(2, 2, 3, 2, D)
    rng = np.random.default_rng(77 + D + horizon)
    seg_len = rng.integers(1, 6000, w.nseg)
    seg_len[3] = 0
    seg_len[5] = 128 * 9 + 1
    c, _ = ki.ragged_cache(w, seg_len, salt=33)
    c = ki.with_horizon(c, horizon)
    hc = host_cache(w, c)
    keep_np = (rng.random(hc.cap) < 1.0 / 16).astype(np.uint8)
    s5 = int(hc.seg_start[5])
    keep_np[s5 + 128:s5 + 3 * 128] = 1                            # two chunks that keep everything
    keep_np[s5 + 4 * 128:s5 + 6 * 128] = 0                        # two that keep nothing
    keep_np[s5 + 9 * 128] = 1                                     # the one-entry tail chunk
    kept_np = np.array([keep_np[s:s + n].sum() for s, n in zip(hc.seg_start, hc.seg_len)], np.int32)
    dst_cap = int(kept_np.sum()) + 3 * w.nseg
    assert dst_cap < hc.cap // 4
    dst_ref = oracle.compact(hc, keep_np, dst_cap, 3)
    ctx = kv.Context(w.n_seq, w.n_layers, w.n_kv_heads, w.n_q_heads, D, hc.cap)
    dst = kv.Cache.empty(w.nseg, D, dst_cap, DEV, with_tail=horizon != 1)
    kv.kvtrim_compact(ctx, kv.Cache.from_dict(c, DEV), torch.from_numpy(keep_np).to(DEV), torch.from_numpy(kept_np).to(DEV),
                      dst, 3)
    assert kv.kvtrim_poll_error(ctx) == 0
    assert compare_caches(device_cache_to_host(w, dst), dst_ref)


@pytest.mark.parametrize("G,D,horizon,many", [(4, 128, 1, False), (1, 128, 2, False), (5, 128, 1, False), (3, 128, 1, True),
                                              (2, 64, 1, False), (4, 64, 2, False)])
def test_sparse_selection_in_the_fused_call_gathers_by_destination_chunk(G, D, horizon, many):
    # compaction + attention in one call with a destination under a quarter of the source and a group of query heads
    # the one-shot kernel serves: its gathering instance runs, a block per 128-row chunk of the DESTINATION reading the
    # source rows the compaction scan has listed.  One entry in sixteen survives on average; some source chunks keep
    # nothing, some everything, one segment is empty, one keeps nothing, one keeps exactly one chunk's worth, segments
    # end in ragged chunks; `many`: more than 1024 segments (the scan's prefix kernel).  Layers [1, 3) attend.
    w = wl(2, 180 if many else 3, 3, G, D)
    rng = np.random.default_rng(1000 + 16 * G + D + horizon)
    seg_len = rng.integers(1, 700 if many else 6000, w.nseg)
    seg_len[3] = 0
    seg_len[5] = 128 * 9 + 1
    seg_len[7] = 300
    seg_len[9] = 128 * 20
    c, _ = ki.ragged_cache(w, seg_len, salt=35)
    c = ki.with_horizon(c, horizon)
    hc = host_cache(w, c)
    keep_np = (rng.random(hc.cap) < 1.0 / 16).astype(np.uint8)
    s5, s7, s9 = int(hc.seg_start[5]), int(hc.seg_start[7]), int(hc.seg_start[9])
    keep_np[s5 + 128:s5 + 3 * 128] = 1                            # two source chunks that keep everything
    keep_np[s5 + 4 * 128:s5 + 6 * 128] = 0                        # two that keep nothing
    keep_np[s5 + 9 * 128] = 1                                     # the one-entry tail chunk
    keep_np[s7:s7 + 300] = 0                                      # a segment that keeps nothing
    keep_np[s9:s9 + 128 * 20] = 0
    keep_np[s9 + 5:s9 + 128 * 20:20] = 1                          # exactly 128 survivors: one full destination chunk
    kept_np = np.array([keep_np[s:s + n].sum() for s, n in zip(hc.seg_start, hc.seg_len)], np.int32)
    assert kept_np[7] == 0 and kept_np[9] == 128
    dst_cap = int(kept_np.sum()) + 2 * w.nseg
    assert dst_cap < hc.cap // 4
    dst_ref = oracle.compact(hc, keep_np, dst_cap, 2)
    q = ki.decode_inputs(w, 3)["q"]
    scale = 1.0 / math.sqrt(D)
    ref, ref_lse = oracle.attend(dst_ref, bf16_bits(q), scale)
    ctx = kv.Context(w.n_seq, w.n_layers, w.n_kv_heads, w.n_q_heads, D, hc.cap)
    dst = kv.Cache.empty(w.nseg, D, dst_cap, DEV, with_tail=horizon != 1)
    out = torch.full(ref.shape, 99.0, dtype=torch.float32, device=DEV)
    lse = torch.full(ref_lse.shape, 99.0, dtype=torch.float32, device=DEV)
    keep_d, kept_d = torch.from_numpy(keep_np).to(DEV), torch.from_numpy(kept_np).to(DEV)
    kv.kvtrim_profile_begin(ctx, (1 << kv.binding.N_KERNELS) - 1)
    kv.kvtrim_compact_attn(ctx, kv.Cache.from_dict(c, DEV), keep_d, kept_d, dst, 2, q.to(DEV), 1, 3, scale, out, lse)
    times = kv.kvtrim_profile_end(ctx)
    assert kv.kvtrim_poll_error(ctx) == 0
    assert times["k_cmp_attn"][1] == 1 and "k_cmp_copy" not in times      # the fused kernel ran, not the two stages
    assert compare_caches(device_cache_to_host(w, dst), dst_ref)
    o = out.cpu().numpy()
    assert np.all(o[:, 0] == 99.0)
    assert attn_error(o[:, 1:3], ref[:, 1:3]) <= ATTN_TOL
    fin = np.isfinite(ref_lse[:, 1:3])
    assert np.abs(lse.cpu().numpy()[:, 1:3][fin] - ref_lse[:, 1:3][fin]).max() <= 2e-3
    assert np.all(np.isneginf(lse.cpu().numpy()[:, 1:3][~fin]))
    # a mask with more survivors than `kept` says is reported (as that, not as a failed HIP call)
    keep_bad = keep_np.copy()
    keep_bad[s7:s7 + 300] = 1
    guard = kv.Cache.empty(w.nseg, D, dst_cap, DEV, with_tail=horizon != 1)
    kv.kvtrim_compact_attn(ctx, kv.Cache.from_dict(c, DEV), torch.from_numpy(keep_bad).to(DEV), kept_d, guard, 2, q.to(DEV),
                           1, 3, scale, out, lse)
    assert kv.kvtrim_poll_error(ctx) == -5                         # KVTRIM_EMISMATCH
    assert kv.kvtrim_poll_error(ctx) == 0


# ---------------------------------------------------------------------------------- degenerate budgets, ties

def run_select_compact(w, c, now, budget, score_override=None, reserve=1):
    """One score -> select -> compact on both sides; returns (gpu results, oracle results)."""
    hc = host_cache(w, c)
    total = int(hc.seg_len.sum())
    dst_cap = min(int(sum(budget)), total) + w.nseg * reserve + 4
    ctx = kv.Context(w.n_seq, w.n_layers, w.n_kv_heads, w.n_q_heads, w.head_dim, max(hc.cap, dst_cap))
    src = kv.Cache.from_dict(c, DEV)
    dst = kv.Cache.empty(w.nseg, w.head_dim, dst_cap, DEV)
    score = torch.zeros(hc.cap, dtype=torch.float32, device=DEV)
    keep = torch.full((hc.cap,), 7, dtype=torch.uint8, device=DEV)
    kept = torch.zeros(w.nseg, dtype=torch.int32, device=DEV)
    thr = torch.zeros(w.n_seq, dtype=torch.int32, device=DEV)
    kv.kvtrim_score(ctx, src, now.to(DEV), score)
    score_ref = oracle.score(hc, now.numpy())
    if score_override is not None:
        score_ref = score_override.copy()
        score.copy_(torch.from_numpy(score_override))
    b = torch.tensor(budget, dtype=torch.int64, device=DEV)
    kv.kvtrim_select_global(ctx, src, score, b, keep, kept, thr)
    kv.kvtrim_compact(ctx, src, keep, kept, dst, reserve)
    assert kv.kvtrim_poll_error(ctx) == 0
    keep_ref, kept_ref, thr_ref = oracle.select(hc, score_ref, np.array(budget, np.int64))
    dst_ref = oracle.compact(hc, keep_ref, dst_cap, reserve)
    live = live_mask(hc)
    assert np.array_equal(score.cpu().numpy()[live].view(np.uint32), score_ref[live].view(np.uint32))
    assert np.array_equal(keep.cpu().numpy()[live], keep_ref[live])
    assert np.array_equal(kept.cpu().numpy(), kept_ref)
    assert np.array_equal(thr.cpu().numpy().view(np.uint32), thr_ref)
    assert compare_caches(device_cache_to_host(w, dst), dst_ref)
    return kept_ref


@pytest.mark.parametrize("frac", [0.0, 1.0, 2.0, 0.5])
def test_budget_zero_full_and_above_full(frac):
    w = wl(2, 2, 2, 2, 64)
    rng = np.random.default_rng(11)
    seg_len = rng.integers(0, 3000, w.nseg)
    c, now = ki.ragged_cache(w, seg_len, salt=5)
    per_seq = [int(seg_len[s * 4:(s + 1) * 4].sum()) for s in range(2)]
    kept = run_select_compact(w, c, now, [int(frac * n) for n in per_seq])
    for s in range(2):
        assert kept[s * 4:(s + 1) * 4].sum() == min(int(frac * per_seq[s]), per_seq[s])


def test_all_scores_equal_keeps_the_first_entries_in_storage_order():
    w = wl(1, 2, 2, 2, 64)
    seg_len = [3000, 2500, 4100, 100]
    c, now = ki.ragged_cache(w, seg_len, salt=6)
    score = np.full(sum(seg_len) + 4, -3.0, np.float32)
    for B in (1, 2999, 3000, 3001, 5500, 7777, 9699, 9700):
        kept = run_select_compact(w, c, now, [B], score_override=score)
        expect, left = [], B
        for n in seg_len:
            expect.append(min(n, left))
            left -= expect[-1]
        assert kept.tolist() == expect


def test_heavy_ties_signed_zeros_and_infinities():
    w = wl(2, 1, 3, 2, 64)
    rng = np.random.default_rng(12)
    seg_len = rng.integers(1000, 5000, w.nseg)
    c, now = ki.ragged_cache(w, seg_len, salt=7)
    cap = int(seg_len.sum()) + w.nseg
    vals = np.array([-np.inf, -7.5, -7.5, -1e-20, -0.0, 0.0, -2.0000002, -2.0], np.float32)
    score = rng.choice(vals, size=cap).astype(np.float32)
    for frac in (0.1, 0.37, 0.5, 0.93):
        budget = [int(frac * seg_len[:3].sum()), int(frac * seg_len[3:].sum())]
        run_select_compact(w, c, now, budget, score_override=score)


def test_keys_differing_only_in_low_bits():
    w = wl(1, 1, 2, 2, 64)
    seg_len = [5000, 5000]
    c, now = ki.ragged_cache(w, seg_len, salt=8)
    rng = np.random.default_rng(13)
    bits = (np.float32(-1.5).view(np.uint32) + rng.integers(0, 1 << 9, sum(seg_len) + 2).astype(np.uint32))
    score = bits.view(np.float32)
    for B in (1, 100, 4999, 9000):
        run_select_compact(w, c, now, [B], score_override=score)


# ---------------------------------------------------------------------------------- attention alone

@pytest.mark.parametrize("D,G", [(128, 4), (128, 7), (64, 2), (128, 1), (64, 8)])
def test_attention_against_oracle_and_layer_ranges(D, G):
    w = wl(2, 3, 2, G, D)
    rng = np.random.default_rng(D + G)
    seg_len = rng.integers(0, 1500, w.nseg)
    seg_len[0] = 0
    seg_len[1] = 1
    seg_len[2] = 257
    c, _ = ki.ragged_cache(w, seg_len, salt=9)
    hc = host_cache(w, c)
    dc = kv.Cache.from_dict(c, DEV)
    ctx = kv.Context(w.n_seq, w.n_layers, w.n_kv_heads, w.n_q_heads, D, hc.cap)
    q = ki.decode_inputs(w, 0)["q"]
    scale = 1.0 / math.sqrt(D)
    ref, ref_lse = oracle.attend(hc, bf16_bits(q), scale)
    out = torch.full(ref.shape, 99.0, dtype=torch.float32, device=DEV)
    lse = torch.full(ref_lse.shape, 99.0, dtype=torch.float32, device=DEV)
    kv.kvtrim_decode_attn(ctx, dc, q.to(DEV), 0, w.n_layers, scale, out, lse)
    assert kv.kvtrim_poll_error(ctx) == 0
    assert attn_error(out.cpu().numpy(), ref) <= ATTN_TOL
    o = out.cpu().numpy()
    assert np.all(o[0, 0, :G] == 0.0)                                   # empty segment
    assert np.isneginf(lse.cpu().numpy()[0, 0, :G]).all()
    fin = np.isfinite(ref_lse)
    assert np.abs(lse.cpu().numpy()[fin] - ref_lse[fin]).max() <= 2e-3
    # a layer range writes only its layers
    out2 = torch.full(ref.shape, 99.0, dtype=torch.float32, device=DEV)
    kv.kvtrim_decode_attn(ctx, dc, q.to(DEV), 1, 2, scale, out2, None)
    o2 = out2.cpu().numpy()
    assert np.all(o2[:, 0] == 99.0) and np.all(o2[:, 2] == 99.0)
    # (the rows are shared out among the kernel's blocks per call, so the order of the fp32 sums - not their terms -
    # depends on the layer range)
    assert attn_error(o2[:, 1], o[:, 1]) <= 2e-6


@pytest.mark.parametrize("blocks", [1, 2, 3, 7, 50, 100000])
def test_attention_for_any_size_of_the_fixed_grid(blocks, monkeypatch):
    # the attention kernel's blocks share the chunk table in equal parts of 64 rows and leave one partial result per
    # block and segment; whatever the number of blocks (a tuning knob read when the context is created) - one block
    # that walks everything, shares that end inside a chunk or inside a segment, more blocks than chunks - the
    # merge must find exactly those partial results
    monkeypatch.setenv("KVTRIM_ATT_BLOCKS", str(blocks))
    w = wl(2, 2, 2, 4, 128)
    seg_len = [3000, 0, 513, 64, 1, 2049, 700, 5000]
    c, _ = ki.ragged_cache(w, seg_len, salt=21)
    hc = host_cache(w, c)
    dc = kv.Cache.from_dict(c, DEV)
    ctx = kv.Context(w.n_seq, w.n_layers, w.n_kv_heads, w.n_q_heads, 128, hc.cap)
    q = ki.decode_inputs(w, 0)["q"]
    scale = 1.0 / math.sqrt(128)
    ref, ref_lse = oracle.attend(hc, bf16_bits(q), scale)
    for rng in ((0, 2), (1, 2)):
        out = torch.full(ref.shape, 99.0, dtype=torch.float32, device=DEV)
        lse = torch.full(ref_lse.shape, 99.0, dtype=torch.float32, device=DEV)
        kv.kvtrim_decode_attn(ctx, dc, q.to(DEV), rng[0], rng[1], scale, out, lse)
        assert kv.kvtrim_poll_error(ctx) == 0
        o, l = out.cpu().numpy()[:, rng[0]:rng[1]], lse.cpu().numpy()[:, rng[0]:rng[1]]
        assert attn_error(o, ref[:, rng[0]:rng[1]]) <= ATTN_TOL, (blocks, rng)
        fin = np.isfinite(ref_lse[:, rng[0]:rng[1]])
        assert np.abs(l[fin] - ref_lse[:, rng[0]:rng[1]][fin]).max() <= 2e-3
        assert np.array_equal(np.isneginf(l), ~fin)


@pytest.mark.parametrize("seed", range(8))
def test_attention_on_random_shapes_ranges_and_grids(seed, monkeypatch):
    # random segment lengths (many empty or tiny ones beside long ones), a random layer range and a random number of
    # blocks for the attention kernel's fixed grid: the shares of the blocks start and end anywhere
    rng = np.random.default_rng(1000 + seed)
    S, L, H = int(rng.integers(1, 4)), int(rng.integers(1, 4)), int(rng.integers(1, 4))
    G, D = int(rng.choice([1, 2, 4, 7])), int(rng.choice([64, 128]))
    monkeypatch.setenv("KVTRIM_ATT_BLOCKS", str(int(rng.choice([1, 2, 3, 5, 9, 17, 40, 768]))))
    w = wl(S, L, H, G, D)
    kinds = rng.integers(0, 5, w.nseg)
    seg_len = np.where(kinds == 0, 0, np.where(kinds == 1, rng.integers(1, 70, w.nseg),
                       np.where(kinds == 2, rng.integers(400, 700, w.nseg), rng.integers(1000, 6000, w.nseg))))
    c, _ = ki.ragged_cache(w, seg_len, salt=30 + seed)
    hc = host_cache(w, c)
    dc = kv.Cache.from_dict(c, DEV)
    ctx = kv.Context(S, L, H, H * G, D, hc.cap)
    q = ki.decode_inputs(w, seed)["q"]
    scale = 1.0 / math.sqrt(D)
    ref, ref_lse = oracle.attend(hc, bf16_bits(q), scale)
    lb = int(rng.integers(0, L))
    le = int(rng.integers(lb + 1, L + 1))
    out = torch.full(ref.shape, 99.0, dtype=torch.float32, device=DEV)
    lse = torch.full(ref_lse.shape, 99.0, dtype=torch.float32, device=DEV)
    kv.kvtrim_decode_attn(ctx, dc, q.to(DEV), lb, le, scale, out, lse)
    assert kv.kvtrim_poll_error(ctx) == 0
    o, l = out.cpu().numpy(), lse.cpu().numpy()
    outside = [x for x in range(L) if not lb <= x < le]
    assert np.all(o[:, outside] == 99.0) and np.all(l[:, outside] == 99.0)
    if np.abs(ref[:, lb:le]).max() > 0:
        assert attn_error(o[:, lb:le], ref[:, lb:le]) <= ATTN_TOL, (seed, seg_len.tolist(), lb, le)
    else:
        assert np.all(o[:, lb:le] == 0.0)
    fin = np.isfinite(ref_lse[:, lb:le])
    assert np.array_equal(np.isneginf(l[:, lb:le]), ~fin)
    if fin.any():
        assert np.abs(l[:, lb:le][fin] - ref_lse[:, lb:le][fin]).max() <= 2e-3


def test_attention_with_large_logits_stays_finite():
    w = wl(1, 1, 1, 4, 128)
    c, _ = ki.ragged_cache(w, [900], salt=10)
    c["k"] *= 6.0
    hc = host_cache(w, c)
    q = ki.decode_inputs(w, 1)["q"] * 6.0
    ctx = kv.Context(1, 1, 1, 4, 128, hc.cap)
    ref, _ = oracle.attend(hc, bf16_bits(q), 1.0)
    out = torch.zeros(ref.shape, dtype=torch.float32, device=DEV)
    kv.kvtrim_decode_attn(ctx, kv.Cache.from_dict(c, DEV), q.to(DEV), 0, 1, 1.0, out, None)
    o = out.cpu().numpy()
    assert np.isfinite(o).all() and attn_error(o, ref) <= ATTN_TOL


# ---------------------------------------------------------------------------------- error paths (kernels exit normally)

def test_device_side_errors_are_reported_and_nothing_overflows():
    w = wl(1, 1, 4, 2, 64)
    seg_len = [300, 10, 0, 500]
    c, now = ki.ragged_cache(w, seg_len, reserve=1, salt=14)
    cap = sum(seg_len) + 4
    ctx = kv.Context(1, 1, 4, 8, 64, cap)
    src = kv.Cache.from_dict(c, DEV)
    keep = torch.ones(cap, dtype=torch.uint8, device=DEV)
    kept = torch.tensor(seg_len, dtype=torch.int32, device=DEV)
    small = kv.Cache.empty(4, 64, 700, DEV)
    small.k.fill_(1.0)
    kv.kvtrim_compact(ctx, src, keep, kept, small, 1)
    assert kv.kvtrim_poll_error(ctx) == -4                               # KVTRIM_ECAP
    assert torch.all(small.k == 1.0)                                     # nothing was written
    assert kv.kvtrim_poll_error(ctx) == 0                                # flag cleared
    big = kv.Cache.empty(4, 64, cap, DEV)
    wrong = kept.clone()
    wrong[0] -= 1
    kv.kvtrim_compact(ctx, src, keep, wrong, big, 1)
    assert kv.kvtrim_poll_error(ctx) == -5                               # KVTRIM_EMISMATCH
    # appending two tokens where one slot is reserved
    new = ki.decode_inputs(w, 0)
    two = lambda t: torch.stack([t, t], 1).contiguous().to(DEV)
    before = src.seg_len.clone()
    kv.kvtrim_append(ctx, src, two(new["k_new"]), two(new["v_new"]), two(new["log_beta_new"]),
                     torch.zeros(4, 2, dtype=torch.int32, device=DEV), 2)
    assert kv.kvtrim_poll_error(ctx) == -4
    assert torch.equal(src.seg_len, before)
    # an inconsistent segment table
    bad = kv.Cache(src.k, src.v, src.log_beta, src.pos, src.seg_start, torch.tensor([300, 10, 0, 900], dtype=torch.int32, device=DEV))
    score = torch.zeros(cap, dtype=torch.float32, device=DEV)
    kv.kvtrim_score(ctx, bad, now.to(DEV), score)
    kv.kvtrim_select_global(ctx, bad, score, torch.tensor([5], dtype=torch.int64, device=DEV), keep, kept)
    assert kv.kvtrim_poll_error(ctx) == -6                               # KVTRIM_ELAYOUT


@pytest.mark.parametrize("nseg", [6, 1500])
def test_compaction_rejects_overlapping_segments_and_leaves_the_destination_alone(nseg):
    # a segment that runs into its successor (still inside the buffers) must not reach the row movers, in either
    # form of the compaction scan (one block per segment summing all segments itself: up to 1024 segments; a prefix
    # kernel first: more); and a destination that is too small is left untouched, segment table included
    w = wl(1, 1, nseg, 1, 64)
    seg_len = [20] * nseg
    c, now = ki.ragged_cache(w, seg_len, reserve=1, salt=3)
    cap = c["cap"]
    ctx = kv.Context(1, 1, nseg, nseg, 64, cap + 64)
    src = kv.Cache.from_dict(c, DEV)
    keep = torch.ones(cap, dtype=torch.uint8, device=DEV)
    kept = torch.tensor(seg_len, dtype=torch.int32, device=DEV)
    q = torch.zeros(1, 1, nseg, 64, dtype=torch.bfloat16, device=DEV)
    out = torch.zeros(1, 1, nseg, 64, dtype=torch.float32, device=DEV)

    def fresh(n):
        d = kv.Cache.empty(nseg, 64, n, DEV)
        d.k.fill_(1.0)
        d.seg_start.fill_(-7)
        d.seg_len.fill_(-7)
        return d

    small = fresh(sum(seg_len) + nseg - 1)                        # one slot short
    for call in ("compact", "compact_attn"):
        if call == "compact":
            kv.kvtrim_compact(ctx, src, keep, kept, small, 1)
        else:
            kv.kvtrim_compact_attn(ctx, src, keep, kept, small, 1, q, 0, 1, 0.125, out)
        assert kv.kvtrim_poll_error(ctx) == -4                    # KVTRIM_ECAP
        assert torch.all(small.k == 1.0) and torch.all(small.seg_start == -7) and torch.all(small.seg_len == -7)
    lens = src.seg_len.clone()
    lens[2] = 25                                                  # 4 entries into segment 3's range
    bad = kv.Cache(src.k, src.v, src.log_beta, src.pos, src.seg_start, lens)
    kept_bad = kept.clone()
    kept_bad[2] = 25
    big = fresh(cap + 64)
    for call in ("compact", "compact_attn", "inplace"):
        if call == "compact":
            kv.kvtrim_compact(ctx, bad, keep, kept_bad, big, 1)
        elif call == "compact_attn":
            kv.kvtrim_compact_attn(ctx, bad, keep, kept_bad, big, 1, q, 0, 1, 0.125, out)
        else:
            spare = kv.Cache.empty(nseg, 64, cap, DEV)
            before = bad.k.clone()
            kv.kvtrim_compact_attn_inplace(ctx, bad, keep, kept_bad, spare, q, 0, 1, 0.125, out)
            assert torch.equal(bad.k, before)
        assert kv.kvtrim_poll_error(ctx) == -6                    # KVTRIM_ELAYOUT
        assert torch.all(big.k == 1.0) and torch.all(big.seg_len == -7)


def test_host_side_argument_checks():
    ctx = kv.Context(1, 1, 2, 4, 64, 100)
    c = kv.Cache.empty(2, 64, 100, DEV)
    too_big = kv.Cache.empty(2, 64, 101, DEV)
    score = torch.zeros(101, dtype=torch.float32, device=DEV)
    now = torch.zeros(1, dtype=torch.int32, device=DEV)
    with pytest.raises(kv.KvtrimError) as e:
        kv.kvtrim_score(ctx, too_big, now, score)
    assert e.value.status == -1
    keep = torch.zeros(100, dtype=torch.uint8, device=DEV)
    kept = torch.zeros(2, dtype=torch.int32, device=DEV)
    with pytest.raises(kv.KvtrimError):
        kv.kvtrim_compact(ctx, c, keep, kept, c, 1)                      # src == dst
    q = torch.zeros(1, 1, 4, 64, dtype=torch.bfloat16, device=DEV)
    out = torch.zeros(1, 1, 4, 64, dtype=torch.float32, device=DEV)
    with pytest.raises(kv.KvtrimError):
        kv.kvtrim_decode_attn(ctx, c, q, 0, 2, 0.125, out)               # layer range beyond L
    with pytest.raises(kv.KvtrimError):
        kv.Context(1, 1, 2, 4, 96, 100)


def test_results_are_deterministic_across_runs():
    w = ki.workload("llama", prefill=500)
    a = run_steps_both(w, steps=2, budget=w.budget, device=DEV)
    b = run_steps_both(w, steps=2, budget=w.budget, device=DEV)
    check(a)
    assert [r["attn_err"] for r in a] == [r["attn_err"] for r in b]


# ---------------------------------------------------------------------------------- soft attention, occupancy

@pytest.mark.parametrize("D,G,S", [(128, 4, 1), (64, 2, 2), (128, 7, 2)])
def test_soft_retention_gated_attention_and_occupancy(D, G, S):
    w = wl(S, 2, 2, G, D)
    rng = np.random.default_rng(D + G + S)
    seg_len = rng.integers(0, 1800, w.nseg)
    seg_len[1] = 0
    c, now = ki.ragged_cache(w, seg_len, salt=40 + G)
    hc = host_cache(w, c)
    dc = kv.Cache.from_dict(c, DEV)
    ctx = kv.Context(w.n_seq, w.n_layers, w.n_kv_heads, w.n_q_heads, D, hc.cap)
    q = ki.decode_inputs(w, 2)["q"]
    scale = 1.0 / math.sqrt(D)
    now_np = now.numpy() + 3
    ref, ref_lse = oracle.attend(hc, bf16_bits(q), scale, soft_now=now_np)
    out = torch.full(ref.shape, 99.0, dtype=torch.float32, device=DEV)
    lse = torch.full(ref_lse.shape, 99.0, dtype=torch.float32, device=DEV)
    now_dev = torch.from_numpy(now_np).to(DEV)
    kv.kvtrim_decode_attn_soft(ctx, dc, q.to(DEV), now_dev, 0, w.n_layers, scale, out, lse)
    assert kv.kvtrim_poll_error(ctx) == 0
    assert attn_error(out.cpu().numpy(), ref) <= ATTN_TOL
    fin = np.isfinite(ref_lse)
    assert np.abs(lse.cpu().numpy()[fin] - ref_lse[fin]).max() <= 2e-3
    assert np.array_equal(np.isneginf(lse.cpu().numpy()), np.isneginf(ref_lse))
    # the soft form differs from the hard one on this input, and beta = 1 makes them coincide
    hard, _ = oracle.attend(hc, bf16_bits(q), scale)
    assert attn_error(out.cpu().numpy(), hard) > 10 * ATTN_TOL
    ones = dict(c)
    ones["log_beta"] = torch.zeros_like(c["log_beta"])
    out1 = torch.zeros_like(out)
    out2 = torch.zeros_like(out)
    d1 = kv.Cache.from_dict(ones, DEV)
    kv.kvtrim_decode_attn_soft(ctx, d1, q.to(DEV), now_dev, 0, w.n_layers, scale, out1)
    kv.kvtrim_decode_attn(ctx, d1, q.to(DEV), 0, w.n_layers, scale, out2)
    assert torch.equal(out1, out2)
    # occupancy
    occ = torch.zeros(S, dtype=torch.float64, device=DEV)
    kv.kvtrim_occupancy(ctx, dc, now_dev, occ)
    np.testing.assert_allclose(occ.cpu().numpy(), oracle.occupancy(hc, now_np), rtol=2e-6)


def test_many_segments_take_the_prefix_kernel_and_report_errors():
    # more than 1024 segments: the segment prefixes of the compaction come from one extra block instead of a
    # reduction in every block; results and device-side errors must be the same
    w = wl(9, 8, 16, 1, 64)                                        # 1152 segments
    rng = np.random.default_rng(77)
    seg_len = rng.integers(0, 40, w.nseg)
    c, now = ki.ragged_cache(w, seg_len, reserve=1, salt=8)
    per_seq = [int(seg_len[s * 128:(s + 1) * 128].sum()) for s in range(9)]
    check(run_steps_both(w, steps=2, budget=[max(1, n // 2) for n in per_seq], device=DEV, cache_dict=c, now0=now.numpy(),
                         fused=True))
    hc = host_cache(w, c)
    ctx = kv.Context(w.n_seq, w.n_layers, w.n_kv_heads, w.n_q_heads, w.head_dim, hc.cap)
    src = kv.Cache.from_dict(c, DEV)
    keep = torch.ones(hc.cap, dtype=torch.uint8, device=DEV)
    kept = torch.from_numpy(hc.seg_len.copy()).to(DEV)
    small = kv.Cache.empty(w.nseg, w.head_dim, int(hc.seg_len.sum()) // 2, DEV)
    kv.kvtrim_compact(ctx, src, keep, kept, small, 0)
    assert kv.kvtrim_poll_error(ctx) == -4                         # destination too small
    roomy = kv.Cache.empty(w.nseg, w.head_dim, hc.cap, DEV)
    kept[5] += 1
    kv.kvtrim_compact(ctx, src, keep, kept, roomy, 0)
    assert kv.kvtrim_poll_error(ctx) == -5                         # kept disagrees with the mask
    kept[5] -= 1
    kv.kvtrim_compact(ctx, src, keep, kept, roomy, 0)
    assert kv.kvtrim_poll_error(ctx) == 0
    assert compare_caches(device_cache_to_host(w, roomy), oracle.compact(hc, np.ones(hc.cap, np.uint8), hc.cap, 0))
