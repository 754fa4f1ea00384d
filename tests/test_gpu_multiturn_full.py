"""GPU parity of the multi-turn workload at its real size: 16 sequences of 4096 .. 65536 tokens, 32 layers x 8 KV
heads, every sequence with its own budget of 8192 * 32 * 8 entries, chunks of 4096 tokens per segment.

A cache of 33.5 M retained entries (17 GB of K/V) cannot go to the host row by row, so every step is checked the way
the 128K first eviction is: the oracle scores and selects on the metadata alone and that is compared WHOLE (score
bits, mask, per-segment counts, threshold keys; 50 M candidates in a chunk step), the compacted cache's segment table
and per-entry metadata WHOLE, K/V rows and the attention output on sampled segments (among them the longest and the
shortest segment of two different sequences).  Steps: a chunk through the four calls, a chunk through
kvtrim_append_compact, a decode step through kvtrim_score_select + kvtrim_compact_attn, and a chunk and a decode step
on the paged layout."""
import math

import numpy as np
import pytest
import torch

import kvtrim_inputs as ki
import oracle
import paper_2605_09649_amd as kv
from harness import attn_error, pick_segments, sampled_step_check
from helpers import bf16_bits, live_mask, shape_of
from paged_harness import PagedHost

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
ATTN_TOL = 5e-3
CHUNK = 4096


class State:
    pass


@pytest.fixture(scope="module")
def at_budget():
    """The 16-sequence cache after its first eviction down to the per-sequence budgets, with room for a chunk behind
    every segment, and the buffers the steps share."""
    w = ki.workload("multiturn")
    st = State()
    st.w = w
    st.per_seq = w.n_layers * w.n_kv_heads
    pre = ki.prefill_cache(w, reserve=1, device=DEV)
    src = kv.Cache.from_dict(pre, DEV)
    del pre
    B = sum(min(b, t * st.per_seq) for b, t in zip(w.budget, w.prefill))      # short sequences stay below their budget
    st.cap = sum(w.budget) + w.nseg * CHUNK + 8
    st.ctx = kv.Context(w.n_seq, w.n_layers, w.n_kv_heads, w.n_q_heads, w.head_dim, max(src.cap, st.cap))
    st.caches = [kv.Cache.empty(w.nseg, w.head_dim, st.cap, DEV) for _ in range(2)]
    n = max(src.cap, st.cap)
    st.score = torch.zeros(n, dtype=torch.float32, device=DEV)
    st.keep = torch.zeros(n, dtype=torch.uint8, device=DEV)
    st.kept = torch.zeros(w.nseg, dtype=torch.int32, device=DEV)
    st.thr = torch.zeros(w.n_seq, dtype=torch.int32, device=DEV)
    st.budget_np = np.array(list(w.budget), np.int64)
    st.budget = torch.from_numpy(st.budget_np).to(DEV)
    st.out = torch.zeros(w.n_seq, w.n_layers, w.n_q_heads, w.head_dim, dtype=torch.float32, device=DEV)
    st.lse = torch.zeros(w.n_seq, w.n_layers, w.n_q_heads, dtype=torch.float32, device=DEV)
    st.scale = 1.0 / math.sqrt(w.head_dim)
    st.now = np.array([t - 1 for t in w.prefill], np.int32)          # position of every sequence's newest token
    # first eviction (not checked here: the 128K test covers a first eviction; this only builds the state)
    kv.kvtrim_score_select(st.ctx, src, torch.from_numpy(st.now).to(DEV), st.budget, st.score, st.keep, st.kept, st.thr, evict_hint=0)
    kv.kvtrim_compact(st.ctx, src, st.keep, st.kept, st.caches[0], CHUNK)
    assert kv.kvtrim_poll_error(st.ctx) == 0
    assert int(st.kept.sum().item()) == B
    del src
    torch.cuda.empty_cache()
    st.cur, st.flip = st.caches[0], 1
    st.chunk = ki.chunk_inputs(w, CHUNK, DEV, 1)
    return st


def chunk_positions(st):
    """Positions of a chunk's tokens for every segment ([nseg][CHUNK], the same for all segments of a sequence)."""
    ar = np.arange(CHUNK, dtype=np.int32)
    pos = np.repeat((st.now[:, None] + 1 + ar[None, :]), st.per_seq, axis=0).astype(np.int32)
    return pos


def assert_step(chk, attention):
    for k in ("score_equal", "keep_equal", "kept_equal", "thr_equal", "tables_equal", "metadata_equal", "rows_equal"):
        assert chk[k], (k, {a: b for a, b in chk.items() if a != "sampled_segments"})
    assert len(chk["sampled_segments"]) >= 10
    if attention:
        assert chk["attn_err"] <= ATTN_TOL and chk["lse_err"] <= 2e-3, chk


def test_chunk_step_through_the_four_calls(at_budget):
    st, w = at_budget, at_budget.w
    pos_new = chunk_positions(st)
    st.now = st.now + CHUNK
    now_dev = torch.from_numpy(st.now).to(DEV)
    src, dst = st.cur, st.caches[st.flip]
    kv.kvtrim_append(st.ctx, src, st.chunk["k_new"], st.chunk["v_new"], st.chunk["log_beta_new"], torch.from_numpy(pos_new).to(DEV), CHUNK)
    kv.kvtrim_score(st.ctx, src, now_dev, st.score)
    kv.kvtrim_select_global(st.ctx, src, st.score, st.budget, st.keep, st.kept, st.thr)
    kv.kvtrim_compact(st.ctx, src, st.keep, st.kept, dst, CHUNK)
    assert kv.kvtrim_poll_error(st.ctx) == 0
    chk = sampled_step_check(w, src, st.now, st.budget_np, CHUNK,
                             {"score": st.score, "keep": st.keep, "kept": st.kept, "thr": st.thr, "dst": dst})
    assert_step(chk, attention=False)
    assert chk["candidates"] > 45_000_000 and chk["kept_total"] == int(sum(w.budget))   # every sequence is at its budget now
    st.cur, st.flip = dst, st.flip ^ 1


def test_chunk_step_through_append_compact(at_budget):
    st, w = at_budget, at_budget.w
    pos_new = chunk_positions(st)
    st.now = st.now + CHUNK
    src, dst = st.cur, st.caches[st.flip]
    old_len = src.seg_len.cpu().numpy().copy()
    kv.kvtrim_append_compact(st.ctx, src, st.chunk["k_new"], st.chunk["v_new"], st.chunk["log_beta_new"],
                             torch.from_numpy(pos_new).to(DEV), CHUNK, torch.from_numpy(st.now).to(DEV), st.budget,
                             st.score, st.keep, st.kept, dst, CHUNK, thr_key_out=st.thr)
    assert kv.kvtrim_poll_error(st.ctx) == 0
    chk = sampled_step_check(w, src, st.now, st.budget_np, CHUNK,
                             {"score": st.score, "keep": st.keep, "kept": st.kept, "thr": st.thr, "dst": dst},
                             new_rows=(st.chunk["k_new"], st.chunk["v_new"], CHUNK, old_len))
    assert_step(chk, attention=False)
    assert chk["kept_total"] == int(sum(w.budget))
    st.cur, st.flip = dst, st.flip ^ 1


@pytest.mark.parametrize("hint", [256, 0])
def test_decode_step_through_score_select_and_compact_attn(at_budget, hint):
    st, w = at_budget, at_budget.w
    inp = ki.decode_inputs(w, 7 + hint, device=DEV)
    st.now = st.now + 1
    pos_new = np.repeat(st.now, st.per_seq).astype(np.int32)
    src, dst = st.cur, st.caches[st.flip]
    kv.kvtrim_append(st.ctx, src, inp["k_new"], inp["v_new"], inp["log_beta_new"], torch.from_numpy(pos_new).to(DEV), 1)
    kv.kvtrim_score_select(st.ctx, src, torch.from_numpy(st.now).to(DEV), st.budget, st.score, st.keep, st.kept, st.thr, evict_hint=hint)
    kv.kvtrim_compact_attn(st.ctx, src, st.keep, st.kept, dst, CHUNK, inp["q"], 0, w.n_layers, st.scale, st.out, st.lse)
    assert kv.kvtrim_poll_error(st.ctx) == 0
    chk = sampled_step_check(w, src, st.now, st.budget_np, CHUNK,
                             {"score": st.score, "keep": st.keep, "kept": st.kept, "thr": st.thr, "dst": dst, "out": st.out, "lse": st.lse},
                             q=inp["q"], scale=st.scale)
    assert_step(chk, attention=True)
    st.cur, st.flip = dst, st.flip ^ 1


def ordered_metadata(pc, w):
    """The pages' live entries as a metadata-only ragged cache (every segment in position order) and the slot of
    every entry."""
    ph = PagedHost(pc, rows=False)
    assert ph.structure_problems() == []
    idx, counts = ph.ordered_slots()
    starts = np.concatenate([[0], np.cumsum(counts.astype(np.int64))[:-1]]).astype(np.int64)
    empty = np.zeros((0, w.head_dim), np.uint16)
    meta = oracle.HostCache.from_arrays(shape_of(w), empty, empty, ph.log_beta[idx], ph.pos[idx], starts, counts)
    return meta, idx, ph


def test_chunk_and_decode_step_on_pages(at_budget):
    st, w = at_budget, at_budget.w
    P = kv.PAGE_SIZE
    src = st.cur
    # the retained entries go into pages (a selection that keeps everything, then the page-aligned gather)
    huge = torch.full((w.n_seq,), 1 << 40, dtype=torch.int64, device=DEV)
    kv.kvtrim_score_select(st.ctx, src, torch.from_numpy(st.now).to(DEV), huge, st.score, st.keep, st.kept, st.thr, evict_hint=0)
    n_live = int(st.kept.sum().item())
    n_pages = (n_live + w.nseg * CHUNK) // P + 3 * w.nseg + 64
    pc = kv.PagedCache(w.nseg, w.head_dim, n_pages, n_pages, DEV)
    kv.kvtrim_paged_build(st.ctx, src, st.keep, st.kept, pc)
    assert kv.kvtrim_poll_error(st.ctx) == 0
    before, _, _ = ordered_metadata(pc, w)
    live_src = live_mask(oracle.HostCache.from_arrays(shape_of(w), np.zeros((0, w.head_dim), np.uint16), np.zeros((0, w.head_dim), np.uint16),
                                                      src.log_beta.cpu().numpy(), src.pos.cpu().numpy(), src.seg_start.cpu().numpy(),
                                                      src.seg_len.cpu().numpy()))
    assert np.array_equal(before.pos, src.pos.cpu().numpy()[live_src]) and np.array_equal(before.seg_len, src.seg_len.cpu().numpy())

    n_slots = n_pages * P
    score = st.score[:n_slots] if st.score.numel() >= n_slots else torch.zeros(n_slots, dtype=torch.float32, device=DEV)
    keep = st.keep[:n_slots] if st.keep.numel() >= n_slots else torch.zeros(n_slots, dtype=torch.uint8, device=DEV)

    def paged_step(k_new, v_new, lb_new, pos_new, n_new, q):
        kv.kvtrim_paged_append(st.ctx, pc, k_new, v_new, lb_new, torch.from_numpy(pos_new).to(DEV), n_new=n_new)
        assert kv.kvtrim_poll_error(st.ctx) == 0
        meta, idx, _ = ordered_metadata(pc, w)                      # after the append: old and new entries, in position order
        kv.kvtrim_paged_score(st.ctx, pc, torch.from_numpy(st.now).to(DEV), score)
        kv.kvtrim_paged_select(st.ctx, pc, score, st.budget, keep, st.kept, st.thr)
        kv.kvtrim_paged_evict(st.ctx, pc, keep)
        if q is not None:
            kv.kvtrim_paged_attn(st.ctx, pc, q, 0, w.n_layers, st.scale, st.out, st.lse)
        assert kv.kvtrim_poll_error(st.ctx) == 0
        s_ref = oracle.score(meta, st.now)
        keep_ref, kept_ref, thr_ref = oracle.select(meta, s_ref, st.budget_np)
        idx_dev = torch.from_numpy(idx).to(DEV)
        assert np.array_equal(score[idx_dev].cpu().numpy().view(np.uint32), s_ref.view(np.uint32))
        assert np.array_equal(keep[idx_dev].cpu().numpy(), keep_ref)
        assert np.array_equal(st.kept.cpu().numpy(), kept_ref)
        assert np.array_equal(st.thr.cpu().numpy().view(np.uint32), thr_ref)
        after, idx_after, _ = ordered_metadata(pc, w)
        sel = keep_ref.astype(bool)
        assert np.array_equal(after.seg_len, kept_ref)
        assert np.array_equal(after.pos, meta.pos[sel]) and np.array_equal(after.log_beta.view(np.uint32), meta.log_beta[sel].view(np.uint32))
        # no K/V moves: a surviving entry is still in the slot it had before the eviction
        assert np.array_equal(idx_after, idx[sel])
        return meta, idx, keep_ref, kept_ref, after, idx_after

    # ---- a chunk of 4096 tokens per segment
    pos_new = chunk_positions(st)
    old_pos_max = st.now.copy()
    st.now = st.now + CHUNK
    meta, idx, keep_ref, kept_ref, after, idx_after = paged_step(st.chunk["k_new"], st.chunk["v_new"], st.chunk["log_beta_new"],
                                                                  pos_new, CHUNK, None)
    assert int(meta.seg_len.sum()) == n_live + w.nseg * CHUNK and int(kept_ref.sum()) == int(sum(w.budget))
    # the appended metadata: every segment holds its old positions and the chunk's, with the chunk's log beta
    lb_new = st.chunk["log_beta_new"].cpu().numpy()
    sample = pick_segments(w, kept_ref, 8, seed=11)
    assert len(sample) >= 10
    src_pos, src_start = src.pos.cpu().numpy(), src.seg_start.cpu().numpy()
    for g in sample:
        seq = g // st.per_seq
        a0, an = int(meta.seg_start[g]), int(meta.seg_len[g])
        p = meta.pos[a0:a0 + an]
        n_old = int(before.seg_len[g])
        assert np.array_equal(p[:n_old], before.pos[int(before.seg_start[g]):int(before.seg_start[g]) + n_old])
        assert np.array_equal(p[n_old:], pos_new[g]) and np.array_equal(meta.log_beta[a0 + n_old:a0 + an].view(np.uint32), lb_new[g].view(np.uint32))
        # rows of the survivors: old ones from the ragged cache (same order as `before`), new ones from the chunk
        b0, bn = int(after.seg_start[g]), int(after.seg_len[g])
        ap = after.pos[b0:b0 + bn]
        slots = torch.from_numpy(idx_after[b0:b0 + bn]).to(DEV)
        is_new = ap > old_pos_max[seq]
        old_at = np.searchsorted(before.pos[int(before.seg_start[g]):int(before.seg_start[g]) + n_old], ap[~is_new])
        exp_k = np.concatenate([bf16_bits(src.k[torch.from_numpy(src_start[g] + old_at).to(DEV)]),
                                bf16_bits(st.chunk["k_new"][g][torch.from_numpy(ap[is_new] - old_pos_max[seq] - 1).to(DEV)])])
        exp_v = np.concatenate([bf16_bits(src.v[torch.from_numpy(src_start[g] + old_at).to(DEV)]),
                                bf16_bits(st.chunk["v_new"][g][torch.from_numpy(ap[is_new] - old_pos_max[seq] - 1).to(DEV)])])
        assert np.array_equal(bf16_bits(pc.k[slots]), exp_k) and np.array_equal(bf16_bits(pc.v[slots]), exp_v), g

    # ---- a decode step with attention over the pages
    inp = ki.decode_inputs(w, 99, device=DEV)
    st.now = st.now + 1
    pos1 = np.repeat(st.now, st.per_seq).astype(np.int32)
    meta, idx, keep_ref, kept_ref, after, idx_after = paged_step(inp["k_new"], inp["v_new"], inp["log_beta_new"], pos1, 1, inp["q"])
    sample = pick_segments(w, kept_ref, 8, seed=12)
    G, D = w.group, w.head_dim
    q_host = bf16_bits(inp["q"]).reshape(w.n_seq, w.n_layers, w.n_q_heads, D)
    out_gpu, lse_gpu = st.out.cpu().numpy(), st.lse.cpu().numpy()
    rows_k, rows_v, lens, qs, outs, lses = [], [], [], [], [], []
    for g in sample:
        b0, bn = int(after.seg_start[g]), int(after.seg_len[g])
        slots = torch.from_numpy(idx_after[b0:b0 + bn]).to(DEV)
        rows_k.append(bf16_bits(pc.k[slots]))
        rows_v.append(bf16_bits(pc.v[slots]))
        lens.append(bn)
        seq, lh = divmod(g, st.per_seq)
        layer, head = divmod(lh, w.n_kv_heads)
        qs.append(q_host[seq, layer, head * G:(head + 1) * G])
        outs.append(out_gpu[seq, layer, head * G:(head + 1) * G])
        lses.append(lse_gpu[seq, layer, head * G:(head + 1) * G])
    starts = np.concatenate([[0], np.cumsum(lens)[:-1]]).astype(np.int64)
    n_tot = int(np.sum(lens))
    small = oracle.HostCache.from_arrays(oracle.Shape(1, 1, len(sample), len(sample) * G, D), np.concatenate(rows_k), np.concatenate(rows_v),
                                         np.zeros(n_tot, np.float32), np.zeros(n_tot, np.int32), starts, np.array(lens, np.int32))
    ref, lse_ref = oracle.attend(small, np.concatenate(qs), st.scale)
    assert attn_error(np.concatenate(outs), ref[0, 0]) <= ATTN_TOL
    assert np.abs(np.concatenate(lses) - lse_ref[0, 0]).max() <= 2e-3


def test_fused_call_takes_the_two_stage_path_when_the_source_has_too_many_chunks():
    # A source cache of more than 524288 chunks of 128 entries (67 M entries of capacity) does not fit the fused
    # kernel's per-chunk partial results: kvtrim_compact_attn then runs the two stages one after the other.  The
    # destination has a quarter of the source's capacity, so it is this limit and not the "few survivors" rule that
    # decides.  Few entries are live, so the oracle compares everything.
    w = ki.Workload("big", 0, 1, 2, 2, 8, 128, (0,), (0,), 1, 3.0, 1.5)
    seg_len = [5000, 0, 3333, 129]
    c, now = ki.ragged_cache(w, seg_len, reserve=1, salt=4)
    n_small = c["cap"]
    cap = 524288 * 128 + 4096
    big = kv.Cache.empty(w.nseg, w.head_dim, cap, DEV)
    for name in ("k", "v", "log_beta", "pos"):
        getattr(big, name)[:n_small].copy_(c[name])
    big.seg_start.copy_(c["seg_start"])
    big.seg_len.copy_(c["seg_len"])
    dst = kv.Cache.empty(w.nseg, w.head_dim, cap // 4 + 8, DEV)
    ctx = kv.Context(1, 2, 2, 8, 128, cap)
    score = torch.zeros(cap, dtype=torch.float32, device=DEV)
    keep = torch.zeros(cap, dtype=torch.uint8, device=DEV)
    kept = torch.zeros(w.nseg, dtype=torch.int32, device=DEV)
    thr = torch.zeros(1, dtype=torch.int32, device=DEV)
    budget = torch.tensor([6000], dtype=torch.int64, device=DEV)
    out = torch.zeros(1, 2, 8, 128, dtype=torch.float32, device=DEV)
    lse = torch.zeros(1, 2, 8, dtype=torch.float32, device=DEV)
    g = torch.Generator().manual_seed(3)
    q = torch.randn(1, 2, 8, 128, generator=g).to(torch.bfloat16)
    scale = 1.0 / math.sqrt(128)
    kv.kvtrim_score_select(ctx, big, now.to(DEV), budget, score, keep, kept, thr, evict_hint=0)
    kv.kvtrim_profile_begin(ctx, (1 << kv.binding.N_KERNELS) - 1)
    kv.kvtrim_compact_attn(ctx, big, keep, kept, dst, 1, q.to(DEV), 0, 2, scale, out, lse)
    prof = kv.kvtrim_profile_end(ctx)
    assert kv.kvtrim_poll_error(ctx) == 0
    assert "k_cmp_copy" in prof and "k_att_partial" in prof and "k_cmp_attn" not in prof, prof
    from helpers import host_cache
    hc = host_cache(w, c)
    s_ref = oracle.score(hc, now.numpy())
    keep_ref, kept_ref, thr_ref = oracle.select(hc, s_ref, np.array([6000], np.int64))
    hc2 = oracle.compact(hc, keep_ref, 6000 + 4 + 8, 1)
    out_ref, lse_ref = oracle.attend(hc2, bf16_bits(q), scale)
    assert np.array_equal(kept.cpu().numpy(), kept_ref) and np.array_equal(thr.cpu().numpy().view(np.uint32), thr_ref)
    assert np.array_equal(dst.seg_start.cpu().numpy(), hc2.seg_start) and np.array_equal(dst.seg_len.cpu().numpy(), hc2.seg_len)
    m = live_mask(hc2)
    n = hc2.cap
    assert np.array_equal(bf16_bits(dst.k[:n])[m], hc2.k[m]) and np.array_equal(bf16_bits(dst.v[:n])[m], hc2.v[m])
    assert np.array_equal(dst.pos[:n].cpu().numpy()[m], hc2.pos[m])
    assert attn_error(out.cpu().numpy(), out_ref) <= ATTN_TOL
    lse_gpu, fin = lse.cpu().numpy(), np.isfinite(lse_ref)
    assert np.array_equal(np.isneginf(lse_gpu), np.isneginf(lse_ref)) and np.abs(lse_gpu[fin] - lse_ref[fin]).max() <= 2e-3   # (one segment is empty)
