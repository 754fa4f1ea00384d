"""Runs the decode loop on the paged layout (append -> score -> select -> evict -> attend, no K/V
moved) through the C ABI on the GPU, next to the CPU oracle's ragged loop on the same inputs.

A paged segment holds its entries in no particular order, so the comparison goes through the
positions (unique inside a segment): the live slots of every segment, sorted by position, must be
the oracle's segment entry for entry, bit for bit."""
import math

import numpy as np
import torch

import kvtrim_inputs as ki
import oracle
import paper_2605_09649_amd as kv
from harness import attn_error
from helpers import bf16_bits, host_cache, live_mask

P = kv.PAGE_SIZE


class PagedHost:
    """Host copy of the bookkeeping (and, on request, the rows) of a paged cache."""

    def __init__(self, pc, rows=True):
        self.n_pages, self.max_pps, self.nseg = pc.n_pages, pc.max_pages_per_seg, pc.nseg
        self.bt = pc.block_table.cpu().numpy()
        self.seg_pages = pc.seg_pages.cpu().numpy()
        self.seg_live = pc.seg_live.cpu().numpy()
        self.owner = pc.page_owner.cpu().numpy()
        self.page_live = pc.page_live.cpu().numpy()
        self.free_list = pc.free_list.cpu().numpy()
        self.n_free = int(pc.n_free.cpu().numpy()[0])
        self.pos = pc.pos.cpu().numpy()
        self.log_beta = pc.log_beta.cpu().numpy()
        self.log_tail = None if pc.log_tail is None else pc.log_tail.cpu().numpy()
        if rows:
            self.k, self.v = bf16_bits(pc.k), bf16_bits(pc.v)

    def structure_problems(self):
        """Everything that must hold between two calls, as a list of findings (empty = fine)."""
        bad = []
        sp = self.seg_pages
        if (sp < 0).any() or (sp > self.max_pps).any():
            return ["seg_pages out of range"]
        live_slots = (self.pos.reshape(self.n_pages, P) >= 0).sum(1)
        seen = np.full(self.n_pages, -1, np.int64)
        for g in range(self.nseg):
            pages = self.bt[g, :sp[g]]
            if (pages < 0).any() or (pages >= self.n_pages).any():
                bad.append(f"segment {g}: page id out of range")
                continue
            if (seen[pages] >= 0).any() or len(np.unique(pages)) != len(pages):
                bad.append(f"segment {g}: page listed twice")
            seen[pages] = g
            if (self.owner[pages] != g).any():
                bad.append(f"segment {g}: owner mismatch")
            if (live_slots[pages] < 1).any():
                bad.append(f"segment {g}: empty page in the table")
            if int(live_slots[pages].sum()) != int(self.seg_live[g]):
                bad.append(f"segment {g}: seg_live {self.seg_live[g]} != {int(live_slots[pages].sum())}")
        if not np.array_equal(self.page_live[seen >= 0], live_slots[seen >= 0]):
            bad.append("page_live differs from the slots")
        free = np.flatnonzero(seen < 0)
        if (self.owner[free] != -1).any() or (self.page_live[free] != 0).any() or (live_slots[free] != 0).any():
            bad.append("free page with an owner or live slots")
        if self.n_free != len(free):
            bad.append(f"n_free {self.n_free} != {len(free)}")
        elif not np.array_equal(np.sort(self.free_list[:self.n_free]), free):
            bad.append("free list differs from the set of free pages")
        return bad

    def ordered_slots(self):
        """Live slots of all segments, segment by segment, each sorted by position; and counts."""
        idx, counts = [], []
        lane = np.arange(P, dtype=np.int64)[None, :]
        for g in range(self.nseg):
            pages = self.bt[g, :self.seg_pages[g]].astype(np.int64)
            slots = (pages[:, None] * P + lane).ravel()
            slots = slots[self.pos[slots] >= 0]
            slots = slots[np.argsort(self.pos[slots], kind="stable")]
            idx.append(slots)
            counts.append(len(slots))
        return (np.concatenate(idx) if idx else np.zeros(0, np.int64)), np.array(counts, np.int32)

    def as_ragged(self, shape, reserve=1):
        """The same entries as the oracle's ragged cache: every segment in position order, each
        followed by `reserve` free slots."""
        idx, counts = self.ordered_slots()
        starts = np.concatenate([[0], np.cumsum(counts.astype(np.int64) + reserve)[:-1]]).astype(np.int64)
        at = np.concatenate([st + np.arange(n) for st, n in zip(starts, counts)]) if len(idx) else idx
        n_host = int(counts.sum()) + reserve * self.nseg

        def spread(a):
            o = np.zeros((n_host,) + a.shape[1:], a.dtype)
            o[at] = a[idx]
            return o
        return oracle.HostCache.from_arrays(shape, spread(self.k), spread(self.v), spread(self.log_beta),
                                            spread(self.pos), starts, counts,
                                            log_tail=None if self.log_tail is None else spread(self.log_tail))

    def equals(self, hc):
        """Same entries per segment as the oracle's ragged cache hc."""
        idx, counts = self.ordered_slots()
        if not np.array_equal(counts, hc.seg_len):
            return False
        m = live_mask(hc)
        ok = (np.array_equal(self.pos[idx], hc.pos[m])
              and np.array_equal(self.log_beta[idx].view(np.uint32), hc.log_beta[m].view(np.uint32))
              and np.array_equal(self.k[idx], hc.k[m]) and np.array_equal(self.v[idx], hc.v[m]))
        if hc.log_tail is not None:
            ok = ok and self.log_tail is not None and np.array_equal(self.log_tail[idx].view(np.uint32),
                                                                      hc.log_tail[m].view(np.uint32))
        return bool(ok)


def attn_result(out_gpu, lse_gpu, out_ref, lse_ref):
    fin = np.isfinite(lse_ref)
    return {"attn_err": attn_error(out_gpu, out_ref),
            "lse_err": float(np.abs(lse_gpu[fin] - lse_ref[fin]).max()) if fin.any() else 0.0,
            "lse_inf_equal": bool(np.array_equal(np.isneginf(lse_gpu), np.isneginf(lse_ref)))}


def ties_overflow(w, hc, score_ref, live, thr_ref, budget_np):
    """True if in some sequence the entries at or above the threshold outnumber the budget, i.e.
    the ties at the threshold had to be ranked by (layer, head, position)."""
    per_seq = w.n_layers * w.n_kv_heads
    u = score_ref.view(np.uint32)
    key = np.where(u & np.uint32(0x80000000), ~u, u | np.uint32(0x80000000))
    seq_of = np.zeros(hc.cap, np.int64)
    for g, (s, n) in enumerate(zip(hc.seg_start, hc.seg_len)):
        seq_of[s:s + n] = g // per_seq
    for seq in range(w.n_seq):
        m = live & (seq_of == seq)
        if 0 < budget_np[seq] < int(m.sum()) and int((key[m] >= thr_ref[seq]).sum()) > int(budget_np[seq]):
            return True
    return False


def run_paged_both(w, budgets, device="cuda:0", cache_dict=None, now0=None, n_pages=None, max_pps=None, horizon=1,
                   tweak_new=None, defrag_at=(), hint=None, one_call=False, layer_range=None):
    """budgets: one per-sequence budget list per step; step 0 selects on the ragged prefill cache
    and builds the pages, the later steps run on the pages.  tweak_new(step, inputs) may edit the
    generated inputs of a step (used to plant ties).  In the steps listed in defrag_at the pages are
    defragmented between eviction and attention.  hint: None runs stages 1 and 2 on the pages as two calls,
    a number runs kvtrim_paged_score_select with that evict_hint.  one_call: the paged steps run
    kvtrim_paged_decode_step (append, score_select, evict and attention in one call; hint required).  layer_range
    (one_call only): the steps on the pages attend these layers only - their rows are compared, and the other rows of
    `out` and `lse` must stay as they were.  Returns one dict of findings per step."""
    reserve = 1
    if cache_dict is None:
        cache_dict = ki.prefill_cache(w, reserve=reserve)
        now0 = [t - 1 for t in w.prefill]
    cache_dict = ki.with_horizon(cache_dict, horizon)
    hc = host_cache(w, cache_dict)
    src = kv.Cache.from_dict(cache_dict, device)
    per_seq = w.n_layers * w.n_kv_heads
    steps = len(budgets)
    if n_pages is None:
        most = max(int(sum(b)) for b in budgets)
        n_pages = (min(most, int(cache_dict["seg_len"].sum()) + steps * w.nseg) + P - 1) // P + 2 * w.nseg + 8
    if max_pps is None:
        max_pps = n_pages
    slots = n_pages * P
    ctx = kv.Context(w.n_seq, w.n_layers, w.n_kv_heads, w.n_q_heads, w.head_dim, max(src.cap, slots))
    pc = kv.PagedCache(w.nseg, w.head_dim, n_pages, max_pps, device, with_tail=horizon != 1)
    cap = max(src.cap, slots)
    score = torch.zeros(cap, dtype=torch.float32, device=device)
    keep = torch.zeros(cap, dtype=torch.uint8, device=device)
    kept = torch.zeros(w.nseg, dtype=torch.int32, device=device)
    thr = torch.zeros(w.n_seq, dtype=torch.int32, device=device)
    out = torch.zeros(w.n_seq, w.n_layers, w.n_q_heads, w.head_dim, dtype=torch.float32, device=device)
    lse = torch.zeros(w.n_seq, w.n_layers, w.n_q_heads, dtype=torch.float32, device=device)
    scale = 1.0 / math.sqrt(w.head_dim)
    now = np.array(now0, np.int32)
    dst_cap = int(cache_dict["seg_len"].sum()) + (steps + reserve) * w.nseg + 8
    results = []
    for step in range(steps):
        inp = ki.decode_inputs(w, step, horizon=horizon)
        if tweak_new is not None:
            tweak_new(step, inp)
        now = now + 1
        pos_new = np.repeat(now, per_seq).astype(np.int32)
        budget_np = np.array(list(budgets[step]), np.int64)
        lt_new = None if horizon == 1 else inp["log_tail_new"]
        # ---- oracle: ragged loop
        oracle.append(hc, bf16_bits(inp["k_new"]), bf16_bits(inp["v_new"]), inp["log_beta_new"].numpy(), pos_new,
                      log_tail_new=None if lt_new is None else lt_new.numpy())
        score_ref = oracle.score(hc, now)
        keep_ref, kept_ref, thr_ref = oracle.select(hc, score_ref, budget_np)
        hc_next = oracle.compact(hc, keep_ref, dst_cap, reserve)
        out_ref, lse_ref = oracle.attend(hc_next, bf16_bits(inp["q"]), scale)
        live = live_mask(hc)
        # ---- GPU
        d = {k: v.to(device) for k, v in inp.items()}
        now_dev, pos_dev = torch.from_numpy(now).to(device), torch.from_numpy(pos_new).to(device)
        budget_dev = torch.from_numpy(budget_np).to(device)
        res = {"step": step}
        if step == 0:
            kv.kvtrim_append(ctx, src, d["k_new"], d["v_new"], d["log_beta_new"], pos_dev, 1,
                             log_tail_new=d.get("log_tail_new"))
            kv.kvtrim_score(ctx, src, now_dev, score)
            kv.kvtrim_select_global(ctx, src, score, budget_dev, keep, kept, thr)
            kv.kvtrim_paged_build(ctx, src, keep, kept, pc)
            res["score_equal"] = bool(np.array_equal(score[:hc.cap].cpu().numpy()[live].view(np.uint32),
                                                     score_ref[live].view(np.uint32)))
            res["keep_equal"] = bool(np.array_equal(keep[:hc.cap].cpu().numpy()[live], keep_ref[live]))
        elif one_call:
            pos_before = pc.pos.clone()
            lb, le = layer_range if layer_range is not None else (0, w.n_layers)
            if layer_range is not None:
                out.fill_(7.0)
                lse.fill_(7.0)
            kv.kvtrim_paged_decode_step(ctx, pc, d["k_new"], d["v_new"], d["log_beta_new"], pos_dev, now_dev, budget_dev, score, keep,
                                        kept, d["q"], lb, le, scale, out, lse, thr_key_out=thr,
                                        log_tail_new=d.get("log_tail_new"), evict_hint=hint)
            res["status_select"] = kv.kvtrim_poll_error(ctx)
            # the evicted slots are empty already: scores and mask are checked on the survivors (matched through their
            # positions) and the mask on the slots that were live before the call and are empty after it
            post = PagedHost(pc, rows=False)
            idx, counts = post.ordered_slots()
            kept_live = live & (keep_ref != 0)
            same = np.array_equal(counts, kept_ref)
            res["score_equal"] = bool(same and np.array_equal(score.cpu().numpy()[idx].view(np.uint32),
                                                              score_ref[kept_live].view(np.uint32)))
            gone = (pos_before.cpu().numpy().reshape(-1) >= 0) & (post.pos.reshape(-1) < 0)
            n_gone_ref = int(live.sum()) - int(kept_ref.sum())
            res["keep_equal"] = bool(same and np.all(keep.cpu().numpy()[idx] == 1) and not keep.cpu().numpy()[:gone.size][gone].any()
                                     and n_gone_ref - w.nseg <= int(gone.sum()) <= n_gone_ref)
        else:
            kv.kvtrim_paged_append(ctx, pc, d["k_new"], d["v_new"], d["log_beta_new"], pos_dev,
                                   log_tail_new=d.get("log_tail_new"))
            if hint is None:
                kv.kvtrim_paged_score(ctx, pc, now_dev, score)
                kv.kvtrim_paged_select(ctx, pc, score, budget_dev, keep, kept, thr)
            else:
                kv.kvtrim_paged_score_select(ctx, pc, now_dev, budget_dev, score, keep, kept, thr, evict_hint=hint)
            res["status_select"] = kv.kvtrim_poll_error(ctx)
            pre = PagedHost(pc, rows=False)
            res["structure_pre"] = pre.structure_problems()
            idx, counts = pre.ordered_slots()
            same = np.array_equal(counts, hc.seg_len)
            res["score_equal"] = bool(same and np.array_equal(score.cpu().numpy()[idx].view(np.uint32),
                                                              score_ref[live].view(np.uint32)))
            res["keep_equal"] = bool(same and np.array_equal(keep.cpu().numpy()[idx], keep_ref[live]))
            kv.kvtrim_paged_evict(ctx, pc, keep)
        if step in defrag_at:
            before = PagedHost(pc, rows=False)
            kv.kvtrim_paged_defrag(ctx, pc)
            after = PagedHost(pc, rows=False)
            res["defrag"] = {"pages_before": int(before.seg_pages.sum()), "pages_after": int(after.seg_pages.sum()),
                             "tight": bool(np.array_equal(after.seg_pages, (after.seg_live + P - 1) // P)),
                             "live_unchanged": bool(np.array_equal(before.seg_live, after.seg_live)),
                             "free_gain": after.n_free - before.n_free}
        if not (one_call and step > 0):
            kv.kvtrim_paged_attn(ctx, pc, d["q"], 0, w.n_layers, scale, out, lse)
        res["status"] = kv.kvtrim_poll_error(ctx)
        res["kept_equal"] = bool(np.array_equal(kept.cpu().numpy(), kept_ref)
                                 and np.array_equal(thr.cpu().numpy().view(np.uint32), thr_ref))
        ph = PagedHost(pc)
        res["structure"] = ph.structure_problems()
        res["cache_equal"] = ph.equals(hc_next)
        if one_call and step > 0 and layer_range is not None:
            lb, le = layer_range
            o, l = out.cpu().numpy(), lse.cpu().numpy()
            outside = [x for x in range(w.n_layers) if not lb <= x < le]
            res["untouched_outside_range"] = bool((o[:, outside] == 7.0).all() and (l[:, outside] == 7.0).all())
            res.update(attn_result(o[:, lb:le], l[:, lb:le], out_ref[:, lb:le], lse_ref[:, lb:le]))
        else:
            res.update(attn_result(out.cpu().numpy(), lse.cpu().numpy(), out_ref, lse_ref))
        res["kept_total"] = int(kept_ref.sum())
        res["pages_in_use"] = int(ph.seg_pages.sum())
        res["ties_overflow"] = ties_overflow(w, hc, score_ref, live, thr_ref, budget_np)
        res["path_counts"] = kv.kvtrim_select_path_counts(ctx)
        results.append(res)
        hc = hc_next
    return results


def run_multiturn_paged(w, lengths, chunk, decode_per_turn, budget, device="cuda:0", turns=4):
    """The chunked multi-turn flow on the paged layout: pages start empty; every turn appends each sequence's tokens
    in chunks (ragged last chunks padded with negative positions), with score + select + evict after every chunk,
    then decodes a few tokens with attention.  The oracle runs the same flow on its ragged cache."""
    per_seq = w.n_layers * w.n_kv_heads
    S, nseg, D = w.n_seq, w.nseg, w.head_dim
    live_bound = sum(min(int(budget[s]), (lengths[s] + turns * decode_per_turn) * per_seq) for s in range(S))
    n_pages = (live_bound + nseg * chunk) // P + 3 * nseg + 8
    cap = live_bound + 2 * nseg * chunk + 8
    shape = oracle.Shape(w.n_seq, w.n_layers, w.n_kv_heads, w.n_q_heads, w.head_dim)
    hc = oracle.HostCache(shape, cap)
    hc.seg_start[:] = np.arange(nseg, dtype=np.int64) * chunk
    ctx = kv.Context(w.n_seq, w.n_layers, w.n_kv_heads, w.n_q_heads, D, max(cap, n_pages * P))
    pc = kv.PagedCache(nseg, D, n_pages, n_pages, device)
    empty = kv.Cache.empty(nseg, D, 8, device)                     # pages are initialised from an empty ragged cache
    kv.kvtrim_paged_build(ctx, empty, torch.zeros(8, dtype=torch.uint8, device=device),
                          torch.zeros(nseg, dtype=torch.int32, device=device), pc)
    slots = n_pages * P
    score = torch.zeros(slots, dtype=torch.float32, device=device)
    keep = torch.zeros(slots, dtype=torch.uint8, device=device)
    kept = torch.zeros(nseg, dtype=torch.int32, device=device)
    thr = torch.zeros(S, dtype=torch.int32, device=device)
    budget_np = np.array(list(budget), np.int64)
    budget_dev = torch.from_numpy(budget_np).to(device)
    out = torch.zeros(S, w.n_layers, w.n_q_heads, D, dtype=torch.float32, device=device)
    lse = torch.zeros(S, w.n_layers, w.n_q_heads, dtype=torch.float32, device=device)
    scale = 1.0 / math.sqrt(D)
    next_pos = np.zeros(S, np.int64)
    results = []

    def one(pos_new, n_new, inp, attend_q, label):
        nonlocal hc
        now = (next_pos - 1).astype(np.int32)
        oracle.append(hc, bf16_bits(inp["k_new"]), bf16_bits(inp["v_new"]), inp["log_beta_new"].numpy(), pos_new)
        s_ref = oracle.score(hc, now)
        k_ref, kept_ref, thr_ref = oracle.select(hc, s_ref, budget_np)
        live = live_mask(hc)
        hc_next = oracle.compact(hc, k_ref, cap, chunk)
        d = {k: v.to(device) for k, v in inp.items()}
        kv.kvtrim_paged_append(ctx, pc, d["k_new"], d["v_new"], d["log_beta_new"], torch.from_numpy(pos_new).to(device),
                               n_new=n_new)
        kv.kvtrim_paged_score(ctx, pc, torch.from_numpy(now).to(device), score)
        kv.kvtrim_paged_select(ctx, pc, score, budget_dev, keep, kept, thr)
        res = {"what": label, "status_select": kv.kvtrim_poll_error(ctx)}
        pre = PagedHost(pc, rows=False)
        res["structure_pre"] = pre.structure_problems()
        idx, counts = pre.ordered_slots()
        same = np.array_equal(counts, hc.seg_len)
        res["score_equal"] = bool(same and np.array_equal(score.cpu().numpy()[idx].view(np.uint32), s_ref[live].view(np.uint32)))
        res["keep_equal"] = bool(same and np.array_equal(keep.cpu().numpy()[idx], k_ref[live]))
        kv.kvtrim_paged_evict(ctx, pc, keep)
        if attend_q is not None:
            kv.kvtrim_paged_attn(ctx, pc, attend_q.to(device), 0, w.n_layers, scale, out, lse)
        res["status"] = kv.kvtrim_poll_error(ctx)
        res["kept_equal"] = bool(np.array_equal(kept.cpu().numpy(), kept_ref)
                                 and np.array_equal(thr.cpu().numpy().view(np.uint32), thr_ref))
        ph = PagedHost(pc)
        res["structure"] = ph.structure_problems()
        res["cache_equal"] = ph.equals(hc_next)
        res["pages_in_use"] = int(ph.seg_pages.sum())
        if attend_q is not None:
            out_ref, lse_ref = oracle.attend(hc_next, bf16_bits(attend_q), scale)
            res.update(attn_result(out.cpu().numpy(), lse.cpu().numpy(), out_ref, lse_ref))
        results.append(res)
        hc = hc_next

    turn_len = [[(lengths[s] // turns) + (lengths[s] % turns if t == turns - 1 else 0) for t in range(turns)] for s in range(S)]
    for t in range(turns):
        left = np.array([turn_len[s][t] for s in range(S)], np.int64)
        c = 0
        while left.max() > 0:
            take = np.minimum(left, chunk)
            pos_new = np.full((nseg, chunk), -1, np.int32)
            for s in range(S):
                row = np.full(chunk, -1, np.int32)
                row[:take[s]] = next_pos[s] + np.arange(take[s])
                pos_new[s * per_seq:(s + 1) * per_seq] = row
            next_pos += take
            left -= take
            one(pos_new, chunk, ki.chunk_inputs(w, chunk, "cpu", t, c), None, f"turn {t} chunk {c}")
            c += 1
        for dstep in range(decode_per_turn):
            inp = ki.decode_inputs(w, t * 1000 + dstep)
            pos_new = np.repeat(next_pos, per_seq).astype(np.int32).reshape(nseg, 1)
            next_pos += 1
            q = inp.pop("q")
            one(pos_new, 1, inp, q, f"turn {t} decode {dstep}")
    return results
