"""Runs the decode loop (append -> score -> select -> compact -> attend) through the C ABI on the
GPU and through the CPU oracle on the same generated inputs, and compares every stage."""
import math

import numpy as np
import torch

import kvtrim_inputs as ki
import oracle
import paper_2605_09649_amd as kv
from helpers import bf16_bits, host_cache, live_mask


def device_cache_to_host(w, dc):
    d = {n: getattr(dc, n) for n in ("k", "v", "log_beta", "pos", "seg_start", "seg_len", "log_tail")}
    return host_cache(w, d)


def compare_caches(hc_gpu, hc_ref):
    """Segment tables equal and every live entry bit-equal."""
    if not (np.array_equal(hc_gpu.seg_start, hc_ref.seg_start) and np.array_equal(hc_gpu.seg_len, hc_ref.seg_len)):
        return False
    m = live_mask(hc_ref)
    n = min(hc_gpu.cap, hc_ref.cap)
    if m[n:].any():
        return False
    m = m[:n]
    if (hc_gpu.log_tail is None) != (hc_ref.log_tail is None):
        return False
    if hc_ref.log_tail is not None and not np.array_equal(hc_gpu.log_tail[:n][m].view(np.uint32),
                                                          hc_ref.log_tail[:n][m].view(np.uint32)):
        return False
    return (np.array_equal(hc_gpu.k[:n][m], hc_ref.k[:n][m]) and np.array_equal(hc_gpu.v[:n][m], hc_ref.v[:n][m])
            and np.array_equal(hc_gpu.log_beta[:n][m].view(np.uint32), hc_ref.log_beta[:n][m].view(np.uint32))
            and np.array_equal(hc_gpu.pos[:n][m], hc_ref.pos[:n][m]))


def attn_error(out_gpu, out_ref):
    """max |o_gpu - o_ref| / max |o_ref| (the tolerance metric of the benchmark)."""
    denom = np.abs(out_ref).max()
    return float(np.abs(out_gpu.astype(np.float64) - out_ref).max() / (denom if denom > 0 else 1.0))


class GpuLoop:
    """Device-side state of the decode loop: ping-pong caches and the per-step scratch outputs."""

    def __init__(self, w, cache_dict, budget, reserve, extra_entries, device, fused=False, hint=None, one_call=False):
        self.w, self.device, self.reserve, self.fused, self.hint = w, device, reserve, fused, hint
        self.calls, self.one_call = 0, one_call
        self.src = kv.Cache.from_dict(cache_dict, device)
        total = int(cache_dict["seg_len"].sum())
        dst_cap = min(int(sum(budget)), total + extra_entries) + w.nseg * reserve + 8
        self.ctx = kv.Context(w.n_seq, w.n_layers, w.n_kv_heads, w.n_q_heads, w.head_dim,
                              max(self.src.cap, dst_cap))
        self.spare = [kv.Cache.empty(w.nseg, w.head_dim, dst_cap, device, with_tail=self.src.log_tail is not None)
                      for _ in range(2)]
        cap = max(self.src.cap, dst_cap)
        self.score = torch.zeros(cap, dtype=torch.float32, device=device)
        self.keep = torch.zeros(cap, dtype=torch.uint8, device=device)
        self.kept = torch.zeros(w.nseg, dtype=torch.int32, device=device)
        self.thr = torch.zeros(w.n_seq, dtype=torch.int32, device=device)
        self.budget = torch.tensor(list(budget), dtype=torch.int64, device=device)
        self.out = torch.zeros(w.n_seq, w.n_layers, w.n_q_heads, w.head_dim, dtype=torch.float32, device=device)
        self.lse = torch.zeros(w.n_seq, w.n_layers, w.n_q_heads, dtype=torch.float32, device=device)
        self.scale = 1.0 / math.sqrt(w.head_dim)
        self.flip = 0

    def step(self, inp, now_dev, pos_new_dev):
        ctx = self.ctx
        if self.one_call:                          # the whole step through kvtrim_decode_step
            hint = self.hint[min(self.calls, len(self.hint) - 1)] if isinstance(self.hint, (list, tuple)) else (self.hint or 0)
            self.calls += 1
            dst = self.spare[self.flip]
            kv.kvtrim_decode_step(ctx, self.src, inp["k_new"], inp["v_new"], inp["log_beta_new"], pos_new_dev, 1, now_dev,
                                  self.budget, self.score, self.keep, self.kept, dst, self.reserve, inp["q"], 0, self.w.n_layers,
                                  self.scale, self.out, self.lse, thr_key_out=self.thr, log_tail_new=inp.get("log_tail_new"),
                                  evict_hint=hint)
            return dst
        kv.kvtrim_append(ctx, self.src, inp["k_new"], inp["v_new"], inp["log_beta_new"], pos_new_dev, 1,
                         log_tail_new=inp.get("log_tail_new"))
        if self.hint is None:
            kv.kvtrim_score(ctx, self.src, now_dev, self.score)
            kv.kvtrim_select_global(ctx, self.src, self.score, self.budget, self.keep, self.kept, self.thr)
        else:                                      # stages 1 + 2 in one call (hint 0: radix passes; > 0: decode-step form)
            hint = self.hint[min(self.calls, len(self.hint) - 1)] if isinstance(self.hint, (list, tuple)) else self.hint
            self.calls += 1
            kv.kvtrim_score_select(ctx, self.src, now_dev, self.budget, self.score, self.keep, self.kept, self.thr,
                                   evict_hint=hint)
        dst = self.spare[self.flip]
        if self.fused:
            kv.kvtrim_compact_attn(ctx, self.src, self.keep, self.kept, dst, self.reserve, inp["q"], 0,
                                   self.w.n_layers, self.scale, self.out, self.lse)
        else:
            kv.kvtrim_compact(ctx, self.src, self.keep, self.kept, dst, self.reserve)
            kv.kvtrim_decode_attn(ctx, dst, inp["q"], 0, self.w.n_layers, self.scale, self.out, self.lse)
        return dst

    def advance(self, dst):
        if self.src is not self.spare[0] and self.src is not self.spare[1]:
            self.first = self.src                  # keep the prefill cache alive until the caller drops it
        self.src = dst
        self.flip ^= 1


def run_steps_both(w, steps, budget, device="cuda:0", reserve=1, cache_dict=None, now0=None, fused=False, horizon=1,
                   hint=None, budget_per_step=None, one_call=False):
    """Returns one dict per step with the comparison results.  hint: None = kvtrim_score + kvtrim_select_global,
    otherwise kvtrim_score_select with that evict_hint.  budget_per_step: a list of budgets, one per step."""
    if cache_dict is None:
        cache_dict = ki.prefill_cache(w, reserve=reserve)
        now0 = [t - 1 for t in w.prefill]
    cache_dict = ki.with_horizon(cache_dict, horizon)
    hc = host_cache(w, cache_dict)
    gpu = GpuLoop(w, cache_dict, budget, reserve, steps * w.nseg, device, fused=fused, hint=hint, one_call=one_call)
    budget_np = np.array(list(budget), np.int64)
    now = np.array(now0, np.int32)
    per_seq = w.n_layers * w.n_kv_heads
    results = []
    for step in range(steps):
        if budget_per_step is not None:
            budget_np = np.array(list(budget_per_step[step]), np.int64)
            gpu.budget.copy_(torch.from_numpy(budget_np))
        inp = ki.decode_inputs(w, step, horizon=horizon)
        now = now + 1
        pos_new = np.repeat(now, per_seq).astype(np.int32)
        # ---- oracle
        oracle.append(hc, bf16_bits(inp["k_new"]), bf16_bits(inp["v_new"]), inp["log_beta_new"].numpy(), pos_new,
                      log_tail_new=None if horizon == 1 else inp["log_tail_new"].numpy())
        score_ref = oracle.score(hc, now)
        keep_ref, kept_ref, thr_ref = oracle.select(hc, score_ref, budget_np)
        dst_cap = gpu.spare[0].cap
        hc_next = oracle.compact(hc, keep_ref, dst_cap, reserve)
        out_ref, lse_ref = oracle.attend(hc_next, bf16_bits(inp["q"]), gpu.scale)
        # ---- GPU through the C ABI
        inp_dev = {k: v.to(device) for k, v in inp.items()}
        dst = gpu.step(inp_dev, torch.from_numpy(now).to(device), torch.from_numpy(pos_new).to(device))
        status = kv.kvtrim_poll_error(gpu.ctx)
        live = live_mask(hc)
        n = hc.cap
        score_gpu = gpu.score[:n].cpu().numpy()
        keep_gpu = gpu.keep[:n].cpu().numpy()
        res = {
            "status": status,
            "score_equal": bool(np.array_equal(score_gpu[live].view(np.uint32), score_ref[live].view(np.uint32))),
            "keep_equal": bool(np.array_equal(keep_gpu[live], keep_ref[live])
                               and np.array_equal(gpu.kept.cpu().numpy(), kept_ref)
                               and np.array_equal(gpu.thr.cpu().numpy().view(np.uint32), thr_ref)),
            "cache_equal": compare_caches(device_cache_to_host(w, dst), hc_next),
            "attn_err": attn_error(gpu.out.cpu().numpy(), out_ref),
            "kept_total": int(kept_ref.sum()),
        }
        if one_call:                               # the source cache afterwards: the new token is in it
            res["src_equal"] = bool(compare_cache_contents(device_cache_to_host(w, gpu.src), hc)) and \
                bool(np.array_equal(gpu.src.seg_len.cpu().numpy(), hc.seg_len))
        if hint is not None:
            res["path_counts"] = kv.kvtrim_select_path_counts(gpu.ctx)
        fin = np.isfinite(lse_ref)
        lse_gpu = gpu.lse.cpu().numpy()
        res["lse_err"] = float(np.abs(lse_gpu[fin] - lse_ref[fin]).max()) if fin.any() else 0.0
        res["lse_inf_equal"] = bool(np.array_equal(np.isneginf(lse_gpu), np.isneginf(lse_ref)))
        results.append(res)
        gpu.advance(dst)
        hc = hc_next
    return results


def run_multiturn_both(w, lengths, chunk, decode_per_turn, budget, device="cuda:0", turns=4, fused=True,
                       one_call_chunks=False):
    """The chunked multi-turn flow: every sequence's tokens are split into `turns` turns; a turn appends its tokens
    in chunks of `chunk` (sequences run out at different times: their rows are padded with negative positions) and
    after every chunk the cache is rescored, selected and compacted (no attention); then `decode_per_turn` tokens
    are decoded with full steps.  Both sides start from empty caches.  Returns one dict of findings per call group.
    one_call_chunks: the GPU side runs a chunk through kvtrim_append_compact instead of the four calls."""
    per_seq = w.n_layers * w.n_kv_heads
    S, nseg, D = w.n_seq, w.nseg, w.head_dim
    reserve = chunk                                                # room behind every segment for the next chunk
    cap = sum(min(int(budget[s]), (lengths[s] + turns * decode_per_turn) * per_seq) for s in range(S)) + nseg * reserve + chunk * nseg + 8
    shape = oracle.Shape(w.n_seq, w.n_layers, w.n_kv_heads, w.n_q_heads, w.head_dim)
    starts = np.arange(nseg, dtype=np.int64) * reserve
    hc = oracle.HostCache(shape, cap)
    hc.seg_start[:] = starts
    caches = [kv.Cache.empty(nseg, D, cap, device) for _ in range(2)]
    caches[0].seg_start.copy_(torch.from_numpy(starts))
    cur, flip = caches[0], 1
    ctx = kv.Context(w.n_seq, w.n_layers, w.n_kv_heads, w.n_q_heads, D, cap)
    score = torch.zeros(cap, dtype=torch.float32, device=device)
    keep = torch.zeros(cap, dtype=torch.uint8, device=device)
    kept = torch.zeros(nseg, dtype=torch.int32, device=device)
    thr = torch.zeros(S, dtype=torch.int32, device=device)
    budget_np = np.array(list(budget), np.int64)
    budget_dev = torch.from_numpy(budget_np).to(device)
    out = torch.zeros(S, w.n_layers, w.n_q_heads, D, dtype=torch.float32, device=device)
    lse = torch.zeros(S, w.n_layers, w.n_q_heads, dtype=torch.float32, device=device)
    scale = 1.0 / math.sqrt(D)
    next_pos = np.zeros(S, np.int64)                               # position of the next token of each sequence
    results = []

    def select_compact(pos_new, n_new, inp, attend_q, label):
        nonlocal hc, cur, flip
        now = (next_pos - 1).astype(np.int32)
        # ---- oracle
        oracle.append(hc, bf16_bits(inp["k_new"]), bf16_bits(inp["v_new"]), inp["log_beta_new"].numpy(), pos_new)
        s_ref = oracle.score(hc, now)
        k_ref, kept_ref, thr_ref = oracle.select(hc, s_ref, budget_np)
        hc_next = oracle.compact(hc, k_ref, cap, reserve)
        # ---- GPU
        d = {k: v.to(device) for k, v in inp.items()}
        dst = caches[flip]
        res = {"what": label}
        one_call = attend_q is None and one_call_chunks
        if one_call:
            kv.kvtrim_append_compact(ctx, cur, d["k_new"], d["v_new"], d["log_beta_new"], torch.from_numpy(pos_new).to(device),
                                     n_new, torch.from_numpy(now).to(device), budget_dev, score, keep, kept, dst, reserve,
                                     thr_key_out=thr)
        else:
            kv.kvtrim_append(ctx, cur, d["k_new"], d["v_new"], d["log_beta_new"], torch.from_numpy(pos_new).to(device), n_new)
            kv.kvtrim_score(ctx, cur, torch.from_numpy(now).to(device), score)
            kv.kvtrim_select_global(ctx, cur, score, budget_dev, keep, kept, thr)
        if one_call:
            pass
        elif attend_q is None:
            kv.kvtrim_compact(ctx, cur, keep, kept, dst, reserve)
        elif fused:
            kv.kvtrim_compact_attn(ctx, cur, keep, kept, dst, reserve, attend_q.to(device), 0, w.n_layers, scale, out, lse)
        else:
            kv.kvtrim_compact(ctx, cur, keep, kept, dst, reserve)
            kv.kvtrim_decode_attn(ctx, dst, attend_q.to(device), 0, w.n_layers, scale, out, lse)
        res["status"] = kv.kvtrim_poll_error(ctx)
        live = live_mask(hc)
        res["score_equal"] = bool(np.array_equal(score[:cap].cpu().numpy()[live].view(np.uint32), s_ref[live].view(np.uint32)))
        res["keep_equal"] = bool(np.array_equal(keep[:cap].cpu().numpy()[live], k_ref[live])
                                 and np.array_equal(kept.cpu().numpy(), kept_ref)
                                 and np.array_equal(thr.cpu().numpy().view(np.uint32), thr_ref))
        res["cache_equal"] = compare_caches(device_cache_to_host(w, dst), hc_next)
        res["entries"] = int(kept_ref.sum())
        if attend_q is not None:
            out_ref, lse_ref = oracle.attend(hc_next, bf16_bits(attend_q), scale)
            res["attn_err"] = attn_error(out.cpu().numpy(), out_ref)
            fin = np.isfinite(lse_ref)
            res["lse_err"] = float(np.abs(lse.cpu().numpy()[fin] - lse_ref[fin]).max()) if fin.any() else 0.0
        results.append(res)
        hc, cur, flip = hc_next, dst, flip ^ 1

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
            select_compact(pos_new, chunk, ki.chunk_inputs(w, chunk, "cpu", t, c), None, f"turn {t} chunk {c}")
            c += 1
        for dstep in range(decode_per_turn):
            inp = ki.decode_inputs(w, t * 1000 + dstep)
            pos_new = np.repeat(next_pos, per_seq).astype(np.int32).reshape(nseg, 1)
            next_pos += 1
            q = inp.pop("q")
            select_compact(pos_new, 1, inp, q, f"turn {t} decode {dstep}")
    return results


def compare_cache_contents(hc_gpu, hc_ref):
    """Segment lengths equal and the live entries, taken segment by segment, bit-equal - whatever the segment starts
    are (a cache compacted in place keeps its starts, the oracle packs its segments)."""
    if not np.array_equal(hc_gpu.seg_len, hc_ref.seg_len):
        return False
    mg, mr = live_mask(hc_gpu), live_mask(hc_ref)
    if (hc_gpu.log_tail is None) != (hc_ref.log_tail is None):
        return False
    if hc_ref.log_tail is not None and not np.array_equal(hc_gpu.log_tail[mg].view(np.uint32), hc_ref.log_tail[mr].view(np.uint32)):
        return False
    return (np.array_equal(hc_gpu.k[mg], hc_ref.k[mr]) and np.array_equal(hc_gpu.v[mg], hc_ref.v[mr])
            and np.array_equal(hc_gpu.log_beta[mg].view(np.uint32), hc_ref.log_beta[mr].view(np.uint32))
            and np.array_equal(hc_gpu.pos[mg], hc_ref.pos[mr]))


def run_steps_inplace_both(w, steps, budget, room, cache_dict, now0, device="cuda:0", horizon=1, rebalance_at=(),
                           two_call=False, rebalance_room=None, one_call=False, hint=0):
    """The decode loop with stages 3 + 4 done inside the cache (kvtrim_compact_attn_inplace): `cache_dict` must leave
    `room` free slots behind every segment (one is used per step).  At the steps listed in `rebalance_at` the GPU
    side runs the out-of-place fused call instead, into a second cache with `room` free slots per segment again
    (`rebalance_room(step)` slots if given: a budget that evicts nothing leaves no space to restore the whole room).
    two_call: stage 3 alone in place (kvtrim_compact_inplace), then kvtrim_decode_attn on the same cache.
    one_call: the whole step through kvtrim_decode_step_inplace (kvtrim_decode_step at the rebalancing steps) with
    evict_hint `hint`.
    The oracle runs its four stages; scores, mask, counts, threshold, segment contents and attention are compared."""
    cache_dict = ki.with_horizon(cache_dict, horizon)
    hc = host_cache(w, cache_dict)
    cur = kv.Cache.from_dict(cache_dict, device)
    cap = cur.cap
    other = kv.Cache.empty(w.nseg, w.head_dim, cap, device, with_tail=cur.log_tail is not None)
    ctx = kv.Context(w.n_seq, w.n_layers, w.n_kv_heads, w.n_q_heads, w.head_dim, cap)
    score = torch.zeros(cap, dtype=torch.float32, device=device)
    keep = torch.zeros(cap, dtype=torch.uint8, device=device)
    kept = torch.zeros(w.nseg, dtype=torch.int32, device=device)
    thr = torch.zeros(w.n_seq, dtype=torch.int32, device=device)
    budget_np = np.array(list(budget), np.int64)
    budget_dev = torch.from_numpy(budget_np).to(device)
    out = torch.zeros(w.n_seq, w.n_layers, w.n_q_heads, w.head_dim, dtype=torch.float32, device=device)
    lse = torch.zeros(w.n_seq, w.n_layers, w.n_q_heads, dtype=torch.float32, device=device)
    scale = 1.0 / math.sqrt(w.head_dim)
    now = np.array(now0, np.int32)
    per_seq = w.n_layers * w.n_kv_heads
    results = []
    for step in range(steps):
        inp = ki.decode_inputs(w, step, horizon=horizon)
        now = now + 1
        pos_new = np.repeat(now, per_seq).astype(np.int32)
        oracle.append(hc, bf16_bits(inp["k_new"]), bf16_bits(inp["v_new"]), inp["log_beta_new"].numpy(), pos_new,
                      log_tail_new=None if horizon == 1 else inp["log_tail_new"].numpy())
        score_ref = oracle.score(hc, now)
        keep_ref, kept_ref, thr_ref = oracle.select(hc, score_ref, budget_np)
        hc_next = oracle.compact(hc, keep_ref, cap, 1)             # (the oracle packs its segments; one slot for the next token)
        out_ref, lse_ref = oracle.attend(hc_next, bf16_bits(inp["q"]), scale)
        d = {k: v.to(device) for k, v in inp.items()}
        if one_call:
            before = device_cache_to_host(w, cur)
            before.seg_len = before.seg_len + 1                    # the layout the scores and the mask refer to
            live_gpu = live_mask(before)
            args = (d["k_new"], d["v_new"], d["log_beta_new"], torch.from_numpy(pos_new).to(device), 1,
                    torch.from_numpy(now).to(device), budget_dev, score, keep, kept)
            if step in rebalance_at:
                kv.kvtrim_decode_step(ctx, cur, *args, other, room if rebalance_room is None else rebalance_room(step),
                                      d["q"], 0, w.n_layers, scale, out, lse, thr_key_out=thr,
                                      log_tail_new=d.get("log_tail_new"), evict_hint=hint)
                cur, other = other, cur
            else:
                kv.kvtrim_decode_step_inplace(ctx, cur, *args, other, d["q"], 0, w.n_layers, scale, out, lse, thr_key_out=thr,
                                              log_tail_new=d.get("log_tail_new"), evict_hint=hint)
            score_gpu, keep_gpu = score.cpu().numpy(), keep.cpu().numpy()
        else:
            kv.kvtrim_append(ctx, cur, d["k_new"], d["v_new"], d["log_beta_new"], torch.from_numpy(pos_new).to(device), 1,
                             log_tail_new=d.get("log_tail_new"))
            kv.kvtrim_score(ctx, cur, torch.from_numpy(now).to(device), score)
            kv.kvtrim_select_global(ctx, cur, score, budget_dev, keep, kept, thr)
            live_gpu = live_mask(device_cache_to_host(w, cur))     # the GPU cache's own layout, after the append
            score_gpu, keep_gpu = score.cpu().numpy(), keep.cpu().numpy()
        if one_call:
            pass
        elif step in rebalance_at:
            kv.kvtrim_compact_attn(ctx, cur, keep, kept, other, room if rebalance_room is None else rebalance_room(step),
                                   d["q"], 0, w.n_layers, scale, out, lse)
            cur, other = other, cur
        elif two_call:
            kv.kvtrim_compact_inplace(ctx, cur, keep, kept, other)
            kv.kvtrim_decode_attn(ctx, cur, d["q"], 0, w.n_layers, scale, out, lse)
        else:
            kv.kvtrim_compact_attn_inplace(ctx, cur, keep, kept, other, d["q"], 0, w.n_layers, scale, out, lse)
        res = {"status": kv.kvtrim_poll_error(ctx), "in_place": step not in rebalance_at}
        live_ref = live_mask(hc)
        res["score_equal"] = bool(np.array_equal(score_gpu[live_gpu].view(np.uint32), score_ref[live_ref].view(np.uint32)))
        res["keep_equal"] = bool(np.array_equal(keep_gpu[live_gpu], keep_ref[live_ref])
                                 and np.array_equal(kept.cpu().numpy(), kept_ref)
                                 and np.array_equal(thr.cpu().numpy().view(np.uint32), thr_ref))
        hg = device_cache_to_host(w, cur)
        res["cache_equal"] = compare_cache_contents(hg, hc_next)
        res["starts_kept"] = True
        res["attn_err"] = attn_error(out.cpu().numpy(), out_ref)
        fin = np.isfinite(lse_ref)
        lse_gpu = lse.cpu().numpy()
        res["lse_err"] = float(np.abs(lse_gpu[fin] - lse_ref[fin]).max()) if fin.any() else 0.0
        res["lse_inf_equal"] = bool(np.array_equal(np.isneginf(lse_gpu), np.isneginf(lse_ref)))
        res["moved_chunks"] = int((keep_ref[live_ref] == 0).sum())
        results.append(res)
        hc = hc_next
    return results


def pick_segments(w, kept, n_random=8, seed=7):
    """Segments to look at row by row: a few at random plus, for the first and the last sequence, the longest and
    the shortest non-empty segment after the step (different sequences, extreme lengths)."""
    rng = np.random.default_rng(seed)
    per_seq = w.n_layers * w.n_kv_heads
    pick = set(int(x) for x in rng.choice(w.nseg, min(n_random, w.nseg), replace=False))
    for s in sorted({0, w.n_seq - 1}):
        ks = kept[s * per_seq:(s + 1) * per_seq]
        pick.add(s * per_seq + int(np.argmax(ks)))
        nz = np.nonzero(ks)[0]
        if len(nz):
            pick.add(s * per_seq + int(nz[np.argmin(ks[nz])]))
    return sorted(pick)


def sampled_step_check(w, src, now, budget_np, reserve, gpu, q=None, scale=None, n_random=8, seed=7, new_rows=None,
                       in_place_starts=None):
    """One step at a size where the K/V rows cannot all go to the host: the oracle scores and selects on the metadata
    alone (compared WHOLE: score bits, mask, per-segment counts, threshold keys), the destination's segment table and
    per-entry metadata are compared WHOLE, K/V rows and the attention output on sampled segments.

    src: the device cache the step selected on, after the append (its metadata holds the new tokens).
    gpu: dict with the GPU's results - score, keep, kept, thr and, optionally, dst (device cache), out, lse.
    new_rows: (k_new, v_new, n_new, old_len) when the rows of a segment's entries from old_len[g] on are in the
      caller's new-token buffers and not in src (kvtrim_append_compact).
    in_place_starts: segment starts of the destination when it was compacted in place (else the tight table).
    Returns a dict of findings; everything that should be True / small is under its own key."""
    D, G = w.head_dim, w.group
    sh = oracle.Shape(w.n_seq, w.n_layers, w.n_kv_heads, w.n_q_heads, D)
    empty = np.zeros((0, D), np.uint16)
    meta = oracle.HostCache.from_arrays(sh, empty, empty, src.log_beta.cpu().numpy(), src.pos.cpu().numpy(),
                                        src.seg_start.cpu().numpy(), src.seg_len.cpu().numpy(),
                                        log_tail=None if src.log_tail is None else src.log_tail.cpu().numpy())
    score_ref = oracle.score(meta, np.asarray(now, np.int32))
    keep_ref, kept_ref, thr_ref = oracle.select(meta, score_ref, np.asarray(budget_np, np.int64))
    live = live_mask(meta)
    n = meta.cap
    res = {
        "score_equal": bool(np.array_equal(gpu["score"][:n].cpu().numpy()[live].view(np.uint32), score_ref[live].view(np.uint32))),
        "keep_equal": bool(np.array_equal(gpu["keep"][:n].cpu().numpy()[live], keep_ref[live])),
        "kept_equal": bool(np.array_equal(gpu["kept"].cpu().numpy(), kept_ref)),
        "thr_equal": bool(np.array_equal(gpu["thr"].cpu().numpy().view(np.uint32), thr_ref)),
        "kept_total": int(kept_ref.sum()), "candidates": int(live.sum()),
    }
    dst = gpu.get("dst")
    if dst is None:
        return res
    if in_place_starts is None:
        exp_start = np.concatenate([[0], np.cumsum(kept_ref.astype(np.int64) + reserve)[:-1]])
    else:
        exp_start = np.asarray(in_place_starts, np.int64)
    res["tables_equal"] = bool(np.array_equal(dst.seg_start.cpu().numpy(), exp_start)
                               and np.array_equal(dst.seg_len.cpu().numpy(), kept_ref))
    sel = keep_ref.astype(bool) & live
    dlive = np.zeros(dst.cap, bool)
    for s, m in zip(exp_start, kept_ref):
        dlive[s:s + m] = True
    ok = (np.array_equal(dst.log_beta.cpu().numpy()[dlive].view(np.uint32), meta.log_beta[sel].view(np.uint32))
          and np.array_equal(dst.pos.cpu().numpy()[dlive], meta.pos[sel]))
    if meta.log_tail is not None:
        ok = ok and np.array_equal(dst.log_tail.cpu().numpy()[dlive].view(np.uint32), meta.log_tail[sel].view(np.uint32))
    res["metadata_equal"] = bool(ok)
    sample = pick_segments(w, kept_ref, n_random, seed)
    res["sampled_segments"] = sample
    rows_ok = True
    rows_k, rows_v, lens, qs, out_rows, lse_rows = [], [], [], [], [], []
    dev = dst.k.device
    for g in sample:
        s0, ln = int(meta.seg_start[g]), int(meta.seg_len[g])
        m = keep_ref[s0:s0 + ln].astype(bool)
        idx = np.nonzero(m)[0]
        if new_rows is None:
            ii = torch.from_numpy(s0 + idx).to(dev)
            ks, vs = bf16_bits(src.k[ii]), bf16_bits(src.v[ii])
        else:                                      # rows from old_len[g] on are in the caller's buffers
            k_new, v_new, n_new, old_len = new_rows
            old = idx[idx < old_len[g]]
            new = idx[idx >= old_len[g]] - int(old_len[g])
            io = torch.from_numpy(s0 + old).to(dev)
            inn = torch.from_numpy(g * n_new + new).to(dev)
            ks = np.concatenate([bf16_bits(src.k[io]), bf16_bits(k_new.reshape(-1, D)[inn])])
            vs = np.concatenate([bf16_bits(src.v[io]), bf16_bits(v_new.reshape(-1, D)[inn])])
        d0, dn = int(exp_start[g]), int(kept_ref[g])
        rows_ok = rows_ok and np.array_equal(bf16_bits(dst.k[d0:d0 + dn]), ks) and np.array_equal(bf16_bits(dst.v[d0:d0 + dn]), vs)
        rows_k.append(ks)
        rows_v.append(vs)
        lens.append(dn)
    res["rows_equal"] = bool(rows_ok)
    if q is not None:
        q_host = bf16_bits(q).reshape(w.n_seq, w.n_layers, w.n_q_heads, D)
        out_gpu = gpu["out"].cpu().numpy()
        lse_gpu = gpu["lse"].cpu().numpy()
        per_seq = w.n_layers * w.n_kv_heads
        for g in sample:
            seq, lh = divmod(g, per_seq)
            layer, head = divmod(lh, w.n_kv_heads)
            qs.append(q_host[seq, layer, head * G:(head + 1) * G])
            out_rows.append(out_gpu[seq, layer, head * G:(head + 1) * G])
            lse_rows.append(lse_gpu[seq, layer, head * G:(head + 1) * G])
        starts = np.concatenate([[0], np.cumsum(lens)[:-1]]).astype(np.int64)
        n_tot = int(np.sum(lens))
        small_shape = oracle.Shape(1, 1, len(sample), len(sample) * G, D)
        small = oracle.HostCache.from_arrays(small_shape, np.concatenate(rows_k).reshape(-1, D), np.concatenate(rows_v).reshape(-1, D),
                                             np.zeros(n_tot, np.float32), np.zeros(n_tot, np.int32), starts, np.array(lens, np.int32))
        ref, lse_ref = oracle.attend(small, np.concatenate(qs), scale)
        res["attn_err"] = attn_error(np.concatenate(out_rows), ref[0, 0])
        lr, lg = lse_ref[0, 0], np.concatenate(lse_rows)
        fin = np.isfinite(lr)
        res["lse_err"] = float(np.abs(lg[fin] - lr[fin]).max()) if fin.any() else 0.0
    return res
