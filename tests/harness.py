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

    def __init__(self, w, cache_dict, budget, reserve, extra_entries, device, fused=False):
        self.w, self.device, self.reserve, self.fused = w, device, reserve, fused
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
        kv.kvtrim_append(ctx, self.src, inp["k_new"], inp["v_new"], inp["log_beta_new"], pos_new_dev, 1,
                         log_tail_new=inp.get("log_tail_new"))
        kv.kvtrim_score(ctx, self.src, now_dev, self.score)
        kv.kvtrim_select_global(ctx, self.src, self.score, self.budget, self.keep, self.kept, self.thr)
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


def run_steps_both(w, steps, budget, device="cuda:0", reserve=1, cache_dict=None, now0=None, fused=False, horizon=1):
    """Returns one dict per step with the comparison results."""
    if cache_dict is None:
        cache_dict = ki.prefill_cache(w, reserve=reserve)
        now0 = [t - 1 for t in w.prefill]
    cache_dict = ki.with_horizon(cache_dict, horizon)
    hc = host_cache(w, cache_dict)
    gpu = GpuLoop(w, cache_dict, budget, reserve, steps * w.nseg, device, fused=fused)
    budget_np = np.array(list(budget), np.int64)
    now = np.array(now0, np.int32)
    per_seq = w.n_layers * w.n_kv_heads
    results = []
    for step in range(steps):
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
        fin = np.isfinite(lse_ref)
        lse_gpu = gpu.lse.cpu().numpy()
        res["lse_err"] = float(np.abs(lse_gpu[fin] - lse_ref[fin]).max()) if fin.any() else 0.0
        res["lse_inf_equal"] = bool(np.array_equal(np.isneginf(lse_gpu), np.isneginf(lse_ref)))
        results.append(res)
        gpu.advance(dst)
        hc = hc_next
    return results
