"""The step calls only enqueue kernels on the caller's stream (no allocation, no synchronisation, no
memset), so a decode step can be captured into a HIP graph.  Captured steps are replayed several
times with fresh inputs, with eager work and synchronisations in between, and every replay must
reproduce the eager run of the same steps bit for bit (caches, selection, attention output)."""
import math

import numpy as np
import pytest
import torch

import kvtrim_inputs as ki
import paper_2605_09649_amd as kv
from paged_harness import PagedHost

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


class Loop:
    """Device state of one decode loop with static input buffers (so that a captured step finds its inputs at
    fixed addresses)."""

    def __init__(self, w, paged, inplace=False, calls="four"):
        self.w, self.paged, self.inplace, self.calls = w, paged, inplace, calls
        self.room = 8 if inplace else 1                           # free slots behind every segment after the first step
        pre = ki.prefill_cache(w, reserve=1)
        self.src = kv.Cache.from_dict(pre, DEV)
        total = int(pre["seg_len"].sum())
        B = sum(w.budget)
        cap = max(self.src.cap, B + 64 * w.nseg)
        self.ctx = kv.Context(w.n_seq, w.n_layers, w.n_kv_heads, w.n_q_heads, w.head_dim, cap)
        self.spare = [kv.Cache.empty(w.nseg, w.head_dim, B + (self.room + 1) * w.nseg + 8, DEV) for _ in range(2)]
        n_pages = (B + kv.PAGE_SIZE - 1) // kv.PAGE_SIZE + 3 * w.nseg + 8
        self.pc = kv.PagedCache(w.nseg, w.head_dim, n_pages, n_pages, DEV) if paged else None
        cap = max(cap, n_pages * kv.PAGE_SIZE)
        self.score = torch.zeros(cap, dtype=torch.float32, device=DEV)
        self.keep = torch.zeros(cap, dtype=torch.uint8, device=DEV)
        self.kept = torch.zeros(w.nseg, dtype=torch.int32, device=DEV)
        self.thr = torch.zeros(w.n_seq, dtype=torch.int32, device=DEV)
        self.budget = torch.tensor(list(w.budget), dtype=torch.int64, device=DEV)
        self.scale = 1.0 / math.sqrt(w.head_dim)
        # two sets of static inputs / outputs: a captured graph holds two consecutive steps
        self.inp = [{k: torch.zeros_like(v, device=DEV) for k, v in ki.decode_inputs(w, 0).items()} for _ in range(2)]
        self.now = [torch.zeros(w.n_seq, dtype=torch.int32, device=DEV) for _ in range(2)]
        self.pos = [torch.zeros(w.nseg, dtype=torch.int32, device=DEV) for _ in range(2)]
        self.out = [torch.zeros(w.n_seq, w.n_layers, w.n_q_heads, w.head_dim, dtype=torch.float32, device=DEV)
                    for _ in range(2)]
        self.flip = 0
        self.total = total

    def load_inputs(self, slot, step):
        w = self.w
        for k, v in ki.decode_inputs(w, step).items():
            self.inp[slot][k].copy_(v)
        now = np.array([t + step for t in w.prefill], np.int32)
        self.now[slot].copy_(torch.from_numpy(now))
        self.pos[slot].copy_(torch.from_numpy(np.repeat(now, w.n_layers * w.n_kv_heads).astype(np.int32)))

    def first_step(self):
        self.load_inputs(0, 0)
        i, ctx, w = self.inp[0], self.ctx, self.w
        kv.kvtrim_append(ctx, self.src, i["k_new"], i["v_new"], i["log_beta_new"], self.pos[0], 1)
        kv.kvtrim_score(ctx, self.src, self.now[0], self.score)
        kv.kvtrim_select_global(ctx, self.src, self.score, self.budget, self.keep, self.kept, self.thr)
        if self.paged:
            kv.kvtrim_paged_build(ctx, self.src, self.keep, self.kept, self.pc)
            kv.kvtrim_paged_attn(ctx, self.pc, i["q"], 0, w.n_layers, self.scale, self.out[0])
        else:
            kv.kvtrim_compact_attn(ctx, self.src, self.keep, self.kept, self.spare[0], self.room, i["q"], 0, w.n_layers,
                                   self.scale, self.out[0])
            self.cur, self.flip = self.spare[0], 1

    def step(self, slot):
        i, ctx, w = self.inp[slot], self.ctx, self.w
        if self.paged and self.calls == "paged_decode_step":
            kv.kvtrim_paged_decode_step(ctx, self.pc, i["k_new"], i["v_new"], i["log_beta_new"], self.pos[slot], self.now[slot],
                                        self.budget, self.score, self.keep, self.kept, i["q"], 0, w.n_layers, self.scale,
                                        self.out[slot], thr_key_out=self.thr, evict_hint=w.n_layers * w.n_kv_heads)
        elif self.paged:
            kv.kvtrim_paged_append(ctx, self.pc, i["k_new"], i["v_new"], i["log_beta_new"], self.pos[slot])
            kv.kvtrim_paged_score(ctx, self.pc, self.now[slot], self.score)
            kv.kvtrim_paged_select(ctx, self.pc, self.score, self.budget, self.keep, self.kept, self.thr)
            kv.kvtrim_paged_evict(ctx, self.pc, self.keep)
            kv.kvtrim_paged_attn(ctx, self.pc, i["q"], 0, w.n_layers, self.scale, self.out[slot])
        else:
            dst = self.spare[self.flip]
            hint = w.n_layers * w.n_kv_heads                      # evictions per sequence and step once at the budget
            if self.calls == "decode_step_inplace":               # the whole step in one call, inside the cache
                kv.kvtrim_decode_step_inplace(ctx, self.cur, i["k_new"], i["v_new"], i["log_beta_new"], self.pos[slot], 1,
                                              self.now[slot], self.budget, self.score, self.keep, self.kept, dst, i["q"], 0,
                                              w.n_layers, self.scale, self.out[slot], thr_key_out=self.thr, evict_hint=hint)
                return
            if self.calls == "decode_step":                       # the whole step in one call
                kv.kvtrim_decode_step(ctx, self.cur, i["k_new"], i["v_new"], i["log_beta_new"], self.pos[slot], 1, self.now[slot],
                                      self.budget, self.score, self.keep, self.kept, dst, 1, i["q"], 0, w.n_layers, self.scale,
                                      self.out[slot], thr_key_out=self.thr, evict_hint=hint)
                self.cur, self.flip = dst, self.flip ^ 1
                return
            kv.kvtrim_append(ctx, self.cur, i["k_new"], i["v_new"], i["log_beta_new"], self.pos[slot], 1)
            if self.calls == "score_select":                      # stages 1 + 2 in one call, decode-step form
                kv.kvtrim_score_select(ctx, self.cur, self.now[slot], self.budget, self.score, self.keep, self.kept, self.thr,
                                       evict_hint=hint)
            else:
                kv.kvtrim_score(ctx, self.cur, self.now[slot], self.score)
                kv.kvtrim_select_global(ctx, self.cur, self.score, self.budget, self.keep, self.kept, self.thr)
            if self.inplace:                                      # the other cache only lends its arrays
                kv.kvtrim_compact_attn_inplace(ctx, self.cur, self.keep, self.kept, dst, i["q"], 0, w.n_layers, self.scale,
                                               self.out[slot])
                return
            kv.kvtrim_compact_attn(ctx, self.cur, self.keep, self.kept, dst, 1, i["q"], 0, w.n_layers, self.scale,
                                   self.out[slot])
            self.cur, self.flip = dst, self.flip ^ 1

    def snapshot(self):
        """Everything a step leaves behind, as host arrays."""
        s = {"out0": self.out[0].cpu().numpy(), "out1": self.out[1].cpu().numpy(), "kept": self.kept.cpu().numpy(),
             "thr": self.thr.cpu().numpy()}
        if self.paged:
            ph = PagedHost(self.pc)
            assert ph.structure_problems() == []
            idx, counts = ph.ordered_slots()
            s.update(counts=counts, pos=ph.pos[idx], lb=ph.log_beta[idx], k=ph.k[idx], v=ph.v[idx])
        else:
            c = self.cur
            n = int(c.seg_len.sum().item()) + self.w.nseg
            s.update(seg_len=c.seg_len.cpu().numpy(), seg_start=c.seg_start.cpu().numpy())
            live = np.zeros(c.cap, bool)
            for a, m in zip(s["seg_start"], s["seg_len"]):
                live[a:a + m] = True
            s.update(pos=c.pos.cpu().numpy()[live], lb=c.log_beta.cpu().numpy()[live],
                     k=c.k.cpu().view(torch.int16).numpy()[live], v=c.v.cpu().view(torch.int16).numpy()[live])
            del n
        return s


def same(a, b):
    return all(np.array_equal(a[k].view(np.uint8) if a[k].dtype.kind == "f" else a[k],
                              b[k].view(np.uint8) if b[k].dtype.kind == "f" else b[k]) for k in a) and a.keys() == b.keys()


@pytest.mark.parametrize("paged", [False, True, "inplace", "score_select", "decode_step", "decode_step_inplace", "paged_decode_step"])
def test_two_captured_steps_replayed_three_times_match_the_eager_loop(paged):
    w = ki.workload("tiny", prefill=900)
    calls = paged if paged in ("score_select", "decode_step", "decode_step_inplace", "paged_decode_step") else "four"
    inplace, paged = paged in ("inplace", "decode_step_inplace"), paged is True or paged == "paged_decode_step"
    eager, graphed = Loop(w, paged, inplace, calls), Loop(w, paged, inplace, calls)
    for loop in (eager, graphed):
        loop.first_step()
        assert kv.kvtrim_poll_error(loop.ctx) == 0
    assert same(eager.snapshot(), graphed.snapshot())

    # capture steps "slot 0, slot 1" (for the ragged loop that is one full ping-pong of the two caches)
    graphed.load_inputs(0, 1)
    graphed.load_inputs(1, 2)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        graphed.step(0)
        graphed.step(1)
    torch.cuda.synchronize()
    # capture does not run anything: the state is still that of the first step
    scratch = torch.zeros(1 << 20, device=DEV)
    for r in range(3):
        s0, s1 = 1 + 2 * r, 2 + 2 * r
        graphed.load_inputs(0, s0)
        graphed.load_inputs(1, s1)
        g.replay()
        scratch.add_(1.0).sum().item()                           # eager work and a synchronisation between replays
        eager.load_inputs(0, s0)
        eager.step(0)
        eager.load_inputs(1, s1)
        eager.step(1)
        torch.cuda.synchronize()
        assert kv.kvtrim_poll_error(eager.ctx) == 0 and kv.kvtrim_poll_error(graphed.ctx) == 0
        assert same(eager.snapshot(), graphed.snapshot()), f"replay {r} differs from the eager steps {s0}, {s1}"


@pytest.mark.parametrize("n_tok,prepared", [(1, False), (3, True), (40, True), (130, False)])
def test_captured_gate_forward_matches_the_eager_call(n_tok, prepared):
    # the gate forward is two or three kernel launches on the caller's stream: captured once, replayed with new
    # token representations in the same buffers, it must give the eager call's bits
    L, H, d_model, d_g, d_p = 3, 2, 512, 128, 16
    wts = ki.gate_weights(L, H, d_model, d_g, d_p, seed=5)
    gate = kv.Gate.from_dict(wts, DEV)
    ctx = kv.Context(1, L, H, H, 64, 1024)
    prep = None
    if prepared:
        prep = torch.empty(kv.kvtrim_gate_prepared_bytes(gate, L, H) // 4, dtype=torch.float32, device=DEV)
        kv.kvtrim_gate_prepare(ctx, gate, prep)
    x = torch.zeros(L, n_tok, d_model, dtype=torch.bfloat16, device=DEV)
    scratch = torch.empty(kv.kvtrim_gate_scratch_bytes(gate, n_tok, L) // 4, dtype=torch.float32, device=DEV)
    lb_g, lt_g = (torch.zeros(n_tok, L, H, dtype=torch.float32, device=DEV) for _ in range(2))
    lb_e, lt_e = (torch.zeros(n_tok, L, H, dtype=torch.float32, device=DEV) for _ in range(2))

    def call(lb, lt):
        if prepared:
            kv.kvtrim_gate_forward_prepared(ctx, gate, prep, x, n_tok, 0, L, 2, scratch, lb, lt)
        else:
            kv.kvtrim_gate_forward(ctx, gate, x, n_tok, 0, L, 2, scratch, lb, lt)

    x.copy_(ki.gate_inputs(L, n_tok, d_model, salt=0))
    call(lb_e, lt_e)                                              # warm-up outside the capture
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        call(lb_g, lt_g)
    torch.cuda.synchronize()
    for r in range(1, 4):
        x.copy_(ki.gate_inputs(L, n_tok, d_model, salt=r))
        g.replay()
        torch.cuda.synchronize()
        scratch.fill_(float("nan"))                               # eager work between the replays
        call(lb_e, lt_e)
        torch.cuda.synchronize()
        assert kv.kvtrim_poll_error(ctx) == 0
        assert torch.equal(lb_g.view(torch.int32), lb_e.view(torch.int32)), (n_tok, prepared, r)
        assert torch.equal(lt_g.view(torch.int32), lt_e.view(torch.int32)), (n_tok, prepared, r)
