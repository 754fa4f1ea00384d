"""Out-of-bounds canaries: every caller-owned output buffer of a step sits between guard zones; after several
steps through the two-call, the fused and the paged path the guards must be untouched (and the results still
match the oracle, which the other suites check - here only that nothing is written outside the buffers)."""
import math

import numpy as np
import pytest
import torch

import kvtrim_inputs as ki
import paper_2605_09649_amd as kv

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
GUARD = 4096                      # bytes on each side (keeps the 16-byte alignment of the payload)


class Guarded:
    def __init__(self):
        self.items = []

    def make(self, shape, dtype):
        n = int(np.prod(shape))
        g = GUARD // torch.empty(0, dtype=dtype).element_size()
        big = torch.empty(n + 2 * g, dtype=dtype, device=DEV)
        raw = big.view(torch.uint8)
        raw.fill_(0x5A)
        view = big[g:g + n].view(*shape)
        view.zero_()
        self.items.append((raw, g * big.element_size(), n * big.element_size()))
        return view

    def intact(self):
        for raw, lo, nbytes in self.items:
            if not bool((raw[:lo] == 0x5A).all()) or not bool((raw[lo + nbytes:] == 0x5A).all()):
                return False
        return True


def guarded_cache(gd, nseg, D, cap, with_tail=False):
    return kv.Cache(gd.make((cap, D), torch.bfloat16), gd.make((cap, D), torch.bfloat16), gd.make((cap,), torch.float32),
                    gd.make((cap,), torch.int32), gd.make((nseg,), torch.int64), gd.make((nseg,), torch.int32),
                    gd.make((cap,), torch.float32) if with_tail else None)


@pytest.mark.parametrize("mode", ["two-call", "fused", "paged"])
@pytest.mark.parametrize("G,D", [(2, 64), (4, 128), (7, 128)])
def test_nothing_is_written_outside_the_callers_buffers(mode, G, D):
    w = ki.Workload("c", 0, 2, 2, 3, 3 * G, D, (0, 0), (0, 0), 1, 3.0, 1.5)
    rng = np.random.default_rng(G * 100 + D)
    seg_len = rng.integers(0, 700, w.nseg)
    seg_len[2] = 0
    seg_len[5] = 3 * 128                                           # whole chunks / pages, no tail
    c, now0 = ki.ragged_cache(w, seg_len, reserve=1, salt=1)
    gd = Guarded()
    src = guarded_cache(gd, w.nseg, D, c["cap"])
    for name in ("k", "v", "log_beta", "pos", "seg_start", "seg_len"):
        getattr(src, name).copy_(c[name])
    per_seq = [int(seg_len[:6].sum()), int(seg_len[6:].sum())]
    budget = torch.tensor([per_seq[0] // 2, per_seq[1] // 3], dtype=torch.int64, device=DEV)
    dst_cap = sum(per_seq) // 2 + 8 * w.nseg
    spare = [guarded_cache(gd, w.nseg, D, dst_cap) for _ in range(2)]
    n_pages = dst_cap // kv.PAGE_SIZE + 3 * w.nseg
    cap = max(src.cap, dst_cap, n_pages * kv.PAGE_SIZE)
    ctx = kv.Context(w.n_seq, w.n_layers, w.n_kv_heads, w.n_q_heads, D, cap)
    score = gd.make((cap,), torch.float32)
    keep = gd.make((cap,), torch.uint8)
    kept = gd.make((w.nseg,), torch.int32)
    thr = gd.make((w.n_seq,), torch.int32)
    out = gd.make((w.n_seq, w.n_layers, w.n_q_heads, D), torch.float32)
    lse = gd.make((w.n_seq, w.n_layers, w.n_q_heads), torch.float32)
    pc = None
    if mode == "paged":
        pc = kv.PagedCache.__new__(kv.PagedCache)
        n = n_pages * kv.PAGE_SIZE
        pc.n_pages, pc.max_pages_per_seg, pc.nseg, pc.slots = n_pages, n_pages, w.nseg, n
        pc.k, pc.v = gd.make((n, D), torch.bfloat16), gd.make((n, D), torch.bfloat16)
        pc.log_beta, pc.pos, pc.log_tail = gd.make((n,), torch.float32), gd.make((n,), torch.int32), None
        pc.block_table = gd.make((w.nseg, n_pages), torch.int32)
        pc.seg_pages, pc.seg_live = gd.make((w.nseg,), torch.int32), gd.make((w.nseg,), torch.int32)
        pc.page_owner, pc.page_live = gd.make((n_pages,), torch.int32), gd.make((n_pages,), torch.int32)
        pc.free_list, pc.n_free = gd.make((n_pages,), torch.int32), gd.make((1,), torch.int32)
        B = kv.binding
        pc.c = B._PagedCache(B._ptr(pc.k).value, B._ptr(pc.v).value, B._ptr(pc.log_beta).value, B._ptr(pc.pos).value, None,
                             B._ptr(pc.block_table).value, B._ptr(pc.seg_pages).value, B._ptr(pc.seg_live).value,
                             B._ptr(pc.page_owner).value, B._ptr(pc.page_live).value, B._ptr(pc.free_list).value,
                             B._ptr(pc.n_free).value, n_pages, n_pages)
    scale = 1.0 / math.sqrt(D)
    now = now0.numpy().astype(np.int32)
    cur, flip = src, 0
    for step in range(4):
        inp = {k: v.to(DEV) for k, v in ki.decode_inputs(w, step).items()}
        now = now + 1
        now_dev = torch.from_numpy(now).to(DEV)
        pos_new = torch.from_numpy(np.repeat(now, w.n_layers * w.n_kv_heads).astype(np.int32)).to(DEV)
        if mode == "paged" and step > 0:
            kv.kvtrim_paged_append(ctx, pc, inp["k_new"], inp["v_new"], inp["log_beta_new"], pos_new)
            kv.kvtrim_paged_score(ctx, pc, now_dev, score)
            kv.kvtrim_paged_select(ctx, pc, score, budget, keep, kept, thr)
            kv.kvtrim_paged_evict(ctx, pc, keep)
            kv.kvtrim_paged_attn(ctx, pc, inp["q"], 0, w.n_layers, scale, out, lse)
        else:
            kv.kvtrim_append(ctx, cur, inp["k_new"], inp["v_new"], inp["log_beta_new"], pos_new, 1)
            kv.kvtrim_score(ctx, cur, now_dev, score)
            kv.kvtrim_select_global(ctx, cur, score, budget, keep, kept, thr)
            if mode == "paged":
                kv.kvtrim_paged_build(ctx, cur, keep, kept, pc)
                kv.kvtrim_paged_attn(ctx, pc, inp["q"], 0, w.n_layers, scale, out, lse)
            elif mode == "fused":
                kv.kvtrim_compact_attn(ctx, cur, keep, kept, spare[flip], 1, inp["q"], 0, w.n_layers, scale, out, lse)
                cur, flip = spare[flip], flip ^ 1
            else:
                kv.kvtrim_compact(ctx, cur, keep, kept, spare[flip], 1)
                kv.kvtrim_decode_attn(ctx, spare[flip], inp["q"], 0, w.n_layers, scale, out, lse)
                cur, flip = spare[flip], flip ^ 1
        assert kv.kvtrim_poll_error(ctx) == 0, (mode, step)
        assert gd.intact(), (mode, step)
    assert torch.isfinite(out).all()


@pytest.mark.parametrize("L,H,d_model,d_g,d_p,n_tok", [
    (2, 2, 256, 64, 8, 5),            # per-token kernels: u in the scratch buffer
    (2, 2, 256, 128, 8, 40),          # ... 40 tokens: with prepared weights already the folded kernel
    (2, 2, 256, 192, 8, 300),         # LDS-tiled first layer + readout
    (3, 3, 1024, 512, 16, 257),       # folded path, W1 straight from its rows (the scratch cannot hold the copy)
    (9, 2, 256, 256, 8, 260),         # folded path with the tiled copy of W1 in the scratch buffer
    (2, 8, 256, 384, 8, 513),         # ... eight heads, token tail of one
])
def test_gate_forward_stays_inside_scratch_and_outputs(L, H, d_model, d_g, d_p, n_tok):
    wts = ki.gate_weights(L, H, d_model, d_g, d_p, seed=3)
    gate = kv.Gate.from_dict(wts, DEV)
    ctx = kv.Context(1, L, H, H, 64, 1024)
    gd = Guarded()
    x = gd.make((L, n_tok, d_model), torch.bfloat16)
    x.copy_(ki.gate_inputs(L, n_tok, d_model, salt=1))
    scratch = gd.make((kv.kvtrim_gate_scratch_bytes(gate, n_tok, L) // 4,), torch.float32)
    lb = gd.make((n_tok, L, H), torch.float32)
    lt = gd.make((n_tok, L, H), torch.float32)
    for _ in range(2):
        kv.kvtrim_gate_forward(ctx, gate, x, n_tok, 0, L, 2, scratch, lb, lt)
    assert kv.kvtrim_poll_error(ctx) == 0
    torch.cuda.synchronize()
    assert gd.intact()
    assert bool(torch.isfinite(lb).all()) and bool((lb < 0).all()) and bool(torch.isfinite(lt).all())
    # the same with the weight-only work done once into a guarded buffer
    prepared = gd.make((kv.kvtrim_gate_prepared_bytes(gate, L, H) // 4,), torch.float32)
    kv.kvtrim_gate_prepare(ctx, gate, prepared)
    lb2 = gd.make((n_tok, L, H), torch.float32)
    for _ in range(2):
        kv.kvtrim_gate_forward_prepared(ctx, gate, prepared, x, n_tok, 0, L, 2, scratch, lb2, lt)
    assert kv.kvtrim_poll_error(ctx) == 0
    torch.cuda.synchronize()
    assert gd.intact()
    assert bool(((lb2 - lb).abs() <= 2e-4 * lb.abs()).all())


@pytest.mark.parametrize("D", [64, 128])
def test_chunk_steps_in_one_call_stay_inside_the_buffers(D):
    # kvtrim_append_compact over three chunks (the last one ragged): the source gets metadata only, the destination
    # the surviving rows; the guards of both caches, of the new-token buffers and of the outputs stay untouched
    w = ki.Workload("c", 0, 2, 2, 3, 6, D, (0, 0), (0, 0), 1, 3.0, 1.5)
    n_new, per_seq = 50, w.n_layers * w.n_kv_heads
    budget_per_seq = 40 * per_seq
    cap = 2 * budget_per_seq + w.nseg * n_new + 8
    gd = Guarded()
    caches = [guarded_cache(gd, w.nseg, D, cap) for _ in range(2)]
    caches[0].seg_start.copy_(torch.arange(w.nseg, dtype=torch.int64) * n_new)
    ctx = kv.Context(w.n_seq, w.n_layers, w.n_kv_heads, w.n_q_heads, D, cap)
    score, keep = gd.make((cap,), torch.float32), gd.make((cap,), torch.uint8)
    kept, thr = gd.make((w.nseg,), torch.int32), gd.make((w.n_seq,), torch.int32)
    budget = torch.full((w.n_seq,), budget_per_seq, dtype=torch.int64, device=DEV)
    k_new, v_new = gd.make((w.nseg, n_new, D), torch.bfloat16), gd.make((w.nseg, n_new, D), torch.bfloat16)
    lb_new, pos_new = gd.make((w.nseg, n_new), torch.float32), gd.make((w.nseg, n_new), torch.int32)
    next_pos = np.zeros(w.n_seq, np.int64)
    cur = 0
    for step, take in enumerate([(50, 50), (50, 50), (50, 7)]):
        inp = ki.chunk_inputs(w, n_new, DEV, step)
        k_new.copy_(inp["k_new"]); v_new.copy_(inp["v_new"]); lb_new.copy_(inp["log_beta_new"])
        pn = np.full((w.nseg, n_new), -1, np.int32)
        for s in range(w.n_seq):
            pn[s * per_seq:(s + 1) * per_seq, :take[s]] = next_pos[s] + np.arange(take[s])
        next_pos += np.array(take)
        pos_new.copy_(torch.from_numpy(pn))
        now = torch.from_numpy((next_pos - 1).astype(np.int32)).to(DEV)
        kv.kvtrim_append_compact(ctx, caches[cur], k_new, v_new, lb_new, pos_new, n_new, now, budget, score, keep, kept,
                                 caches[cur ^ 1], n_new, thr_key_out=thr)
        assert kv.kvtrim_poll_error(ctx) == 0, step
        assert gd.intact(), step
        cur ^= 1
    live = caches[cur].seg_len.cpu().numpy().reshape(w.n_seq, per_seq).sum(1)
    assert list(live) == [budget_per_seq, budget_per_seq]          # 150 and 107 tokens per list came in, 40 per list stay


@pytest.mark.parametrize("G,D", [(2, 64), (4, 128)])
def test_in_place_steps_stay_inside_the_buffers(G, D):
    # kvtrim_compact_attn_inplace: the cache, the spare arrays that park rows, and every output between guard zones
    w = ki.Workload("c", 0, 2, 2, 3, 3 * G, D, (0, 0), (0, 0), 1, 3.0, 1.5)
    rng = np.random.default_rng(G + D)
    seg_len = rng.integers(1, 900, w.nseg)
    seg_len[2] = 0
    seg_len[5] = 3 * 128
    room = 4
    c, now0 = ki.ragged_cache(w, seg_len, reserve=room, salt=2)
    gd = Guarded()
    cache = guarded_cache(gd, w.nseg, D, c["cap"])
    for name in ("k", "v", "log_beta", "pos", "seg_start", "seg_len"):
        getattr(cache, name).copy_(c[name])
    spare = guarded_cache(gd, w.nseg, D, c["cap"])
    cap = c["cap"]
    ctx = kv.Context(w.n_seq, w.n_layers, w.n_kv_heads, w.n_q_heads, D, cap)
    per_seq = [int(seg_len[:6].sum()), int(seg_len[6:].sum())]
    budget = torch.tensor([per_seq[0] - 20, per_seq[1] // 2], dtype=torch.int64, device=DEV)
    score, keep = gd.make((cap,), torch.float32), gd.make((cap,), torch.uint8)
    kept, thr = gd.make((w.nseg,), torch.int32), gd.make((w.n_seq,), torch.int32)
    out = gd.make((w.n_seq, w.n_layers, w.n_q_heads, D), torch.float32)
    lse = gd.make((w.n_seq, w.n_layers, w.n_q_heads), torch.float32)
    now = now0.numpy().astype(np.int32)
    for step in range(room):
        inp = {k: v.to(DEV) for k, v in ki.decode_inputs(w, step).items()}
        now = now + 1
        now_dev = torch.from_numpy(now).to(DEV)
        pos_new = torch.from_numpy(np.repeat(now, w.n_layers * w.n_kv_heads).astype(np.int32)).to(DEV)
        kv.kvtrim_append(ctx, cache, inp["k_new"], inp["v_new"], inp["log_beta_new"], pos_new, 1)
        kv.kvtrim_score(ctx, cache, now_dev, score)
        kv.kvtrim_select_global(ctx, cache, score, budget, keep, kept, thr)
        kv.kvtrim_compact_attn_inplace(ctx, cache, keep, kept, spare, inp["q"], 0, w.n_layers, 1.0 / math.sqrt(D), out, lse)
        assert kv.kvtrim_poll_error(ctx) == 0, step
        assert gd.intact(), step
    assert torch.isfinite(out).all()
    assert int(cache.seg_len.sum().item()) == int(budget.sum().item())
