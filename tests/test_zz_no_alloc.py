"""GPU: kvtrim_select_global_noalloc (stage 2 without a context, tables in a fixed device array inside the
library) gives bit for bit what kvtrim_select_global gives - on two calls in a row, the second on a smaller
cache, so that whatever the first call left in the shared array is still there when the second runs - and
agrees with the oracle's full sort."""
import numpy as np
import pytest
import torch

import kvtrim_inputs as ki
import oracle
import paper_2605_09649_amd as kv
from helpers import host_cache, live_mask

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _select_both_ways(w, seg_len, budget, salt, planted_ties):
    c, now = ki.ragged_cache(w, seg_len, salt=salt)
    hc = host_cache(w, c)
    score_ref = oracle.score(hc, now.numpy())
    if planted_ties:                                   # many equal scores around the threshold: the tie rule decides
        rng = np.random.default_rng(salt)
        score_ref = rng.choice(np.array([-0.5, -0.5, -2.0, -0.0, 0.0, -np.inf], np.float32), size=hc.cap).astype(np.float32)
    keep_ref, kept_ref, thr_ref = oracle.select(hc, score_ref, np.array(budget, np.int64))
    live = live_mask(hc)

    dc = kv.Cache.from_dict(c, DEV)
    cap = dc.cap
    score = torch.from_numpy(score_ref).to(DEV)
    bud = torch.tensor(budget, dtype=torch.int64, device=DEV)
    cfg = (w.n_seq, w.n_layers, w.n_kv_heads, w.n_q_heads, w.head_dim, cap)

    ctx = kv.Context(*cfg)
    keep_a = torch.zeros(cap, dtype=torch.uint8, device=DEV)
    kept_a = torch.zeros(w.nseg, dtype=torch.int32, device=DEV)
    thr_a = torch.zeros(w.n_seq, dtype=torch.int32, device=DEV)
    kv.kvtrim_select_global(ctx, dc, score, bud, keep_a, kept_a, thr_a)
    assert kv.kvtrim_poll_error(ctx) == 0

    keep_b = torch.full((cap,), 7, dtype=torch.uint8, device=DEV)
    kept_b = torch.full((w.nseg,), -1, dtype=torch.int32, device=DEV)
    thr_b = torch.full((w.n_seq,), 5, dtype=torch.int32, device=DEV)
    status = torch.full((1,), 99, dtype=torch.int32, device=DEV)
    kv.kvtrim_select_global_noalloc(cfg, dc, score, bud, keep_b, kept_b, thr_b, status)
    torch.cuda.synchronize()

    assert int(status.item()) == 0
    ka, kb = keep_a.cpu().numpy(), keep_b.cpu().numpy()
    assert np.array_equal(kb[live], ka[live])
    assert np.array_equal(kept_b.cpu().numpy(), kept_a.cpu().numpy())
    assert np.array_equal(thr_b.cpu().numpy(), thr_a.cpu().numpy())
    assert np.array_equal(kb[live], keep_ref[live])
    assert np.array_equal(kept_b.cpu().numpy(), kept_ref)
    assert np.array_equal(thr_b.cpu().numpy().view(np.uint32), thr_ref)
    ctx.close()


def test_noalloc_select_matches_select_global_twice_second_call_smaller():
    # first call: 2 sequences, several 2048-entry chunks per segment and ragged tails
    w1 = ki.Workload("t", 0, 2, 3, 2, 4, 64, (1, 1), (1, 1), 1, 3.0, 1.5)
    rng = np.random.default_rng(3)
    seg1 = rng.integers(0, 9000, w1.nseg).tolist()
    b1 = [int(0.4 * sum(seg1[:6])), int(0.7 * sum(seg1[6:]))]
    _select_both_ways(w1, seg1, b1, salt=31, planted_ties=False)
    # second call, right after, on a smaller cache of another shape (one sequence), ties at the threshold
    w2 = ki.Workload("t", 0, 1, 2, 2, 2, 64, (1,), (1,), 1, 3.0, 1.5)
    seg2 = [700, 0, 2049, 33]
    _select_both_ways(w2, seg2, [1500], salt=32, planted_ties=True)


def test_noalloc_select_rejects_what_does_not_fit_its_array():
    w = ki.Workload("t", 0, 1, 1, 1, 1, 64, (1,), (1,), 1, 3.0, 1.5)
    c, now = ki.ragged_cache(w, [100], salt=1)
    dc = kv.Cache.from_dict(c, DEV)
    score = torch.zeros(dc.cap, dtype=torch.float32, device=DEV)
    bud = torch.tensor([10], dtype=torch.int64, device=DEV)
    keep = torch.zeros(dc.cap, dtype=torch.uint8, device=DEV)
    kept = torch.zeros(1, dtype=torch.int32, device=DEV)
    with pytest.raises(kv.KvtrimError) as e:                       # 64 sequences: the histograms alone exceed the array
        kv.kvtrim_select_global_noalloc((64, 1, 1, 1, 64, dc.cap), dc, score, bud, keep, kept)
    assert e.value.status == -1
    with pytest.raises(kv.KvtrimError) as e:                       # cache larger than the configuration allows
        kv.kvtrim_select_global_noalloc((1, 1, 1, 1, 64, dc.cap - 1), dc, score, bud, keep, kept)
    assert e.value.status == -1
