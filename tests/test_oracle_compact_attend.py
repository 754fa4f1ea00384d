"""Pins of the oracle's compaction and attention (CPU only).

Compaction is checked against numpy boolean indexing (a library routine) and
its invariants; attention against torch's CPU scaled_dot_product_attention in
fp64, special cases with known answers, and the exact dilution identity of
Cor. 3.2 evaluated with numpy.
"""
import math

import numpy as np
import pytest
import torch

import kvtrim_inputs as ki
import oracle
from helpers import bf16_bits, bits_to_f64, host_cache, live_mask


def make(seg_len, S=1, L=2, H=2, G=2, D=64, reserve=1, salt=0):
    w = ki.Workload("t", 0, S, L, H, G * H, D, (0,) * S, (0,) * S, 1, 3.0, 1.5)
    c, now = ki.ragged_cache(w, seg_len, reserve=reserve, salt=salt)
    return w, host_cache(w, c), now.numpy()


def rand_q(w, seed):
    g = torch.Generator().manual_seed(seed)
    q = torch.randn(w.n_seq, w.n_layers, w.n_q_heads, w.head_dim, generator=g).to(torch.bfloat16)
    return bf16_bits(q)


# ----------------------------------------------------------------------------- compaction

@pytest.mark.parametrize("seed", range(4))
def test_compact_is_a_stable_filter_per_segment(seed):
    rng = np.random.default_rng(seed)
    seg_len = rng.integers(0, 60, 8)
    w, hc, _ = make(seg_len, L=2, H=4, reserve=2, salt=seed)
    keep = (rng.random(hc.cap) < 0.4).astype(np.uint8)
    reserve = int(rng.integers(0, 4))
    dst = oracle.compact(hc, keep, int(keep.sum()) + reserve * w.nseg + 5, reserve)
    cursor = 0
    for g in range(w.nseg):
        s0, n = int(hc.seg_start[g]), int(hc.seg_len[g])
        m = keep[s0:s0 + n].astype(bool)
        assert dst.seg_start[g] == cursor and dst.seg_len[g] == m.sum()
        d0 = cursor
        np.testing.assert_array_equal(dst.k[d0:d0 + m.sum()], hc.k[s0:s0 + n][m])
        np.testing.assert_array_equal(dst.v[d0:d0 + m.sum()], hc.v[s0:s0 + n][m])
        np.testing.assert_array_equal(dst.log_beta[d0:d0 + m.sum()].view(np.uint32),
                                      hc.log_beta[s0:s0 + n][m].view(np.uint32))
        np.testing.assert_array_equal(dst.pos[d0:d0 + m.sum()], hc.pos[s0:s0 + n][m])
        assert np.all(np.diff(dst.pos[d0:d0 + m.sum()]) > 0)
        cursor += int(m.sum()) + reserve


def test_compact_with_all_ones_is_identity_and_with_all_zeros_is_empty():
    w, hc, _ = make([7, 0, 19, 4], reserve=1)
    ones = np.ones(hc.cap, np.uint8)
    dst = oracle.compact(hc, ones, hc.cap, 1)
    np.testing.assert_array_equal(dst.seg_start, hc.seg_start)
    np.testing.assert_array_equal(dst.seg_len, hc.seg_len)
    live = live_mask(hc)
    np.testing.assert_array_equal(dst.k[live], hc.k[live])
    np.testing.assert_array_equal(dst.pos[live], hc.pos[live])
    dst = oracle.compact(hc, np.zeros(hc.cap, np.uint8), 8, 2)
    assert dst.seg_len.tolist() == [0, 0, 0, 0] and dst.seg_start.tolist() == [0, 2, 4, 6]


def test_compact_reports_overflow_of_destination():
    w, hc, _ = make([5, 5, 5, 5])
    with pytest.raises(OverflowError):
        oracle.compact(hc, np.ones(hc.cap, np.uint8), 23, 1)


def test_append_writes_behind_segment_end_and_detects_full_segment():
    w, hc, now = make([3, 0, 2, 1], reserve=1)
    k_new = np.arange(w.nseg * 64, dtype=np.uint16).reshape(w.nseg, 64)
    before_len = hc.seg_len.copy()
    oracle.append(hc, k_new, k_new + 1, np.full(w.nseg, -0.5, np.float32), np.full(w.nseg, 99, np.int32))
    np.testing.assert_array_equal(hc.seg_len, before_len + 1)
    for g in range(w.nseg):
        e = hc.seg_start[g] + hc.seg_len[g] - 1
        np.testing.assert_array_equal(hc.k[e], k_new[g])
        np.testing.assert_array_equal(hc.v[e], k_new[g] + 1)
        assert hc.pos[e] == 99 and hc.log_beta[e] == np.float32(-0.5)
    with pytest.raises(OverflowError):
        oracle.append(hc, k_new, k_new, np.zeros(w.nseg, np.float32), np.full(w.nseg, 100, np.int32))


# ----------------------------------------------------------------------------- attention

def sdpa_reference(w, hc, qbits, scale):
    """torch CPU SDPA in fp64, one call per segment."""
    G, D = w.group, w.head_dim
    out = np.zeros((w.n_seq, w.n_layers, w.n_q_heads, D))
    lse = np.full((w.n_seq, w.n_layers, w.n_q_heads), -np.inf)
    q = bits_to_f64(qbits).reshape(w.n_seq, w.n_layers, w.n_q_heads, D)
    for s in range(w.n_seq):
        for l in range(w.n_layers):
            for h in range(w.n_kv_heads):
                g = w.seg_id(s, l, h)
                s0, n = int(hc.seg_start[g]), int(hc.seg_len[g])
                if n == 0:
                    continue
                K = torch.from_numpy(bits_to_f64(hc.k[s0:s0 + n]))
                V = torch.from_numpy(bits_to_f64(hc.v[s0:s0 + n]))
                Q = torch.from_numpy(q[s, l, h * G:(h + 1) * G])
                o = torch.nn.functional.scaled_dot_product_attention(Q[None], K[None], V[None], scale=scale)
                out[s, l, h * G:(h + 1) * G] = o[0].numpy()
                lse[s, l, h * G:(h + 1) * G] = torch.logsumexp(Q @ K.T * scale, dim=-1).numpy()
    return out, lse


@pytest.mark.parametrize("S,L,H,G,D", [(1, 2, 2, 2, 64), (2, 1, 2, 4, 128), (1, 1, 3, 7, 128)])
def test_attend_equals_library_sdpa_in_fp64(S, L, H, G, D):
    rng = np.random.default_rng(S * 100 + G)
    seg_len = rng.integers(0, 70, S * L * H)
    seg_len[0] = 0
    w, hc, _ = make(seg_len, S, L, H, G, D, salt=G)
    q = rand_q(w, 3)
    scale = 1.0 / math.sqrt(D)
    out, lse = oracle.attend(hc, q, scale)
    ref, ref_lse = sdpa_reference(w, hc, q, scale)
    np.testing.assert_allclose(out, ref, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(lse, ref_lse, rtol=1e-12)
    assert np.all(out[0, 0, :G] == 0.0) and np.all(np.isneginf(lse[0, 0, :G]))     # empty segment


def test_attend_single_entry_returns_its_value_row_exactly():
    w, hc, _ = make([1, 1, 1, 1])
    out, lse = oracle.attend(hc, rand_q(w, 1), 0.125)
    for l in range(2):
        for h in range(2):
            e = int(hc.seg_start[w.seg_id(0, l, h)])
            for j in range(2):
                np.testing.assert_array_equal(out[0, l, h * 2 + j], bits_to_f64(hc.v[e]))


def test_attend_uniform_keys_average_the_values_and_is_permutation_invariant():
    w, hc, _ = make([16, 9, 0, 5])
    s0 = int(hc.seg_start[0])
    hc.k[s0:s0 + 16] = hc.k[s0]                         # identical keys -> uniform weights
    q = rand_q(w, 2)
    out, _ = oracle.attend(hc, q, 0.125)
    np.testing.assert_allclose(out[0, 0, 0], bits_to_f64(hc.v[s0:s0 + 16]).mean(0), rtol=1e-13, atol=1e-14)
    s1 = int(hc.seg_start[1])
    perm = np.random.default_rng(0).permutation(9)
    hc.k[s1:s1 + 9] = hc.k[s1:s1 + 9][perm]
    hc.v[s1:s1 + 9] = hc.v[s1:s1 + 9][perm]
    out2, _ = oracle.attend(hc, q, 0.125)
    np.testing.assert_allclose(out2[0, 0, 2:4], out[0, 0, 2:4], rtol=1e-12, atol=1e-14)


def test_layer_range_limits_what_is_written():
    w, hc, _ = make([4, 4, 4, 4])
    q = rand_q(w, 5)
    full, _ = oracle.attend(hc, q, 0.125)
    part, _ = oracle.attend(hc, q, 0.125, layer_begin=1, layer_end=2)
    np.testing.assert_array_equal(part[0, 1], full[0, 1])
    assert np.all(part[0, 0] == 0.0)


def test_budget_covering_everything_gives_full_cache_attention():
    # Sec. 2.1: with r = 1 everywhere Eq. reform is the full-cache attention.
    w, hc, now = make([30, 12, 0, 21], salt=11)
    q = rand_q(w, 7)
    full, full_lse = oracle.attend(hc, q, 0.125)
    keep, kept, _ = oracle.select(hc, oracle.score(hc, now), np.array([10 ** 6], np.int64))
    dst = oracle.compact(hc, keep, hc.cap + 3, 1)
    out, lse = oracle.attend(dst, q, 0.125)
    np.testing.assert_array_equal(out, full)
    np.testing.assert_array_equal(lse, full_lse)


def test_hard_eviction_satisfies_the_dilution_identity():
    # Cor. 3.2: delta^r = (rho_D/rho_U) delta / ((1 - delta) + (rho_D/rho_U) delta), exact for any
    # retention weights; here r in {0,1} comes from score -> select -> compact, and the attention
    # mass on the useful set U is read off the oracle's output by making V[:,0] the indicator of U.
    n = 64
    w, hc, now = make([n], L=1, H=1, G=2, salt=13)
    rng = np.random.default_rng(5)
    s0 = int(hc.seg_start[0])
    useful = rng.random(n) < 0.25
    one, zero = 0x3F80, 0x0000                      # bf16 bit patterns of 1.0 and 0.0
    hc.v[s0:s0 + n, 0] = np.where(useful, one, zero)
    q = rand_q(w, 17)
    scale = 0.125
    full, _ = oracle.attend(hc, q, scale)
    keep, kept, _ = oracle.select(hc, oracle.score(hc, now), np.array([n // 2], np.int64))
    r = keep[s0:s0 + n].astype(np.float64)
    assert 0 < r[useful].sum() and 0 < r[~useful].sum() < (~useful).sum()
    evicted, _ = oracle.attend(oracle.compact(hc, keep, n, 0), q, scale)
    K = bits_to_f64(hc.k[s0:s0 + n])
    for j in range(2):
        z = K @ bits_to_f64(q.reshape(-1, 64)[j]) * scale
        ez = np.exp(z - z.max())
        rho_u = (r[useful] * ez[useful]).sum() / ez[useful].sum()
        rho_d = (r[~useful] * ez[~useful]).sum() / ez[~useful].sum()
        delta = 1.0 - full[0, 0, j, 0]
        delta_r = 1.0 - evicted[0, 0, j, 0]
        ratio = rho_d / rho_u
        assert math.isclose(delta_r, ratio * delta / ((1 - delta) + ratio * delta), rel_tol=1e-10)


# ----------------------------------------------------------------------------- soft (retention-gated) attention, occupancy

def test_soft_attention_equals_library_sdpa_with_an_additive_bias():
    # Sec. 2.2: weights beta^(t-i) e^z, i.e. logits z + (t-i) log(beta); torch SDPA takes that as a float mask
    w, hc, now = make([40, 0, 23, 9], S=1, L=2, H=2, G=2, D=64, salt=31)
    q = rand_q(w, 4)
    scale = 0.125
    out, lse = oracle.attend(hc, q, scale, soft_now=now)
    qf = bits_to_f64(q).reshape(1, 2, 4, 64)
    for l in range(2):
        for h in range(2):
            g = w.seg_id(0, l, h)
            s0, n = int(hc.seg_start[g]), int(hc.seg_len[g])
            if n == 0:
                assert np.all(out[0, l, h * 2:(h + 1) * 2] == 0)
                continue
            K = torch.from_numpy(bits_to_f64(hc.k[s0:s0 + n]))
            V = torch.from_numpy(bits_to_f64(hc.v[s0:s0 + n]))
            Q = torch.from_numpy(qf[0, l, h * 2:(h + 1) * 2])
            bias = torch.from_numpy((now[0] - hc.pos[s0:s0 + n]).astype(np.float64) * hc.log_beta[s0:s0 + n].astype(np.float64))
            o = torch.nn.functional.scaled_dot_product_attention(Q[None], K[None], V[None], attn_mask=bias[None, None, :].expand(1, 2, n),
                                                                 scale=scale)
            np.testing.assert_allclose(out[0, l, h * 2:(h + 1) * 2], o[0].numpy(), rtol=1e-11, atol=1e-13)
            np.testing.assert_allclose(lse[0, l, h * 2:(h + 1) * 2],
                                       torch.logsumexp(Q @ K.T * scale + bias[None, :], dim=-1).numpy(), rtol=1e-12)


def test_soft_attention_with_beta_one_is_standard_attention():
    # Sec. 2.2: beta_i = 1 recovers standard attention
    w, hc, now = make([30, 12, 7, 21], salt=32)
    hc.log_beta[:] = 0.0
    q = rand_q(w, 6)
    hard, hard_lse = oracle.attend(hc, q, 0.125)
    soft, soft_lse = oracle.attend(hc, q, 0.125, soft_now=now)
    np.testing.assert_array_equal(soft, hard)
    np.testing.assert_array_equal(soft_lse, hard_lse)


def test_soft_retention_weights_satisfy_the_dilution_identity():
    # Cor. 3.2 holds for general retention weights r in [0,1], here r_i = beta_i^(t-i)
    n = 48
    w, hc, now = make([n], L=1, H=1, G=2, salt=33)
    rng = np.random.default_rng(9)
    s0 = int(hc.seg_start[0])
    useful = rng.random(n) < 0.3
    hc.v[s0:s0 + n, 0] = np.where(useful, 0x3F80, 0x0000)          # bf16 1.0 / 0.0: V[:,0] = indicator of U
    q = rand_q(w, 8)
    scale = 0.125
    full, _ = oracle.attend(hc, q, scale)
    soft, _ = oracle.attend(hc, q, scale, soft_now=now)
    r = np.exp((now[0] - hc.pos[s0:s0 + n]).astype(np.float64) * hc.log_beta[s0:s0 + n].astype(np.float64))
    K = bits_to_f64(hc.k[s0:s0 + n])
    for j in range(2):
        z = K @ bits_to_f64(q.reshape(-1, 64)[j]) * scale
        ez = np.exp(z - z.max())
        rho_u = (r[useful] * ez[useful]).sum() / ez[useful].sum()
        rho_d = (r[~useful] * ez[~useful]).sum() / ez[~useful].sum()
        delta, delta_r = 1.0 - full[0, 0, j, 0], 1.0 - soft[0, 0, j, 0]
        ratio = rho_d / rho_u
        assert math.isclose(delta_r, ratio * delta / ((1 - delta) + ratio * delta), rel_tol=1e-10)


def test_occupancy_closed_forms():
    # equal beta and positions 0..T-1: sum_{i<T} beta^(t-i) is a geometric series; beta = 1 counts the entries
    L, H, T = 2, 3, 40
    w = ki.Workload("t", 0, 1, L, H, 2 * H, 64, (T,), (0,), 1, 3.0, 1.5)
    hc = host_cache(w, ki.prefill_cache(w, reserve=1))
    beta = 0.93
    hc.log_beta[:] = np.float32(math.log(beta))
    b = math.exp(float(np.float32(math.log(beta))))
    t = T + 4
    occ = oracle.occupancy(hc, np.array([t], np.int32))
    closed = L * H * b ** (t - T + 1) * (1 - b ** T) / (1 - b)
    assert math.isclose(occ[0], closed, rel_tol=1e-12)
    hc.log_beta[:] = 0.0
    assert oracle.occupancy(hc, np.array([t], np.int32))[0] == L * H * T
    # per sequence
    w2, hc2, now2 = make(np.arange(8) + 1, S=2, L=2, H=2, salt=34)
    occ2 = oracle.occupancy(hc2, now2)
    for s in range(2):
        tot = 0.0
        for g in range(s * 4, (s + 1) * 4):
            for j in range(hc2.seg_len[g]):
                e = hc2.seg_start[g] + j
                tot += math.exp(float(now2[s] - hc2.pos[e]) * float(hc2.log_beta[e]))
        assert math.isclose(occ2[s], tot, rel_tol=1e-12)


def test_append_takes_rows_up_to_the_first_padding_row():
    # sequences of a batch may bring different numbers of tokens: rows from the first negative position on are padding
    sh = oracle.Shape(2, 1, 2, 2, 4)
    hc = oracle.HostCache(sh, 64)
    hc.seg_start[:] = [0, 16, 32, 48]
    rng = np.random.default_rng(3)
    k = rng.integers(0, 60000, (4, 5, 4)).astype(np.uint16)
    v = rng.integers(0, 60000, (4, 5, 4)).astype(np.uint16)
    lb = -rng.random((4, 5)).astype(np.float32)
    pos = np.array([[0, 1, 2, 3, 4], [0, 1, 2, 3, 4], [0, 1, -1, 7, 8], [-1, 0, 1, 2, 3]], np.int32)
    oracle.append(hc, k, v, lb, pos)
    assert list(hc.seg_len) == [5, 5, 2, 0]
    for g, n in enumerate(hc.seg_len):
        s0 = hc.seg_start[g]
        assert np.array_equal(hc.k[s0:s0 + n], k[g, :n]) and np.array_equal(hc.v[s0:s0 + n], v[g, :n])
        assert np.array_equal(hc.log_beta[s0:s0 + n], lb[g, :n]) and np.array_equal(hc.pos[s0:s0 + n], pos[g, :n])
    assert not hc.k[34:48].any() and not hc.k[48:].any()          # nothing written behind the taken rows


def test_compact_carries_the_horizon_tail_with_its_entry():
    # a cache with the per-entry constant of a lookahead horizon H > 1 (Eq. global_score: log of the tail sum,
    # fixed like beta when the token is cached): compaction moves it with its entry, bit for bit, and only then
    rng = np.random.default_rng(21)
    seg_len = rng.integers(0, 70, 8)
    w, hc, _ = make(seg_len, L=2, H=4, reserve=2, salt=9)
    tail = (-rng.random(hc.cap) * 3).astype(np.float32)           # distinct values, unrelated to log_beta
    hc = oracle.HostCache.from_arrays(hc.shape, hc.k, hc.v, hc.log_beta, hc.pos, hc.seg_start, hc.seg_len, log_tail=tail.copy())
    keep = (rng.random(hc.cap) < 0.5).astype(np.uint8)
    dst = oracle.compact(hc, keep, int(keep.sum()) + 3 * w.nseg + 5, 3)
    assert dst.log_tail is not None
    for g in range(w.nseg):
        s0, n = int(hc.seg_start[g]), int(hc.seg_len[g])
        m = keep[s0:s0 + n].astype(bool)
        d0 = int(dst.seg_start[g])
        assert dst.seg_len[g] == m.sum()
        np.testing.assert_array_equal(dst.log_tail[d0:d0 + m.sum()].view(np.uint32), tail[s0:s0 + n][m].view(np.uint32))
        np.testing.assert_array_equal(dst.log_beta[d0:d0 + m.sum()].view(np.uint32),
                                      hc.log_beta[s0:s0 + n][m].view(np.uint32))
        np.testing.assert_array_equal(dst.pos[d0:d0 + m.sum()], hc.pos[s0:s0 + n][m])
    # the tail changes the ranking, so a mix-up with log_beta or a shifted index would show: the two arrays differ
    assert not np.array_equal(dst.log_tail[live_mask(dst)], dst.log_beta[live_mask(dst)])
    # without a tail in the source there is none in the destination
    w2, hc2, _ = make([4, 4, 4, 4])
    assert oracle.compact(hc2, np.ones(hc2.cap, np.uint8), hc2.cap, 1).log_tail is None


def test_append_writes_the_horizon_tail_of_the_new_tokens():
    sh = oracle.Shape(2, 1, 2, 2, 4)
    hc = oracle.HostCache(sh, 64, with_tail=True)
    hc.seg_start[:] = [0, 16, 32, 48]
    hc.log_tail[:] = 7.0                                           # sentinel: slots that no token takes keep it
    rng = np.random.default_rng(5)
    k = rng.integers(0, 60000, (4, 3, 4)).astype(np.uint16)
    lb = -rng.random((4, 3)).astype(np.float32)
    lt = rng.random((4, 3)).astype(np.float32)                     # log(1 + beta + ...) >= 0
    pos = np.array([[0, 1, 2], [5, 6, -1], [-1, 0, 1], [3, 4, 9]], np.int32)
    oracle.append(hc, k, k, lb, pos, log_tail_new=lt)
    assert list(hc.seg_len) == [3, 2, 0, 3]
    for g, n in enumerate(hc.seg_len):
        s0 = hc.seg_start[g]
        assert np.array_equal(hc.log_tail[s0:s0 + n].view(np.uint32), lt[g, :n].view(np.uint32))
        assert np.array_equal(hc.log_beta[s0:s0 + n].view(np.uint32), lb[g, :n].view(np.uint32))
        assert np.all(hc.log_tail[s0 + n:s0 + 16] == 7.0)          # padding rows and free slots untouched
    # a second chunk lands behind the first, tails included
    lt2 = rng.random((4, 3)).astype(np.float32)
    oracle.append(hc, k, k, lb, np.where(pos >= 0, pos + 10, pos), log_tail_new=lt2)
    assert list(hc.seg_len) == [6, 4, 0, 6]
    assert np.array_equal(hc.log_tail[3:6], lt2[0]) and np.array_equal(hc.log_tail[18:20], lt2[1, :2])
    with pytest.raises(AssertionError):                            # a cache with tails refuses tokens without one
        oracle.append(hc, k, k, lb, pos)


def test_the_attention_tolerance_is_not_limited_by_the_oracle():
    # the same attention evaluated in fp32 (torch CPU, bf16 inputs widened exactly) lands within 1e-5 of the fp64
    # oracle in the benchmark's error metric: the 5e-3 tolerance of the GPU parity tests has three orders of
    # magnitude of room above what fp32 accumulation costs
    seg_len = [3000, 0, 1, 777]
    w, hc, _ = make(seg_len, 1, 2, 2, 4, 128, salt=9)
    q = rand_q(w, 5)
    scale = 1.0 / math.sqrt(128)
    out, _ = oracle.attend(hc, q, scale)
    G, D = w.group, w.head_dim
    q32 = bits_to_f64(q).reshape(w.n_layers, w.n_q_heads, D).astype(np.float32)
    worst = 0.0
    for l in range(w.n_layers):
        for h in range(w.n_kv_heads):
            g = w.seg_id(0, l, h)
            s0, n = int(hc.seg_start[g]), int(hc.seg_len[g])
            if n == 0:
                continue
            K = torch.from_numpy(bits_to_f64(hc.k[s0:s0 + n]).astype(np.float32))
            V = torch.from_numpy(bits_to_f64(hc.v[s0:s0 + n]).astype(np.float32))
            Q = torch.from_numpy(q32[l, h * G:(h + 1) * G])
            o32 = torch.nn.functional.scaled_dot_product_attention(Q[None], K[None], V[None], scale=scale)[0].numpy()
            worst = max(worst, float(np.abs(o32 - out[0, l, h * G:(h + 1) * G]).max()))
    assert worst / np.abs(out).max() <= 1e-5
