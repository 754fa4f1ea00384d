"""GPU parity of the retention-gate forward (Sec. 4.1, weight-tied gates) against the fp64 oracle.

The path is floating point throughout: bf16 weights and inputs, fp32 accumulation on the matrix
cores, the hidden activations carried to 16 mantissa bits into the second layer.  Tolerance:
|log beta_gpu - log beta_ref| <= 2e-4 |log beta_ref|: d(log beta)/dz = sigmoid(-z) <= |log beta|, so
the relative error of log beta is at most the absolute error of the gate logit z, and fp32
accumulation over <= 4608 products (about sqrt(n) 2^-24 of the summed magnitudes) plus the 2^-17
split keep that near 1e-5 for the logits of the synthetic gates (|z| < 20); the tests print what
they measure (1e-6 .. 2e-5).
"""
import numpy as np
import pytest
import torch

import kvtrim_inputs as ki
import oracle
import paper_2605_09649_amd as kv
from helpers import bf16_bits

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
RTOL = 2e-4


def run_both(L, H, d_model, d_g, d_p, n_tok, b_g=3.5, layer_begin=0, layer_end=None, horizon=None, salt=0, pick=None):
    """GPU on all n_tok tokens; the oracle on all of them, or on the tokens listed in `pick` (a token's
    gates do not depend on the other tokens of the call) - the GPU rows are then cut to the same list."""
    layer_end = L if layer_end is None else layer_end
    w = ki.gate_weights(L, H, d_model, d_g, d_p, b_g=b_g, seed=1234 + salt)
    x = ki.gate_inputs(L, n_tok, d_model, salt=salt)[layer_begin:layer_end].contiguous()
    og = oracle.Gate(bf16_bits(w["w1"]), w["c1"].numpy(), bf16_bits(w["w2"]), w["c2"].numpy(), w["w_g"].numpy(), b_g)
    x_ref = x if pick is None else x[:, pick].contiguous()
    z_ref, lb_ref, lt_ref = oracle.gate_forward(og, bf16_bits(x_ref), layer_begin, layer_end, horizon)
    ctx = kv.Context(1, L, H, H, 64, 1024)
    gate = kv.Gate.from_dict(w, DEV)
    nl = layer_end - layer_begin
    scratch = torch.empty(kv.kvtrim_gate_scratch_bytes(gate, n_tok, nl) // 4, dtype=torch.float32, device=DEV)
    lb = torch.full((n_tok, L, H), float("nan"), dtype=torch.float32, device=DEV)
    lt = torch.full((n_tok, L, H), float("nan"), dtype=torch.float32, device=DEV) if horizon is not None else None
    kv.kvtrim_gate_forward(ctx, gate, x.to(DEV), n_tok, layer_begin, layer_end, 0 if horizon is None else horizon,
                           scratch, lb, lt)
    assert kv.kvtrim_poll_error(ctx) == 0
    if pick is not None:
        lb = lb[pick]
        lt = None if lt is None else lt[pick]
    return z_ref, lb_ref, lt_ref, lb.cpu().numpy(), None if lt is None else lt.cpu().numpy()


def rel_err(got, ref):
    return float(np.max(np.abs(got.astype(np.float64) - ref) / np.abs(ref)))


@pytest.mark.parametrize("L,H,d_model,d_g,d_p,n_tok", [
    (2, 2, 256, 64, 1, 1),            # smallest legal sizes, scalar projection
    (3, 2, 512, 128, 7, 5),           # d_p not a multiple of the 16-row tile
    (2, 4, 1024, 512, 128, 16),       # the paper's hidden width, one full token tile
    (2, 2, 256, 576, 40, 17),         # hidden width beyond one staged chunk, token tail of one
    (1, 2, 512, 64, 33, 20),          # two token tiles per block
    (1, 2, 512, 64, 33, 64),          # four token tiles in one block
    (1, 2, 512, 64, 33, 150),         # four token tiles per block, three blocks along the tokens, ragged tail
    (2, 2, 256, 192, 16, 300),        # LDS-tiled first layer (hidden width not a multiple of 128): 1.5 row tiles, 2.3 token tiles
    (1, 2, 256, 576, 8, 256),         # ... hidden width above 512
    (1, 1, 1024, 512, 128, 257),      # folded prefill path: the paper's hidden width, one token beyond two 128-token tiles
    (2, 3, 512, 128, 20, 300),        # ... one 16-row tile per wavefront, three heads
    (9, 2, 256, 256, 16, 260),        # ... nine layers: the second round of the layer-to-XCD dealing is partly empty
    (1, 8, 256, 384, 5, 513),         # ... eight heads, three tiles per wavefront, token tail of one
    (3, 2, 256, 512, 1, 256),         # ... exactly two full token tiles, scalar projection
    (2, 2, 512, 128, 9, 129),         # ... just above the switch-over: 32-token blocks, a tail of one
    (2, 2, 256, 512, 16, 300),        # ... the paper's hidden width from the tiled copy of W1 (short rows: the copy fits the scratch)
    (32, 2, 1280, 128, 8, 520),       # ... 64-token blocks (32 layers x 9 tiles), W1 straight from its rows
])
def test_gate_forward_matches_the_oracle(L, H, d_model, d_g, d_p, n_tok):
    z_ref, lb_ref, _, lb, _ = run_both(L, H, d_model, d_g, d_p, n_tok, salt=d_p)
    assert np.isfinite(lb).all() and (lb <= 0).all()
    err = rel_err(lb, lb_ref)
    print(f"max relative error of log beta: {err:.2e} (logits {z_ref.min():.2f} .. {z_ref.max():.2f})")
    assert err <= RTOL


def test_layer_range_leaves_other_layers_alone():
    _, lb_ref, _, lb, _ = run_both(4, 2, 256, 64, 16, 3, layer_begin=1, layer_end=3)
    assert np.isnan(lb[:, 0, :]).all() and np.isnan(lb[:, 3, :]).all()
    assert rel_err(lb[:, 1:3, :], lb_ref[:, 1:3, :]) <= RTOL


@pytest.mark.parametrize("horizon", [1, 2, 5, 0])
def test_horizon_tail_constant(horizon):
    # Eq. global_score: the factor sum_{k<H} beta^k, cached in log form with log beta
    _, lb_ref, lt_ref, lb, lt = run_both(2, 2, 256, 128, 32, 9, b_g=1.0, horizon=horizon)
    assert rel_err(lb, lb_ref) <= RTOL
    assert np.max(np.abs(lt - lt_ref)) <= 1e-3 * np.max(np.abs(lt_ref)) + 1e-6
    if horizon == 1:
        assert np.array_equal(lt, np.zeros_like(lt))


def test_prefill_sized_call_with_a_layer_range_and_a_horizon():
    # the folded path (128 tokens and more): layers outside the range stay untouched, the tail constant follows log beta
    _, lb_ref, lt_ref, lb, lt = run_both(5, 2, 256, 128, 12, 300, b_g=1.0, layer_begin=1, layer_end=4, horizon=2)
    assert np.isnan(lb[:, 0, :]).all() and np.isnan(lb[:, 4, :]).all()
    assert np.isnan(lt[:, 0, :]).all() and np.isnan(lt[:, 4, :]).all()
    assert rel_err(lb[:, 1:4, :], lb_ref[:, 1:4, :]) <= RTOL
    assert np.max(np.abs(lt[:, 1:4, :] - lt_ref[:, 1:4, :])) <= 1e-3 * np.max(np.abs(lt_ref[:, 1:4, :])) + 1e-6


def test_both_paths_agree_across_the_token_threshold():
    # 127 tokens run the per-token kernels, 128 the folded ones: the shared 127 tokens get the same gates to rounding
    L, H, d_model, d_g, d_p = 2, 2, 512, 256, 24
    w = ki.gate_weights(L, H, d_model, d_g, d_p, b_g=3.5, seed=77)
    x = ki.gate_inputs(L, 128, d_model, salt=3)
    og = oracle.Gate(bf16_bits(w["w1"]), w["c1"].numpy(), bf16_bits(w["w2"]), w["c2"].numpy(), w["w_g"].numpy(), 3.5)
    _, lb_ref, _ = oracle.gate_forward(og, bf16_bits(x), 0, L, None)
    ctx = kv.Context(1, L, H, H, 64, 1024)
    gate = kv.Gate.from_dict(w, DEV)
    got = {}
    for n_tok in (127, 128):
        xd = x[:, :n_tok].contiguous().to(DEV)
        scratch = torch.empty(kv.kvtrim_gate_scratch_bytes(gate, n_tok, L) // 4, dtype=torch.float32, device=DEV)
        lb = torch.full((n_tok, L, H), float("nan"), dtype=torch.float32, device=DEV)
        kv.kvtrim_gate_forward(ctx, gate, xd, n_tok, 0, L, 1, scratch, lb, None)
        assert kv.kvtrim_poll_error(ctx) == 0
        got[n_tok] = lb.cpu().numpy()
        assert rel_err(got[n_tok], lb_ref[:n_tok]) <= RTOL
    assert np.max(np.abs(got[127] - got[128][:127]) / np.abs(lb_ref[:127])) <= RTOL


@pytest.mark.parametrize("d_g,n_tok", [(64, 4), (128, 130)])     # per-token kernels; folded kernel
def test_initial_bias_of_eighteen_keeps_beta_next_to_one(d_g, n_tok):
    # Sec. 5.1: b_g starts at 18.0 - log beta is about -1.5e-8 and must not flush to 0 or lose its digits
    z_ref, lb_ref, _, lb, _ = run_both(2, 2, 256, d_g, 16, n_tok, b_g=18.0)
    assert (lb < 0).all() and rel_err(lb, lb_ref) <= 2e-3 * np.max(np.abs(z_ref))   # d(log beta)/log beta = -dz here


def test_full_size_gate_one_token_and_sixteen():
    # the benchmark model: 32 layers x 8 KV heads, d_model 4096, hidden width 512 (Sec. 5.1), d_p 128
    for n_tok in (1, 16):
        z_ref, lb_ref, _, lb, _ = run_both(32, 8, 4096, 512, 128, n_tok, salt=n_tok)
        err = rel_err(lb, lb_ref)
        print(f"n_tok {n_tok}: max relative error of log beta {err:.2e}")
        assert err <= RTOL


def test_full_size_gate_prefill_chunk_on_sampled_tokens():
    # a 2048-token chunk through the benchmark model; the oracle takes 12 of its tokens (tile edges and interiors)
    pick = [0, 1, 15, 16, 127, 128, 1000, 1023, 1024, 1500, 2046, 2047]
    z_ref, lb_ref, _, lb, _ = run_both(32, 8, 4096, 512, 128, 2048, salt=7, pick=pick)
    err = rel_err(lb, lb_ref)
    print(f"2048 tokens, {len(pick)} sampled: max relative error of log beta {err:.2e}")
    assert err <= RTOL


@pytest.mark.parametrize("L,H,d_model,d_g,d_p,n_toks", [
    (3, 2, 256, 64, 7, (1, 5, 20, 150)),          # per-token first layer + dot-product readout; hidden width not for the folded kernel
    (2, 3, 512, 128, 20, (16, 23, 24, 127, 300)),  # across the switch-over at 24 tokens: 32-token blocks read W1 from the prepared tiles
    (32, 2, 1280, 128, 8, (520,)),                 # 64-token blocks from the prepared tiles
    (2, 8, 256, 512, 16, (1, 7, 16, 64, 513, 1100)),   # the paper's hidden width, eight heads: one kernel with the readout inside up to 16 tokens, 128-token blocks
    (2, 17, 256, 64, 4, (3,)),                     # more than 16 heads: the readout's parts do not fit the scratch buffer, two kernels
    (2, 2, 256, 576, 8, (256,)),                   # hidden width above 512: LDS-tiled first layer + dot-product readout
])
def test_prepared_gate_matches_the_oracle_and_is_reusable(L, H, d_model, d_g, d_p, n_toks):
    w = ki.gate_weights(L, H, d_model, d_g, d_p, b_g=3.5, seed=99 + d_p)
    og = oracle.Gate(bf16_bits(w["w1"]), w["c1"].numpy(), bf16_bits(w["w2"]), w["c2"].numpy(), w["w_g"].numpy(), 3.5)
    ctx = kv.Context(1, L, H, H, 64, 1024)
    gate = kv.Gate.from_dict(w, DEV)
    nbytes = kv.kvtrim_gate_prepared_bytes(gate, L, H)
    assert nbytes >= L * d_g * d_model * 2 + L * H * (d_g + 1) * 4
    prepared = torch.empty(nbytes // 4, dtype=torch.float32, device=DEV)
    kv.kvtrim_gate_prepare(ctx, gate, prepared)                   # once; every call below reuses it
    for n_tok in n_toks:
        x = ki.gate_inputs(L, n_tok, d_model, salt=n_tok)
        pick = None if n_tok * L * d_g * d_model < 3e9 else sorted({0, 1, 63, 64, n_tok // 2, n_tok - 1})
        x_ref = x if pick is None else x[:, pick].contiguous()
        for lo, hi in ((0, L), (L // 2, L)):
            _, lb_ref, lt_ref = oracle.gate_forward(og, bf16_bits(x_ref[lo:hi].contiguous()), lo, hi, 2)
            scratch = torch.empty(kv.kvtrim_gate_scratch_bytes(gate, n_tok, hi - lo) // 4, dtype=torch.float32, device=DEV)
            lb = torch.full((n_tok, L, H), float("nan"), dtype=torch.float32, device=DEV)
            lt = torch.full((n_tok, L, H), float("nan"), dtype=torch.float32, device=DEV)
            kv.kvtrim_gate_forward_prepared(ctx, gate, prepared, x[lo:hi].contiguous().to(DEV), n_tok, lo, hi, 2, scratch, lb, lt)
            assert kv.kvtrim_poll_error(ctx) == 0
            if n_tok <= 16:                                       # (the last block of a layer adds the parts of the readout: always in the same order)
                lb2 = torch.full((n_tok, L, H), float("nan"), dtype=torch.float32, device=DEV)
                kv.kvtrim_gate_forward_prepared(ctx, gate, prepared, x[lo:hi].contiguous().to(DEV), n_tok, lo, hi, 2, scratch, lb2, None)
                assert torch.equal(lb[:, lo:hi], lb2[:, lo:hi])
            lb_h, lt_h = lb.cpu().numpy(), lt.cpu().numpy()
            assert np.isnan(lb_h[:, :lo, :]).all()                # layers outside the range stay untouched
            if pick is not None:
                lb_h, lt_h = lb_h[pick], lt_h[pick]
            assert rel_err(lb_h[:, lo:hi], lb_ref[:, lo:hi]) <= RTOL, (n_tok, lo, hi)
            assert np.max(np.abs(lt_h[:, lo:hi] - lt_ref[:, lo:hi])) <= 1e-3 * np.max(np.abs(lt_ref[:, lo:hi])) + 1e-6


def test_host_side_argument_checks_of_the_gate():
    L, H = 2, 2
    w = ki.gate_weights(L, H, 256, 64, 8)
    ctx = kv.Context(1, L, H, H, 64, 1024)
    gate = kv.Gate.from_dict(w, DEV)
    x = ki.gate_inputs(L, 2, 256).to(DEV)
    scratch = torch.empty(2 * L * 64, dtype=torch.float32, device=DEV)
    lb = torch.zeros(2, L, H, dtype=torch.float32, device=DEV)
    with pytest.raises(kv.KvtrimError):
        kv.kvtrim_gate_forward(ctx, gate, x, 0, 0, L, 1, scratch, lb)              # no token
    with pytest.raises(kv.KvtrimError):
        kv.kvtrim_gate_forward(ctx, gate, x, 2, 0, L + 1, 1, scratch, lb)          # layer range beyond the model
    with pytest.raises(kv.KvtrimError):
        kv.kvtrim_gate_forward(ctx, gate, x, 2, 0, L, 5000, scratch, lb)           # horizon out of range
    with pytest.raises(kv.KvtrimError):
        kv.kvtrim_gate_forward(ctx, gate, x, 2, 0, L, 1, None, lb)                 # no scratch
    w_bad = ki.gate_weights(L, H, 128, 64, 8)
    with pytest.raises(kv.KvtrimError):                                            # d_model not a multiple of 256
        kv.kvtrim_gate_forward(ctx, kv.Gate.from_dict(w_bad, DEV), x, 2, 0, L, 1, scratch, lb)
    assert kv.kvtrim_gate_scratch_bytes(gate, 2, L) == 2 * L * 64 * 4
    assert kv.kvtrim_gate_scratch_bytes(gate, 0, L) == 0
    assert kv.kvtrim_gate_prepared_bytes(gate, 0, H) == 0 and kv.kvtrim_gate_prepared_bytes(gate, L, H) > 0
    with pytest.raises(kv.KvtrimError):
        kv.kvtrim_gate_prepare(ctx, gate, None)                                    # no buffer
    prepared = torch.empty(kv.kvtrim_gate_prepared_bytes(gate, L, H) // 4, dtype=torch.float32, device=DEV)
    kv.kvtrim_gate_prepare(ctx, gate, prepared)
    with pytest.raises(kv.KvtrimError):
        kv.kvtrim_gate_forward_prepared(ctx, gate, None, x, 2, 0, L, 1, scratch, lb)   # no prepared buffer
    with pytest.raises(kv.KvtrimError):
        kv.kvtrim_gate_forward_prepared(ctx, gate, prepared, x, 2, 1, 1, 1, scratch, lb)   # empty layer range
    kv.kvtrim_gate_forward_prepared(ctx, gate, prepared, x, 2, 0, L, 1, scratch, lb)
    assert kv.kvtrim_poll_error(ctx) == 0
