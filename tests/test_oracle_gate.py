"""Pins of the oracle's retention gate (Sec. 4.1, weight-tied gates): the nested sums written in C
are checked against torch's own fp64 linear / silu / logsigmoid routines on non-square shapes,
against closed forms, and against the invariants the definition implies."""
import numpy as np
import torch
import torch.nn.functional as F

import kvtrim_inputs as ki
import oracle
from helpers import bf16_bits, paper_constants

PAPER = paper_constants()


def make_gate(L=3, H=2, d_model=48, d_g=20, d_p=7, b_g=0.75, seed=1):
    w = ki.gate_weights(L, H, d_model, d_g, d_p, b_g=b_g, seed=seed)
    return w, oracle.Gate(bf16_bits(w["w1"]), w["c1"].numpy(), bf16_bits(w["w2"]), w["c2"].numpy(), w["w_g"].numpy(),
                          w["b_g"])


def torch_gate(w, x, layer):
    """fp64 reference from library routines only; x bf16 [n_tok][d_model] -> z [n_tok][H]."""
    u = F.silu(F.linear(x.double(), w["w1"][layer].double(), w["c1"][layer].double()))
    zs = []
    for h in range(w["w2"].shape[1]):
        p = F.linear(u, w["w2"][layer, h].double(), w["c2"][layer, h].double())
        zs.append(p @ w["w_g"].double() + w["b_g"])
    return torch.stack(zs, 1)


def test_matches_torch_fp64_on_non_square_shapes_and_layer_ranges():
    w, g = make_gate()
    x = ki.gate_inputs(3, 5, 48)
    z, lb, _ = oracle.gate_forward(g, bf16_bits(x))
    for layer in range(3):
        zt = torch_gate(w, x[layer], layer)
        assert np.allclose(z[:, layer, :], zt.numpy(), rtol=1e-12, atol=1e-12)
        assert np.allclose(lb[:, layer, :], F.logsigmoid(zt).numpy(), rtol=1e-12, atol=1e-15)
    z12, lb12, _ = oracle.gate_forward(g, bf16_bits(x[1:3]), layer_begin=1, layer_end=3)
    assert np.isnan(z12[:, 0, :]).all() and np.array_equal(z12[:, 1:, :], z[:, 1:, :])
    assert np.array_equal(lb12[:, 1:, :], lb[:, 1:, :])


def test_zero_projection_gives_the_tied_bias_alone():
    # Sec. 5.1: b_g starts at 18.0; with Proj = 0 every gate is sigmoid(18)
    assert PAPER["gate_bias_init"] == 18.0
    w, _ = make_gate(b_g=PAPER["gate_bias_init"])
    for name in ("w1", "c1", "c2"):
        w[name] = torch.zeros_like(w[name])
    g = oracle.Gate(bf16_bits(w["w1"]), w["c1"].numpy(), bf16_bits(w["w2"]), w["c2"].numpy(), w["w_g"].numpy(),
                    PAPER["gate_bias_init"])
    z, lb, _ = oracle.gate_forward(g, bf16_bits(ki.gate_inputs(3, 4, 48)))
    assert np.array_equal(z, np.full_like(z, 18.0))
    e = 1.0
    for _ in range(18):
        e *= 0.36787944117144233                     # e^-1
    expect = -(e - e * e / 2 + e ** 3 / 3)           # -log(1 + e^-18) by its series
    assert np.allclose(lb, expect, rtol=1e-12, atol=0)
    assert abs(expect + 1.5229979e-8) < 1e-14


def test_the_readout_is_shared_by_all_layers_and_heads():
    w, g = make_gate()
    # the same Proj parameters in (layer 0, head 1) and (layer 2, head 0), the same token in both layers
    w["w1"][2] = w["w1"][0]
    w["c1"][2] = w["c1"][0]
    w["w2"][2, 0] = w["w2"][0, 1]
    w["c2"][2, 0] = w["c2"][0, 1]
    x = ki.gate_inputs(3, 4, 48)
    x[2] = x[0]
    mk = lambda b: oracle.Gate(bf16_bits(w["w1"]), w["c1"].numpy(), bf16_bits(w["w2"]), w["c2"].numpy(),
                               w["w_g"].numpy(), b)
    z, lb, _ = oracle.gate_forward(mk(0.75), bf16_bits(x))
    assert np.array_equal(z[:, 2, 0], z[:, 0, 1]) and np.array_equal(lb[:, 2, 0], lb[:, 0, 1])
    assert not np.array_equal(z[:, 0, 0], z[:, 0, 1])
    # one bias for all: moving b_g moves every logit by the same amount
    z2, lb2, _ = oracle.gate_forward(mk(2.0), bf16_bits(x))
    assert np.allclose(z2 - z, 1.25, rtol=0, atol=1e-12)
    assert (lb2 > lb).all()


def test_hidden_units_and_projection_units_can_be_permuted():
    w, g = make_gate()
    x = bf16_bits(ki.gate_inputs(3, 6, 48))
    z, _, _ = oracle.gate_forward(g, x)
    rng = np.random.default_rng(0)
    pg, pp = rng.permutation(20), rng.permutation(7)
    w1 = bf16_bits(w["w1"])[:, pg, :]
    c1 = w["c1"].numpy()[:, pg]
    w2 = bf16_bits(w["w2"])[:, :, :, pg][:, :, pp, :]
    c2 = w["c2"].numpy()[:, :, pp]
    g2 = oracle.Gate(w1, c1, w2, c2, w["w_g"].numpy()[pp], w["b_g"])
    z2, _, _ = oracle.gate_forward(g2, x)
    assert np.allclose(z2, z, rtol=0, atol=1e-12) and not np.array_equal(pg, np.arange(20))


def test_a_layer_sees_only_its_own_input_and_a_token_only_itself():
    w, g = make_gate()
    x = ki.gate_inputs(3, 4, 48)
    z, _, _ = oracle.gate_forward(g, bf16_bits(x))
    y = x.clone()
    y[1, 2] = -y[1, 2]
    z2, _, _ = oracle.gate_forward(g, bf16_bits(y))
    same = np.ones(z.shape, bool)
    same[2, 1, :] = False
    assert np.array_equal(z2[same], z[same]) and (z2[~same] != z[~same]).all()


def test_log_beta_is_stable_at_both_ends_and_ordered_like_the_logit():
    w, _ = make_gate()
    for name in ("w1", "c1", "c2"):
        w[name] = torch.zeros_like(w[name])
    x = bf16_bits(ki.gate_inputs(3, 2, 48))
    prev = -np.inf
    for b in (-800.0, -50.0, -1.0, 0.0, 1.0, 18.0, 50.0, 800.0):
        g = oracle.Gate(bf16_bits(w["w1"]), w["c1"].numpy(), bf16_bits(w["w2"]), w["c2"].numpy(), w["w_g"].numpy(), b)
        _, lb, _ = oracle.gate_forward(g, x)
        v = lb[0, 0, 0]
        assert np.isfinite(v) and v <= 0.0 and v >= prev and np.all(lb == v)
        prev = v
        if b <= -50:
            assert abs(v - b) < 1e-15 * abs(b) + 1e-20       # log sigmoid(z) -> z
        if b == 0.0:
            assert abs(v + 0.6931471805599453) < 1e-15
    assert prev == 0.0                                        # beta = 1 to fp64 at z = 800


def test_horizon_tail_matches_the_series_and_the_cached_constant_of_the_score():
    w, g = make_gate(b_g=1.0)
    x = bf16_bits(ki.gate_inputs(3, 5, 48))
    _, lb, lt1 = oracle.gate_forward(g, x, horizon=1)
    assert np.array_equal(lt1, np.zeros_like(lt1))
    beta = np.exp(lb)
    assert PAPER["inference_horizon"] in PAPER["ablation_horizons"]
    for H in PAPER["ablation_horizons"][1:]:
        _, _, lt = oracle.gate_forward(g, x, horizon=H)
        direct = np.log(sum(beta ** k for k in range(H)))
        assert np.allclose(lt, direct, rtol=1e-13, atol=1e-15)
        # the constant the score stage caches per entry (rounded once to fp32 from the fp32 log beta)
        cached = ki.log_tail_of(torch.from_numpy(lb.astype(np.float32)), H).numpy()
        assert np.allclose(lt, cached, rtol=3e-7, atol=1e-7)
    _, _, lt_inf = oracle.gate_forward(g, x, horizon=0)
    assert np.allclose(lt_inf, -np.log1p(-beta), rtol=1e-12)
    assert np.allclose(np.log1p(beta), oracle.gate_forward(g, x, horizon=2)[2], rtol=1e-13)


def test_synthetic_gate_has_the_spread_of_the_workload_logits():
    w = ki.gate_weights(4, 2, 256, PAPER["gate_hidden_width"], 128, b_g=3.5)
    g = oracle.Gate(bf16_bits(w["w1"]), w["c1"].numpy(), bf16_bits(w["w2"]), w["c2"].numpy(), w["w_g"].numpy(), 3.5)
    z, lb, _ = oracle.gate_forward(g, bf16_bits(ki.gate_inputs(4, 64, 256)))
    assert abs(z.mean() - 3.5) < 1.0 and 0.8 < z.std() < 2.5
    assert (lb < 0).all()


def test_second_layer_and_readout_collapse_to_one_vector_per_gate():
    # Sec. 4.1 as read here has no nonlinearity between the second layer of Proj and the tied readout, so
    # z = w_g . (W2 u + c2) + b_g = (W2^T w_g) . u + (w_g . c2 + b_g) exactly.  The HIP path uses this for long
    # calls; here the oracle's nested sums are checked against the collapsed form written with library routines.
    w, g = make_gate(L=2, H=3, d_model=64, d_g=24, d_p=9, b_g=-0.375, seed=5)
    x = ki.gate_inputs(2, 6, 64, salt=2)
    z, _, _ = oracle.gate_forward(g, bf16_bits(x))
    for layer in range(2):
        u = F.silu(F.linear(x[layer].double(), w["w1"][layer].double(), w["c1"][layer].double()))
        for h in range(3):
            v = w["w2"][layer, h].double().T @ w["w_g"].double()
            s = w["w_g"].double() @ w["c2"][layer, h].double() + w["b_g"]
            assert np.allclose(z[:, layer, h], (u @ v + s).numpy(), rtol=1e-12, atol=1e-12)
