"""Host-side check of the arithmetic claim behind P.V on the matrix cores: a probability p in [0, 1] enters as two
bf16 terms, hi = bf16(p) and lo = bf16(p - hi), both rounded to nearest even; the part that is lost, p - hi - lo, is
at most 2^-16 of p (in fact 2^-18: two roundings to 8 significant bits), so with bf16 V and fp32 sums the product
P.V differs from the exact one by far less than the attention tolerance of 5e-3."""
import numpy as np
import torch


def split(p):
    hi = p.to(torch.bfloat16).to(torch.float32)
    lo = (p - hi).to(torch.bfloat16).to(torch.float32)
    return hi, lo


def test_two_bf16_terms_carry_a_probability_to_sixteen_bits():
    g = torch.Generator().manual_seed(5)
    p = torch.cat([torch.rand(1 << 20, generator=g), torch.exp2(-30.0 * torch.rand(1 << 20, generator=g)),
                   torch.tensor([0.0, 1.0, 0.5, 1.0 - 2.0 ** -24, 2.0 ** -126, 3.0 * 2.0 ** -140])]).to(torch.float32)
    hi, lo = split(p)
    lost = (p.double() - hi.double() - lo.double()).abs()
    assert bool(torch.all(lost <= p.double() * 2.0 ** -16 + 2.0 ** -130))   # (the absolute term: bf16 subnormals)
    big = p >= 2.0 ** -100
    assert float((lost[big] / p.double()[big]).max()) <= 2.0 ** -17
    assert bool(torch.all((p - hi).double() == p.double() - hi.double()))     # the remainder is exact in fp32


def test_weighted_sum_with_split_probabilities_stays_far_inside_the_tolerance():
    rng = np.random.default_rng(11)
    n, d = 4096, 64
    z = rng.normal(0.0, 3.0, n)
    p = np.exp(z - z.max()).astype(np.float32)
    v = torch.from_numpy(rng.normal(0.0, 1.0, (n, d)).astype(np.float32)).to(torch.bfloat16).to(torch.float32).numpy()
    hi, lo = (t.numpy().astype(np.float64) for t in split(torch.from_numpy(p)))
    exact = (p.astype(np.float64)[:, None] * v).sum(0) / p.astype(np.float64).sum()
    got = ((hi + lo)[:, None] * v).sum(0) / p.astype(np.float64).sum()
    assert np.abs(got - exact).max() / np.abs(exact).max() <= 1e-5
