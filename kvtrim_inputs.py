"""Seeded synthetic workloads for the kvtrim hot path.

This module only draws random inputs (K/V rows, gate logits turned into
the per-token constants a retention gate hands over when a token is cached,
queries, segment layouts).  It holds none of the hot path's arithmetic (no
score, no selection, no compaction, no attention), so both the GPU path and
the CPU oracle may be fed from it.

The five named workloads have the shapes, value distributions and structure
of the benchmark configurations; every one can be scaled down (shorter
prefill, proportionally smaller budget) for tests.  "N(m, s)" always means
mean m and standard deviation s.  A retention gate emits beta = sigmoid(z)
(Sec. 4.1); the cache stores log(beta) = -log1p(exp(-z)), evaluated in fp64
and rounded once to fp32, and - only when the score's lookahead horizon H is
not 1 - log(sum_{k<H} beta^k), likewise fp64 rounded once to fp32.
"""
from dataclasses import dataclass, replace
from typing import Tuple

import torch

BASE_SEED = 96490


@dataclass(frozen=True)
class Workload:
    name: str
    index: int              # position in the benchmark's list of configurations
    n_seq: int
    n_layers: int
    n_kv_heads: int
    n_q_heads: int
    head_dim: int
    prefill: Tuple[int, ...]   # prefilled tokens per sequence
    budget: Tuple[int, ...]    # global budget (entries) per sequence
    steps: int                 # decode steps
    z_mean: float
    z_std: float
    layer_offset_std: float = 0.0                     # per-layer additive offset on z
    evidence_frac: float = 0.0                        # share of token positions with near-permanent z
    evidence_z: Tuple[float, float] = (8.0, 1.0)
    visual_block: Tuple[int, int] = (0, 0)            # [begin, end) positions of the visual tokens
    visual_z: Tuple[float, float] = (1.5, 2.0)
    seed_index: int = 0                               # which of several seeded repetitions of the workload this is

    @property
    def nseg(self):
        return self.n_seq * self.n_layers * self.n_kv_heads

    @property
    def group(self):
        return self.n_q_heads // self.n_kv_heads

    @property
    def seed(self):
        return BASE_SEED + self.index + 1000 * self.seed_index

    def seg_id(self, seq, layer, head):
        return (seq * self.n_layers + layer) * self.n_kv_heads + head


def workload(name: str, prefill: int = None, seed_index: int = 0) -> Workload:
    """One of 'tiny', 'llama', 'long', 'vlm', 'multiturn'.  `prefill` overrides the
    prefilled length (budget fractions are kept) to scale a workload down; `seed_index` > 0 gives
    another draw of every random input of the same recipe."""
    if name == "tiny":
        T = prefill or 2048
        w = Workload("tiny", 0, 1, 4, 4, 8, 64, (T,), (max(1, T // 2),), 16, 3.0, 1.5)
    elif name == "llama":
        T = prefill or 32768
        w = Workload("llama", 1, 1, 32, 8, 32, 128, (T,), (32 * 8 * T // 8,), 256, 3.0, 1.5,
                     layer_offset_std=0.5)
    elif name == "long":
        T = prefill or 131072
        w = Workload("long", 2, 1, 32, 8, 32, 128, (T,), (32 * 8 * T // 16,), 128, 3.5, 1.5,
                     evidence_frac=0.02)
    elif name == "vlm":
        T = prefill or 20480
        vb = (T // 20, T // 20 + T // 5)            # 1024 .. 5120 at full size
        w = Workload("vlm", 3, 2, 28, 4, 28, 128, (T, T), (28 * 4 * T // 10,) * 2, 256, 3.0, 1.5,
                     visual_block=vb)
    elif name == "multiturn":
        lo, hi = (4096, 65536) if prefill is None else (max(1, prefill // 16), prefill)
        g = torch.Generator().manual_seed(BASE_SEED + 4)
        lens = tuple(int(x) for x in torch.randint(lo, hi + 1, (16,), generator=g))
        per_head = 8192 if prefill is None else max(1, prefill // 8)
        w = Workload("multiturn", 4, 16, 32, 8, 32, 128, lens, (per_head * 32 * 8,) * 16, 64, 3.0, 1.5)
    else:
        raise ValueError(name)
    return replace(w, seed_index=seed_index) if seed_index else w


def _gen(w: Workload, device, *salt):
    seed = w.seed
    for s in salt:
        seed = (seed * 1000003 + int(s) + 12345) % (2 ** 62)
    return torch.Generator(device=device).manual_seed(seed)


def _log_beta_of_z(z64: torch.Tensor) -> torch.Tensor:
    return (-torch.log1p(torch.exp(-z64))).to(torch.float32)


def log_tail_of(log_beta: torch.Tensor, horizon: int) -> torch.Tensor:
    """The per-token constant that comes with log(beta) when the lookahead horizon of the score is
    H = `horizon` > 1 (0 means the limit H -> infinity): log(sum_{k<H} beta^k), evaluated in fp64 and
    rounded once to fp32 (Sec. 4.2, Eq. global_score: the factor (1 - beta^H) / (1 - beta))."""
    lb = log_beta.to(torch.float64)
    beta = torch.exp(lb)
    if horizon <= 0:
        return (-torch.log1p(-beta)).to(torch.float32)
    total = torch.zeros_like(beta)
    term = torch.ones_like(beta)
    for _ in range(int(horizon)):
        total += term
        term = term * beta
    return torch.log(total).to(torch.float32)


def prefill_log_beta(w: Workload, seq: int, device="cpu") -> torch.Tensor:
    """log(beta) of the prefilled tokens of one sequence, fp32 [L*Hkv, T]."""
    T = w.prefill[seq]
    LH = w.n_layers * w.n_kv_heads
    g = _gen(w, device, 1, seq)
    z = torch.randn(LH, T, generator=g, device=device, dtype=torch.float64) * w.z_std + w.z_mean
    if w.layer_offset_std > 0:
        off = torch.randn(w.n_layers, generator=_gen(w, device, 2, seq), device=device, dtype=torch.float64)
        z += (off * w.layer_offset_std).repeat_interleave(w.n_kv_heads)[:, None]
    if w.evidence_frac > 0:
        ge = _gen(w, device, 3, seq)
        is_ev = torch.rand(T, generator=ge, device=device) < w.evidence_frac     # shared by all (layer, head)
        zev = torch.randn(LH, T, generator=ge, device=device, dtype=torch.float64) * w.evidence_z[1] \
            + w.evidence_z[0]
        z = torch.where(is_ev[None, :], zev, z)
    vb, ve = w.visual_block
    if ve > vb:
        gv = _gen(w, device, 4, seq)
        zv = torch.randn(LH, ve - vb, generator=gv, device=device, dtype=torch.float64) * w.visual_z[1] \
            + w.visual_z[0]
        z[:, vb:ve] = zv
    return _log_beta_of_z(z)


def rows(w: Workload, n: int, device, *salt) -> torch.Tensor:
    """n bf16 rows of N(0,1), [n, D]."""
    g = _gen(w, device, 5, *salt)
    return torch.randn(n, w.head_dim, generator=g, device=device, dtype=torch.float32).to(torch.bfloat16)


def decode_inputs(w: Workload, step: int, device="cpu", horizon: int = 1):
    """Inputs of decode step `step` (0-based): one new token per segment and one query per head
    (plus the horizon tail constant of the new tokens when horizon != 1)."""
    g = _gen(w, device, 6, step)
    nseg, D = w.nseg, w.head_dim
    k_new = torch.randn(nseg, D, generator=g, device=device, dtype=torch.float32).to(torch.bfloat16)
    v_new = torch.randn(nseg, D, generator=g, device=device, dtype=torch.float32).to(torch.bfloat16)
    z = torch.randn(nseg, generator=g, device=device, dtype=torch.float64) * w.z_std + w.z_mean
    q = torch.randn(w.n_seq, w.n_layers, w.n_q_heads, D, generator=g, device=device,
                    dtype=torch.float32).to(torch.bfloat16)
    d = {"k_new": k_new, "v_new": v_new, "log_beta_new": _log_beta_of_z(z), "q": q}
    if horizon != 1:
        d["log_tail_new"] = log_tail_of(d["log_beta_new"], horizon)
    return d


def alloc_cache(w: Workload, cap: int, device="cpu"):
    """Empty ragged cache (dict of tensors) with room for `cap` entries."""
    D = w.head_dim
    return {
        "k": torch.zeros(cap, D, dtype=torch.bfloat16, device=device),
        "v": torch.zeros(cap, D, dtype=torch.bfloat16, device=device),
        "log_beta": torch.zeros(cap, dtype=torch.float32, device=device),
        "pos": torch.zeros(cap, dtype=torch.int32, device=device),
        "seg_start": torch.zeros(w.nseg, dtype=torch.int64, device=device),
        "seg_len": torch.zeros(w.nseg, dtype=torch.int32, device=device),
        "cap": cap,
    }


def with_horizon(cache: dict, horizon: int) -> dict:
    """Adds the per-entry horizon tail constant to a cache made by prefill_cache / ragged_cache."""
    if horizon != 1:
        cache = dict(cache)
        cache["log_tail"] = log_tail_of(cache["log_beta"], horizon)
    return cache


def prefill_cache(w: Workload, reserve: int = 1, device="cpu"):
    """Ragged cache holding every prefilled token of every segment, positions 0..T-1,
    each segment followed by `reserve` free slots.  Generated segment-group by
    segment-group so that the peak extra memory stays at one layer's rows."""
    LH = w.n_layers * w.n_kv_heads
    cap = sum((T + reserve) * LH for T in w.prefill)
    c = alloc_cache(w, cap, device)
    cursor = 0
    starts, lens = [], []
    for seq in range(w.n_seq):
        T = w.prefill[seq]
        lb = prefill_log_beta(w, seq, device)
        pos = torch.arange(T, dtype=torch.int32, device=device)
        for layer in range(w.n_layers):
            for head in range(w.n_kv_heads):
                lh = layer * w.n_kv_heads + head
                c["k"][cursor:cursor + T] = rows(w, T, device, 0, seq, lh)
                c["v"][cursor:cursor + T] = rows(w, T, device, 1, seq, lh)
                c["log_beta"][cursor:cursor + T] = lb[lh]
                c["pos"][cursor:cursor + T] = pos
                starts.append(cursor)
                lens.append(T)
                cursor += T + reserve
        del lb
    c["seg_start"].copy_(torch.tensor(starts, dtype=torch.int64))
    c["seg_len"].copy_(torch.tensor(lens, dtype=torch.int32))
    return c


def ragged_cache(w: Workload, seg_len, reserve: int = 1, device="cpu", salt: int = 0, pos_stride_max: int = 3):
    """Ragged cache with the given per-segment lengths (any int sequence of size nseg):
    rows N(0,1), log(beta) from the workload's base z distribution, positions strictly
    ascending with random gaps (as after earlier evictions).  Returns (cache, now) where
    now[seq] is larger than every position of that sequence."""
    seg_len = [int(x) for x in seg_len]
    assert len(seg_len) == w.nseg
    cap = sum(seg_len) + reserve * w.nseg
    c = alloc_cache(w, max(cap, 1), device)
    g = _gen(w, device, 7, salt)
    n = sum(seg_len)
    c["k"][:] = torch.randn(c["k"].shape, generator=g, device=device, dtype=torch.float32).to(torch.bfloat16)
    c["v"][:] = torch.randn(c["v"].shape, generator=g, device=device, dtype=torch.float32).to(torch.bfloat16)
    z = torch.randn(c["cap"], generator=g, device=device, dtype=torch.float64) * w.z_std + w.z_mean
    c["log_beta"][:] = _log_beta_of_z(z)
    starts, cursor = [], 0
    now = [0] * w.n_seq
    per_seq = w.n_layers * w.n_kv_heads
    for gidx, ln in enumerate(seg_len):
        starts.append(cursor)
        if ln > 0:
            gaps = torch.randint(1, pos_stride_max + 1, (ln,), generator=g, device=device)
            p = torch.cumsum(gaps, 0).to(torch.int32) - 1
            c["pos"][cursor:cursor + ln] = p
            now[gidx // per_seq] = max(now[gidx // per_seq], int(p[-1]) + 1)
        cursor += ln + reserve
    c["seg_start"].copy_(torch.tensor(starts, dtype=torch.int64))
    c["seg_len"].copy_(torch.tensor(seg_len, dtype=torch.int32))
    del n
    return c, torch.tensor(now, dtype=torch.int32, device=device)


def gate_weights(n_layers: int, n_kv_heads: int, d_model: int, d_g: int = 512, d_p: int = 128, b_g: float = 3.5,
                 z_std: float = 1.5, device="cpu", seed: int = BASE_SEED + 77):
    """Random weights of a retention gate (Sec. 4.1; hidden width d_g = 512 as in Sec. 5.1).  No trained
    gate is available, so the weights are drawn: W1 ~ N(0, 1/d_model), W2 ~ N(0, 1/d_g), biases N(0, 0.1),
    and the tied readout w_g ~ N(0, s^2/d_p) with s chosen so that, for N(0,1) inputs, the gate logit has
    roughly the spread z_std around b_g that the workloads' z distributions have.  W1, W2 are bf16,
    the rest fp32.  Returns a dict of tensors (+ 'b_g')."""
    g = torch.Generator(device=device).manual_seed(seed)
    rn = lambda *shape: torch.randn(*shape, generator=g, device=device, dtype=torch.float32)
    w1 = (rn(n_layers, d_g, d_model) / d_model ** 0.5).to(torch.bfloat16)
    c1 = rn(n_layers, d_g) * 0.1
    w2 = (rn(n_layers, n_kv_heads, d_p, d_g) / d_g ** 0.5).to(torch.bfloat16)
    c2 = rn(n_layers, n_kv_heads, d_p) * 0.1
    w_g = rn(d_p) * (z_std / 0.6) / d_p ** 0.5
    return {"w1": w1, "c1": c1, "w2": w2, "c2": c2, "w_g": w_g, "b_g": float(b_g)}


def gate_inputs(n_layers: int, n_tok: int, d_model: int, device="cpu", salt: int = 0):
    """Token representations entering each transformer block, bf16 [n_layers][n_tok][d_model], N(0,1)."""
    g = torch.Generator(device=device).manual_seed(BASE_SEED + 78 + 1000003 * int(salt))
    return torch.randn(n_layers, n_tok, d_model, generator=g, device=device, dtype=torch.float32).to(torch.bfloat16)


def chunk_inputs(w: Workload, n_tok: int, device="cpu", *salt):
    """n_tok new tokens for every segment (a prefill chunk): K, V bf16 [nseg][n_tok][D] ~ N(0,1) and
    log(beta) fp32 [nseg][n_tok] from the workload's base z distribution."""
    g = _gen(w, device, 8, *salt)
    nseg, D = w.nseg, w.head_dim
    k = torch.randn(nseg, n_tok, D, generator=g, device=device, dtype=torch.float32).to(torch.bfloat16)
    v = torch.randn(nseg, n_tok, D, generator=g, device=device, dtype=torch.float32).to(torch.bfloat16)
    z = torch.randn(nseg, n_tok, generator=g, device=device, dtype=torch.float64) * w.z_std + w.z_mean
    return {"k_new": k, "v_new": v, "log_beta_new": _log_beta_of_z(z)}
