"""Glue shared by the tests: moves the generated inputs to the oracle's host container."""
import numpy as np
import torch

import oracle


def shape_of(w):
    return oracle.Shape(w.n_seq, w.n_layers, w.n_kv_heads, w.n_q_heads, w.head_dim)


def bf16_bits(t):
    """bf16 tensor -> numpy uint16 bit patterns (host)."""
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def bits_to_f64(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def host_cache(w, c):
    """dict of tensors (as made by kvtrim_inputs) -> oracle.HostCache holding the same bytes."""
    return oracle.HostCache.from_arrays(
        shape_of(w), bf16_bits(c["k"]).copy(), bf16_bits(c["v"]).copy(),
        c["log_beta"].cpu().numpy().copy(), c["pos"].cpu().numpy().copy(),
        c["seg_start"].cpu().numpy().copy(), c["seg_len"].cpu().numpy().copy(),
        log_tail=None if c.get("log_tail") is None else c["log_tail"].cpu().numpy().copy())


def live_mask(hc):
    m = np.zeros(hc.cap, bool)
    for s, n in zip(hc.seg_start, hc.seg_len):
        m[s:s + n] = True
    return m


def paper_constants():
    """The values the paper prints that tests refer to (tests/golden/paper_constants.txt)."""
    import os
    out = {}
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "paper_constants.txt")) as f:
        for line in f:
            line = line.split("#")[0].split()
            if line:
                vals = [float(v) if "." in v else int(v) for v in line[1:]]
                out[line[0]] = vals[0] if len(vals) == 1 else vals
    return out
