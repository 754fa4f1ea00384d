"""ctypes binding of the C oracle; numpy arrays in, numpy arrays out.

The arithmetic lives in ``kvtrim_oracle.c``; this file only marshals arguments.
"""
import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "kvtrim_oracle.c")
_SO = os.path.join(_HERE, "libkvtrim_oracle.so")
_lib = None


def build(force=False):
    """Compile the oracle with gcc (plain C, no contraction, OpenMP over segments in attend)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-fopenmp",
               "-Wall", "-Wextra", "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
        # the sanitizer driver (tests build it again with -fsanitize=address,undefined); here just "does it compile"
        subprocess.run(["gcc", "-O1", "-std=c11", "-ffp-contract=off", "-fopenmp", "-Wall", "-Wextra", "-o",
                        os.path.join(_HERE, "selftest_bin"), os.path.join(_HERE, "selftest.c"), "-lm"], check=True)
    return _SO


class _CShape(C.Structure):
    _fields_ = [("n_seq", C.c_int32), ("n_layers", C.c_int32), ("n_kv_heads", C.c_int32),
                ("n_q_heads", C.c_int32), ("head_dim", C.c_int32)]


class _CCache(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p), ("log_beta", C.c_void_p), ("pos", C.c_void_p),
                ("seg_start", C.c_void_p), ("seg_len", C.c_void_p), ("cap", C.c_int64), ("log_tail", C.c_void_p)]


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_SO)
        _lib.kvo_key_of_score.restype = C.c_uint32
        _lib.kvo_key_of_score.argtypes = [C.c_float]
        _lib.kvo_threads.restype = C.c_int
        for name in ("kvo_select", "kvo_compact", "kvo_append"):
            getattr(_lib, name).restype = C.c_int
    return _lib


@dataclass(frozen=True)
class Shape:
    n_seq: int
    n_layers: int
    n_kv_heads: int
    n_q_heads: int
    head_dim: int

    @property
    def nseg(self):
        return self.n_seq * self.n_layers * self.n_kv_heads

    @property
    def group(self):
        return self.n_q_heads // self.n_kv_heads

    def c(self):
        return _CShape(self.n_seq, self.n_layers, self.n_kv_heads, self.n_q_heads, self.head_dim)


class HostCache:
    """Ragged cache in host memory.  k, v hold bf16 bit patterns as uint16."""

    def __init__(self, shape, cap, with_rows=True, with_tail=False):
        self.shape = shape
        self.cap = int(cap)
        self.log_tail = np.zeros(self.cap, np.float32) if with_tail else None
        D = shape.head_dim
        rows = self.cap if with_rows else 0          # metadata-only caches serve score / select
        self.k = np.zeros((rows, D), np.uint16)
        self.v = np.zeros((rows, D), np.uint16)
        self.log_beta = np.zeros(self.cap, np.float32)
        self.pos = np.zeros(self.cap, np.int32)
        self.seg_start = np.zeros(shape.nseg, np.int64)
        self.seg_len = np.zeros(shape.nseg, np.int32)

    @classmethod
    def from_arrays(cls, shape, k, v, log_beta, pos, seg_start, seg_len, log_tail=None):
        self = cls.__new__(cls)
        self.log_tail = None if log_tail is None else np.ascontiguousarray(log_tail, np.float32)
        self.shape = shape
        self.cap = int(log_beta.shape[0])
        self.k = np.ascontiguousarray(k, np.uint16).reshape(-1, shape.head_dim)
        self.v = np.ascontiguousarray(v, np.uint16).reshape(-1, shape.head_dim)
        self.log_beta = np.ascontiguousarray(log_beta, np.float32)
        self.pos = np.ascontiguousarray(pos, np.int32)
        self.seg_start = np.ascontiguousarray(seg_start, np.int64)
        self.seg_len = np.ascontiguousarray(seg_len, np.int32)
        return self

    def c(self):
        p = lambda a: a.ctypes.data_as(C.c_void_p)
        return _CCache(p(self.k), p(self.v), p(self.log_beta), p(self.pos), p(self.seg_start),
                       p(self.seg_len), self.cap, None if self.log_tail is None else p(self.log_tail))

    def entry_index(self):
        """Flat indices of every live entry, in (segment, position) order."""
        return np.concatenate([np.arange(s, s + n, dtype=np.int64)
                               for s, n in zip(self.seg_start, self.seg_len)] or [np.zeros(0, np.int64)])


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def threads():
    return int(lib().kvo_threads())


def set_threads(n):
    """Threads the oracle's attention loop uses from now on (its other stages always run on one)."""
    lib().kvo_set_threads(C.c_int(int(n)))


def key_of_score(s):
    return int(lib().kvo_key_of_score(C.c_float(float(s))))


def score(cache, now):
    now = np.ascontiguousarray(now, np.int32)
    out = np.zeros(cache.cap, np.float32)
    sh, cc = cache.shape.c(), cache.c()
    lib().kvo_score(C.byref(sh), C.byref(cc), _p(now), _p(out))
    return out


def score_horizon(cache, now, horizon):
    now = np.ascontiguousarray(now, np.int32)
    out = np.zeros(cache.cap, np.float64)
    sh, cc = cache.shape.c(), cache.c()
    lib().kvo_score_horizon(C.byref(sh), C.byref(cc), _p(now), C.c_int32(int(horizon)), _p(out))
    return out


def select(cache, score_arr, budget):
    score_arr = np.ascontiguousarray(score_arr, np.float32)
    budget = np.ascontiguousarray(budget, np.int64)
    assert budget.shape == (cache.shape.n_seq,)
    keep = np.zeros(cache.cap, np.uint8)
    kept = np.zeros(cache.shape.nseg, np.int32)
    thr = np.zeros(cache.shape.n_seq, np.uint32)
    sh, cc = cache.shape.c(), cache.c()
    rc = lib().kvo_select(C.byref(sh), C.byref(cc), _p(score_arr), _p(budget), _p(keep), _p(kept), _p(thr))
    if rc != 0:
        raise MemoryError("oracle select: out of memory")
    return keep, kept, thr


def compact(src, keep, dst_cap, reserve):
    keep = np.ascontiguousarray(keep, np.uint8)
    dst = HostCache(src.shape, dst_cap, with_tail=src.log_tail is not None)
    sh, cs, cd = src.shape.c(), src.c(), dst.c()
    rc = lib().kvo_compact(C.byref(sh), C.byref(cs), _p(keep), C.byref(cd), C.c_int32(int(reserve)))
    if rc != 0:
        raise OverflowError("oracle compact: destination capacity too small")
    return dst


def attend(cache, q, scale, layer_begin=0, layer_end=None, want_lse=True, soft_now=None):
    """Hard-eviction attention; with soft_now (int32 [n_seq]) the retention-gated soft form."""
    sh = cache.shape
    if layer_end is None:
        layer_end = sh.n_layers
    q = np.ascontiguousarray(q, np.uint16).reshape(sh.n_seq, sh.n_layers, sh.n_q_heads, sh.head_dim)
    out = np.zeros((sh.n_seq, sh.n_layers, sh.n_q_heads, sh.head_dim), np.float64)
    lse = np.zeros((sh.n_seq, sh.n_layers, sh.n_q_heads), np.float64)
    csh, cc = sh.c(), cache.c()
    if soft_now is None:
        lib().kvo_attend(C.byref(csh), C.byref(cc), _p(q), C.c_int32(layer_begin), C.c_int32(layer_end),
                         C.c_double(float(scale)), _p(out), _p(lse) if want_lse else None)
    else:
        now = np.ascontiguousarray(soft_now, np.int32)
        lib().kvo_attend_soft(C.byref(csh), C.byref(cc), _p(q), _p(now), C.c_int32(layer_begin),
                              C.c_int32(layer_end), C.c_double(float(scale)), _p(out), _p(lse) if want_lse else None)
    return out, lse


def occupancy(cache, now):
    now = np.ascontiguousarray(now, np.int32)
    occ = np.zeros(cache.shape.n_seq, np.float64)
    sh, cc = cache.shape.c(), cache.c()
    lib().kvo_occupancy(C.byref(sh), C.byref(cc), _p(now), _p(occ))
    return occ


def append(cache, k_new, v_new, log_beta_new, pos_new, log_tail_new=None):
    sh = cache.shape
    log_beta_new = np.ascontiguousarray(log_beta_new, np.float32).reshape(sh.nseg, -1)
    n_new = log_beta_new.shape[1]
    k_new = np.ascontiguousarray(k_new, np.uint16).reshape(sh.nseg, n_new, sh.head_dim)
    v_new = np.ascontiguousarray(v_new, np.uint16).reshape(sh.nseg, n_new, sh.head_dim)
    pos_new = np.ascontiguousarray(pos_new, np.int32).reshape(sh.nseg, n_new)
    if cache.log_tail is not None:
        assert log_tail_new is not None, "this cache carries a horizon tail: log_tail_new is required"
        log_tail_new = np.ascontiguousarray(log_tail_new, np.float32).reshape(sh.nseg, n_new)
    else:
        log_tail_new = None
    csh, cc = sh.c(), cache.c()
    rc = lib().kvo_append(C.byref(csh), C.byref(cc), _p(k_new), _p(v_new), _p(log_beta_new),
                          None if log_tail_new is None else _p(log_tail_new), _p(pos_new), C.c_int32(n_new))
    if rc != 0:
        raise OverflowError("oracle append: no room in a segment")


class _CGate(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("n_heads", C.c_int32), ("d_model", C.c_int32), ("d_g", C.c_int32),
                ("d_p", C.c_int32), ("w1", C.c_void_p), ("c1", C.c_void_p), ("w2", C.c_void_p), ("c2", C.c_void_p),
                ("w_g", C.c_void_p), ("b_g", C.c_float)]


class Gate:
    """Weights of the retention gate in host memory: w1 uint16 (bf16 bits) [L][d_g][d_model], c1 fp32 [L][d_g],
    w2 uint16 [L][H][d_p][d_g], c2 fp32 [L][H][d_p], w_g fp32 [d_p], b_g."""

    def __init__(self, w1, c1, w2, c2, w_g, b_g):
        self.w1 = np.ascontiguousarray(w1, np.uint16)
        self.c1 = np.ascontiguousarray(c1, np.float32)
        self.w2 = np.ascontiguousarray(w2, np.uint16)
        self.c2 = np.ascontiguousarray(c2, np.float32)
        self.w_g = np.ascontiguousarray(w_g, np.float32)
        self.b_g = float(b_g)
        self.n_layers, self.d_g, self.d_model = self.w1.shape
        _, self.n_heads, self.d_p, dg = self.w2.shape
        assert self.w2.shape[0] == self.n_layers and dg == self.d_g
        assert self.c1.shape == (self.n_layers, self.d_g) and self.c2.shape == (self.n_layers, self.n_heads, self.d_p)
        assert self.w_g.shape == (self.d_p,)

    def c(self):
        return _CGate(self.n_layers, self.n_heads, self.d_model, self.d_g, self.d_p, _p(self.w1), _p(self.c1),
                      _p(self.w2), _p(self.c2), _p(self.w_g), self.b_g)


def gate_forward(gate, x, layer_begin=0, layer_end=None, horizon=None):
    """x: uint16 (bf16 bits) [layer_end - layer_begin][n_tok][d_model].  Returns (z, log_beta, log_tail), fp64
    [n_tok][L][H]; rows of layers outside the range are NaN; log_tail is None unless a horizon is given."""
    layer_end = gate.n_layers if layer_end is None else layer_end
    x = np.ascontiguousarray(x, np.uint16)
    nl, n_tok, dm = x.shape
    assert nl == layer_end - layer_begin and dm == gate.d_model
    shape = (n_tok, gate.n_layers, gate.n_heads)
    z = np.full(shape, np.nan)
    lb = np.full(shape, np.nan)
    lt = None if horizon is None else np.full(shape, np.nan)
    cg = gate.c()
    lib().kvo_gate_forward(C.byref(cg), _p(x), C.c_int32(n_tok), C.c_int32(layer_begin), C.c_int32(layer_end),
                           C.c_int32(0 if horizon is None else horizon), _p(z), _p(lb), None if lt is None else _p(lt))
    return z, lb, lt
