"""ctypes binding of libkvtrim.so.  PyTorch tensors only provide device memory and the stream."""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libkvtrim.so")
_lib = None

STATUS = {0: "KVTRIM_OK", -1: "KVTRIM_EINVAL", -2: "KVTRIM_ENOMEM", -3: "KVTRIM_EHIP", -4: "KVTRIM_ECAP",
          -5: "KVTRIM_EMISMATCH", -6: "KVTRIM_ELAYOUT"}

EXPORTS = ["kvtrim_create", "kvtrim_destroy", "kvtrim_workspace_bytes", "kvtrim_last_error",
           "kvtrim_poll_error", "kvtrim_score", "kvtrim_select_global", "kvtrim_score_select", "kvtrim_select_path_counts", "kvtrim_compact",
           "kvtrim_decode_attn", "kvtrim_decode_attn_soft", "kvtrim_occupancy", "kvtrim_compact_attn", "kvtrim_min_room", "kvtrim_compact_inplace", "kvtrim_compact_attn_inplace", "kvtrim_append", "kvtrim_append_compact", "kvtrim_decode_step", "kvtrim_decode_step_inplace",
           "kvtrim_paged_build", "kvtrim_paged_append", "kvtrim_paged_score", "kvtrim_paged_select", "kvtrim_paged_score_select", "kvtrim_paged_decode_step",
           "kvtrim_paged_evict", "kvtrim_paged_defrag", "kvtrim_paged_attn", "kvtrim_gate_scratch_bytes", "kvtrim_gate_forward", "kvtrim_gate_prepared_bytes", "kvtrim_gate_prepare",
           "kvtrim_gate_forward_prepared",
           "kvtrim_select_global_noalloc",
           "kvtrim_profile_begin", "kvtrim_profile_end",
           "kvtrim_kernel_name"]
PAGE_SIZE = 128
N_KERNELS = 40


class KvtrimError(RuntimeError):
    def __init__(self, status, text=""):
        self.status = status
        super().__init__(f"{STATUS.get(status, status)} {text}".strip())


class _Config(C.Structure):
    _fields_ = [("n_seq", C.c_int32), ("n_layers", C.c_int32), ("n_kv_heads", C.c_int32),
                ("n_q_heads", C.c_int32), ("head_dim", C.c_int32), ("max_entries", C.c_int64)]


class _Cache(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p), ("log_beta", C.c_void_p), ("pos", C.c_void_p),
                ("seg_start", C.c_void_p), ("seg_len", C.c_void_p), ("cap_entries", C.c_int64),
                ("log_tail", C.c_void_p)]


class _PagedCache(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p), ("log_beta", C.c_void_p), ("pos", C.c_void_p),
                ("log_tail", C.c_void_p), ("block_table", C.c_void_p), ("seg_pages", C.c_void_p),
                ("seg_live", C.c_void_p), ("page_owner", C.c_void_p), ("page_live", C.c_void_p),
                ("free_list", C.c_void_p), ("n_free", C.c_void_p), ("n_pages", C.c_int32),
                ("max_pages_per_seg", C.c_int32)]


class _Gate(C.Structure):
    _fields_ = [("d_model", C.c_int32), ("d_g", C.c_int32), ("d_p", C.c_int32), ("w1", C.c_void_p), ("c1", C.c_void_p),
                ("w2", C.c_void_p), ("c2", C.c_void_p), ("w_g", C.c_void_p), ("b_g", C.c_float)]


def library_path():
    return _LIB_PATH


def load_library():
    """Loads libkvtrim.so; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError(f"{_LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'`")
        lib = C.CDLL(_LIB_PATH)
        lib.kvtrim_create.argtypes = [C.POINTER(C.c_void_p), C.POINTER(_Config)]
        lib.kvtrim_destroy.argtypes = [C.c_void_p]
        lib.kvtrim_workspace_bytes.argtypes = [C.POINTER(_Config)]
        lib.kvtrim_workspace_bytes.restype = C.c_size_t
        lib.kvtrim_last_error.argtypes = [C.c_void_p]
        lib.kvtrim_last_error.restype = C.c_char_p
        lib.kvtrim_poll_error.argtypes = [C.c_void_p, C.c_void_p]
        lib.kvtrim_score.argtypes = [C.c_void_p, C.POINTER(_Cache), C.c_void_p, C.c_void_p, C.c_void_p]
        lib.kvtrim_select_global.argtypes = [C.c_void_p, C.POINTER(_Cache), C.c_void_p, C.c_void_p, C.c_void_p,
                                             C.c_void_p, C.c_void_p, C.c_void_p]
        lib.kvtrim_score_select.argtypes = [C.c_void_p, C.POINTER(_Cache), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                            C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
        lib.kvtrim_select_path_counts.argtypes = [C.c_void_p, C.POINTER(C.c_int64), C.POINTER(C.c_int64), C.c_void_p]
        lib.kvtrim_compact.argtypes = [C.c_void_p, C.POINTER(_Cache), C.c_void_p, C.c_void_p, C.POINTER(_Cache),
                                       C.c_int32, C.c_void_p]
        lib.kvtrim_decode_attn.argtypes = [C.c_void_p, C.POINTER(_Cache), C.c_void_p, C.c_int32, C.c_int32,
                                           C.c_float, C.c_void_p, C.c_void_p, C.c_void_p]
        lib.kvtrim_decode_attn_soft.argtypes = [C.c_void_p, C.POINTER(_Cache), C.c_void_p, C.c_void_p, C.c_int32,
                                                C.c_int32, C.c_float, C.c_void_p, C.c_void_p, C.c_void_p]
        lib.kvtrim_occupancy.argtypes = [C.c_void_p, C.POINTER(_Cache), C.c_void_p, C.c_void_p, C.c_void_p]
        lib.kvtrim_compact_attn.argtypes = [C.c_void_p, C.POINTER(_Cache), C.c_void_p, C.c_void_p, C.POINTER(_Cache),
                                            C.c_int32, C.c_void_p, C.c_int32, C.c_int32, C.c_float, C.c_void_p,
                                            C.c_void_p, C.c_void_p]
        lib.kvtrim_min_room.argtypes = [C.c_void_p, C.POINTER(_Cache), C.c_void_p, C.c_void_p]
        lib.kvtrim_compact_inplace.argtypes = [C.c_void_p, C.POINTER(_Cache), C.c_void_p, C.c_void_p, C.POINTER(_Cache), C.c_void_p]
        lib.kvtrim_compact_attn_inplace.argtypes = [C.c_void_p, C.POINTER(_Cache), C.c_void_p, C.c_void_p, C.POINTER(_Cache),
                                                    C.c_void_p, C.c_int32, C.c_int32, C.c_float, C.c_void_p, C.c_void_p,
                                                    C.c_void_p]
        lib.kvtrim_append.argtypes = [C.c_void_p, C.POINTER(_Cache), C.c_void_p, C.c_void_p, C.c_void_p,
                                      C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]
        lib.kvtrim_append_compact.argtypes = [C.c_void_p, C.POINTER(_Cache), C.c_void_p, C.c_void_p, C.c_void_p,
                                              C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                              C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(_Cache), C.c_int32, C.c_void_p]
        lib.kvtrim_decode_step.argtypes = [C.c_void_p, C.POINTER(_Cache), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                           C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                           C.c_void_p, C.POINTER(_Cache), C.c_int32, C.c_void_p, C.c_int32, C.c_int32,
                                           C.c_float, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
        lib.kvtrim_decode_step_inplace.argtypes = [C.c_void_p, C.POINTER(_Cache), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                                   C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                                   C.c_void_p, C.c_void_p, C.POINTER(_Cache), C.c_void_p, C.c_int32, C.c_int32,
                                                   C.c_float, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
        P = C.POINTER(_PagedCache)
        lib.kvtrim_paged_build.argtypes = [C.c_void_p, C.POINTER(_Cache), C.c_void_p, C.c_void_p, P, C.c_void_p]
        lib.kvtrim_paged_append.argtypes = [C.c_void_p, P, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                            C.c_int32, C.c_void_p]
        lib.kvtrim_paged_score.argtypes = [C.c_void_p, P, C.c_void_p, C.c_void_p, C.c_void_p]
        lib.kvtrim_paged_select.argtypes = [C.c_void_p, P, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                            C.c_void_p]
        lib.kvtrim_paged_score_select.argtypes = [C.c_void_p, P, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                                  C.c_void_p, C.c_int64, C.c_void_p]
        lib.kvtrim_paged_decode_step.argtypes = [C.c_void_p, P] + [C.c_void_p] * 12 + [C.c_int32, C.c_int32, C.c_float, C.c_void_p,
                                                 C.c_void_p, C.c_int64, C.c_void_p]
        lib.kvtrim_paged_evict.argtypes = [C.c_void_p, P, C.c_void_p, C.c_void_p]
        lib.kvtrim_paged_defrag.argtypes = [C.c_void_p, P, C.c_void_p]
        lib.kvtrim_paged_attn.argtypes = [C.c_void_p, P, C.c_void_p, C.c_int32, C.c_int32, C.c_float, C.c_void_p,
                                          C.c_void_p, C.c_void_p]
        lib.kvtrim_gate_scratch_bytes.argtypes = [C.POINTER(_Gate), C.c_int32, C.c_int32]
        lib.kvtrim_gate_scratch_bytes.restype = C.c_size_t
        lib.kvtrim_gate_forward.argtypes = [C.c_void_p, C.POINTER(_Gate), C.c_void_p, C.c_int32, C.c_int32, C.c_int32,
                                            C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        lib.kvtrim_gate_prepared_bytes.argtypes = [C.POINTER(_Gate), C.c_int32, C.c_int32]
        lib.kvtrim_gate_prepared_bytes.restype = C.c_size_t
        lib.kvtrim_gate_prepare.argtypes = [C.c_void_p, C.POINTER(_Gate), C.c_void_p, C.c_void_p]
        lib.kvtrim_gate_forward_prepared.argtypes = [C.c_void_p, C.POINTER(_Gate), C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                                     C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        lib.kvtrim_select_global_noalloc.argtypes = [C.POINTER(_Config), C.POINTER(_Cache), C.c_void_p, C.c_void_p,
                                                     C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        lib.kvtrim_profile_begin.argtypes = [C.c_void_p, C.c_uint64]
        lib.kvtrim_profile_end.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
        lib.kvtrim_kernel_name.argtypes = [C.c_int32]
        lib.kvtrim_kernel_name.restype = C.c_char_p
        for name in EXPORTS:
            if name not in ("kvtrim_workspace_bytes", "kvtrim_last_error", "kvtrim_kernel_name",
                            "kvtrim_gate_scratch_bytes", "kvtrim_gate_prepared_bytes"):
                getattr(lib, name).restype = C.c_int
        _lib = lib
    return _lib


def _config(n_seq, n_layers, n_kv_heads, n_q_heads, head_dim, max_entries):
    return _Config(n_seq, n_layers, n_kv_heads, n_q_heads, head_dim, max_entries)


def kvtrim_workspace_bytes(n_seq, n_layers, n_kv_heads, n_q_heads, head_dim, max_entries):
    cfg = _config(n_seq, n_layers, n_kv_heads, n_q_heads, head_dim, max_entries)
    return int(load_library().kvtrim_workspace_bytes(C.byref(cfg)))


def _ptr(t, dtype=None):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device-resident contiguous tensor required"
    if dtype is not None:
        assert t.dtype == dtype, (t.dtype, dtype)
    return C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


class Cache:
    """Ragged cache: device tensors plus the C view of them."""

    def __init__(self, k, v, log_beta, pos, seg_start, seg_len, log_tail=None):
        self.k, self.v, self.log_beta, self.pos, self.seg_start, self.seg_len = k, v, log_beta, pos, seg_start, seg_len
        self.log_tail = log_tail
        self.cap = int(log_beta.shape[0])
        self.c = _Cache(_ptr(k, torch.bfloat16).value, _ptr(v, torch.bfloat16).value,
                        _ptr(log_beta, torch.float32).value, _ptr(pos, torch.int32).value,
                        _ptr(seg_start, torch.int64).value, _ptr(seg_len, torch.int32).value, self.cap,
                        None if log_tail is None else _ptr(log_tail, torch.float32).value)

    @classmethod
    def from_dict(cls, d, device="cuda"):
        t = {n: d[n].to(device) for n in ("k", "v", "log_beta", "pos", "seg_start", "seg_len")}
        if d.get("log_tail") is not None:
            t["log_tail"] = d["log_tail"].to(device)
        return cls(**t)

    @classmethod
    def empty(cls, nseg, head_dim, cap, device="cuda", with_tail=False):
        return cls(torch.zeros(cap, head_dim, dtype=torch.bfloat16, device=device),
                   torch.zeros(cap, head_dim, dtype=torch.bfloat16, device=device),
                   torch.zeros(cap, dtype=torch.float32, device=device),
                   torch.zeros(cap, dtype=torch.int32, device=device),
                   torch.zeros(nseg, dtype=torch.int64, device=device),
                   torch.zeros(nseg, dtype=torch.int32, device=device),
                   torch.zeros(cap, dtype=torch.float32, device=device) if with_tail else None)


class PagedCache:
    """Paged cache: a pool of PAGE_SIZE-slot pages, block tables and the free-page stack (device
    tensors) plus the C view of them.  kvtrim_paged_build fills in the bookkeeping."""

    def __init__(self, nseg, head_dim, n_pages, max_pages_per_seg, device="cuda", with_tail=False):
        n = n_pages * PAGE_SIZE
        i32 = dict(dtype=torch.int32, device=device)
        self.n_pages, self.max_pages_per_seg, self.nseg = int(n_pages), int(max_pages_per_seg), int(nseg)
        self.k = torch.zeros(n, head_dim, dtype=torch.bfloat16, device=device)
        self.v = torch.zeros(n, head_dim, dtype=torch.bfloat16, device=device)
        self.log_beta = torch.zeros(n, dtype=torch.float32, device=device)
        self.pos = torch.full((n,), -1, **i32)
        self.log_tail = torch.zeros(n, dtype=torch.float32, device=device) if with_tail else None
        self.block_table = torch.zeros(nseg, max_pages_per_seg, **i32)
        self.seg_pages = torch.zeros(nseg, **i32)
        self.seg_live = torch.zeros(nseg, **i32)
        self.page_owner = torch.full((n_pages,), -1, **i32)
        self.page_live = torch.zeros(n_pages, **i32)
        self.free_list = torch.zeros(n_pages, **i32)
        self.n_free = torch.zeros(1, **i32)
        self.slots = n
        self.c = _PagedCache(_ptr(self.k).value, _ptr(self.v).value, _ptr(self.log_beta).value, _ptr(self.pos).value,
                             None if self.log_tail is None else _ptr(self.log_tail).value,
                             _ptr(self.block_table).value, _ptr(self.seg_pages).value, _ptr(self.seg_live).value,
                             _ptr(self.page_owner).value, _ptr(self.page_live).value, _ptr(self.free_list).value,
                             _ptr(self.n_free).value, self.n_pages, self.max_pages_per_seg)


class Gate:
    """Retention-gate weights on the device (tensors as made by kvtrim_inputs.gate_weights) plus the C view."""

    def __init__(self, w1, c1, w2, c2, w_g, b_g):
        self.w1, self.c1, self.w2, self.c2, self.w_g, self.b_g = w1, c1, w2, c2, w_g, float(b_g)
        self.n_layers, self.d_g, self.d_model = w1.shape
        self.n_heads, self.d_p = w2.shape[1], w2.shape[2]
        self.c = _Gate(self.d_model, self.d_g, self.d_p, _ptr(w1, torch.bfloat16).value, _ptr(c1, torch.float32).value,
                       _ptr(w2, torch.bfloat16).value, _ptr(c2, torch.float32).value, _ptr(w_g, torch.float32).value,
                       self.b_g)

    @classmethod
    def from_dict(cls, d, device="cuda"):
        return cls(*(d[n].to(device).contiguous() for n in ("w1", "c1", "w2", "c2", "w_g")), d["b_g"])


class Context:
    """Owns a kvtrim_ctx (the library's workspace on the current device)."""

    def __init__(self, n_seq, n_layers, n_kv_heads, n_q_heads, head_dim, max_entries):
        lib = load_library()
        if not torch.cuda.is_available():
            raise RuntimeError("kvtrim needs a GPU: there is no CPU fallback")
        torch.cuda.init()
        self.shape = (n_seq, n_layers, n_kv_heads, n_q_heads, head_dim)
        self.nseg = n_seq * n_layers * n_kv_heads
        self.max_entries = int(max_entries)
        cfg = _config(n_seq, n_layers, n_kv_heads, n_q_heads, head_dim, max_entries)
        h = C.c_void_p()
        rc = lib.kvtrim_create(C.byref(h), C.byref(cfg))
        if rc != 0:
            raise KvtrimError(rc, (lib.kvtrim_last_error(None) or b"kvtrim_create").decode())
        self.handle = h

    def close(self):
        if getattr(self, "handle", None):
            load_library().kvtrim_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def last_error(self):
        return load_library().kvtrim_last_error(self.handle).decode()


def _check(ctx, rc, what):
    if rc != 0:
        raise KvtrimError(rc, f"{what}: {ctx.last_error()}")


def kvtrim_poll_error(ctx, stream=None):
    """Synchronises the stream; returns the status code of the sticky device flag (0 = OK)."""
    return int(load_library().kvtrim_poll_error(ctx.handle, _stream(stream)))


def kvtrim_score(ctx, cache, now, score_out, stream=None):
    _check(ctx, load_library().kvtrim_score(ctx.handle, C.byref(cache.c), _ptr(now, torch.int32),
                                            _ptr(score_out, torch.float32), _stream(stream)), "kvtrim_score")


def kvtrim_select_global(ctx, cache, score, budget, keep_out, kept_out, thr_key_out=None, stream=None):
    _check(ctx, load_library().kvtrim_select_global(
        ctx.handle, C.byref(cache.c), _ptr(score, torch.float32), _ptr(budget, torch.int64),
        _ptr(keep_out, torch.uint8), _ptr(kept_out, torch.int32), _ptr(thr_key_out), _stream(stream)),
        "kvtrim_select_global")


def kvtrim_score_select(ctx, cache, now, budget, score_out, keep_out, kept_out, thr_key_out=None, evict_hint=0, stream=None):
    _check(ctx, load_library().kvtrim_score_select(
        ctx.handle, C.byref(cache.c), _ptr(now, torch.int32), _ptr(budget, torch.int64), _ptr(score_out, torch.float32),
        _ptr(keep_out, torch.uint8), _ptr(kept_out, torch.int32), _ptr(thr_key_out), int(evict_hint), _stream(stream)),
        "kvtrim_score_select")


def kvtrim_select_path_counts(ctx, stream=None):
    """(selections resolved from the candidate list, selections resolved by the single-block fallback)."""
    a, b = C.c_int64(), C.c_int64()
    _check(ctx, load_library().kvtrim_select_path_counts(ctx.handle, C.byref(a), C.byref(b), _stream(stream)),
           "kvtrim_select_path_counts")
    return int(a.value), int(b.value)


def kvtrim_select_global_noalloc(config, cache, score, budget, keep_out, kept_out, thr_key_out=None, status_out=None,
                                 stream=None):
    """config: (n_seq, n_layers, n_kv_heads, n_q_heads, head_dim, max_entries); no context is involved."""
    cfg = _config(*config)
    rc = load_library().kvtrim_select_global_noalloc(
        C.byref(cfg), C.byref(cache.c), _ptr(score, torch.float32), _ptr(budget, torch.int64),
        _ptr(keep_out, torch.uint8), _ptr(kept_out, torch.int32), _ptr(thr_key_out), _ptr(status_out, torch.int32),
        _stream(stream))
    if rc != 0:
        raise KvtrimError(rc, "kvtrim_select_global_noalloc")


def kvtrim_compact(ctx, src, keep, kept, dst, reserve, stream=None):
    _check(ctx, load_library().kvtrim_compact(ctx.handle, C.byref(src.c), _ptr(keep, torch.uint8),
                                              _ptr(kept, torch.int32), C.byref(dst.c), int(reserve),
                                              _stream(stream)), "kvtrim_compact")


def kvtrim_decode_attn(ctx, cache, q, layer_begin, layer_end, softmax_scale, out, lse=None, stream=None):
    _check(ctx, load_library().kvtrim_decode_attn(ctx.handle, C.byref(cache.c), _ptr(q, torch.bfloat16),
                                                  int(layer_begin), int(layer_end), float(softmax_scale),
                                                  _ptr(out, torch.float32), _ptr(lse, torch.float32),
                                                  _stream(stream)), "kvtrim_decode_attn")


def kvtrim_decode_attn_soft(ctx, cache, q, now, layer_begin, layer_end, softmax_scale, out, lse=None, stream=None):
    _check(ctx, load_library().kvtrim_decode_attn_soft(
        ctx.handle, C.byref(cache.c), _ptr(q, torch.bfloat16), _ptr(now, torch.int32), int(layer_begin),
        int(layer_end), float(softmax_scale), _ptr(out, torch.float32), _ptr(lse, torch.float32), _stream(stream)),
        "kvtrim_decode_attn_soft")


def kvtrim_occupancy(ctx, cache, now, occ_out, stream=None):
    _check(ctx, load_library().kvtrim_occupancy(ctx.handle, C.byref(cache.c), _ptr(now, torch.int32),
                                                _ptr(occ_out, torch.float64), _stream(stream)), "kvtrim_occupancy")


def kvtrim_compact_attn(ctx, src, keep, kept, dst, reserve, q, layer_begin, layer_end, softmax_scale, out, lse=None,
                        stream=None):
    _check(ctx, load_library().kvtrim_compact_attn(
        ctx.handle, C.byref(src.c), _ptr(keep, torch.uint8), _ptr(kept, torch.int32), C.byref(dst.c), int(reserve),
        _ptr(q, torch.bfloat16), int(layer_begin), int(layer_end), float(softmax_scale), _ptr(out, torch.float32),
        _ptr(lse, torch.float32), _stream(stream)), "kvtrim_compact_attn")


def kvtrim_min_room(ctx, cache, min_room_out, stream=None):
    _check(ctx, load_library().kvtrim_min_room(ctx.handle, C.byref(cache.c), _ptr(min_room_out, torch.int32), _stream(stream)),
           "kvtrim_min_room")


def kvtrim_compact_inplace(ctx, cache, keep, kept, spare, stream=None):
    _check(ctx, load_library().kvtrim_compact_inplace(ctx.handle, C.byref(cache.c), _ptr(keep, torch.uint8),
                                                      _ptr(kept, torch.int32), C.byref(spare.c), _stream(stream)),
           "kvtrim_compact_inplace")


def kvtrim_compact_attn_inplace(ctx, cache, keep, kept, spare, q, layer_begin, layer_end, softmax_scale, out, lse=None,
                                stream=None):
    _check(ctx, load_library().kvtrim_compact_attn_inplace(
        ctx.handle, C.byref(cache.c), _ptr(keep, torch.uint8), _ptr(kept, torch.int32), C.byref(spare.c),
        _ptr(q, torch.bfloat16), int(layer_begin), int(layer_end), float(softmax_scale), _ptr(out, torch.float32),
        _ptr(lse, torch.float32), _stream(stream)), "kvtrim_compact_attn_inplace")


def kvtrim_append(ctx, cache, k_new, v_new, log_beta_new, pos_new, n_new, log_tail_new=None, stream=None):
    _check(ctx, load_library().kvtrim_append(ctx.handle, C.byref(cache.c), _ptr(k_new, torch.bfloat16),
                                             _ptr(v_new, torch.bfloat16), _ptr(log_beta_new, torch.float32),
                                             _ptr(log_tail_new, torch.float32), _ptr(pos_new, torch.int32),
                                             int(n_new), _stream(stream)),
           "kvtrim_append")


def kvtrim_append_compact(ctx, src, k_new, v_new, log_beta_new, pos_new, n_new, now, budget, score_out, keep_out,
                          kept_out, dst, reserve, thr_key_out=None, log_tail_new=None, stream=None):
    _check(ctx, load_library().kvtrim_append_compact(
        ctx.handle, C.byref(src.c), _ptr(k_new, torch.bfloat16), _ptr(v_new, torch.bfloat16),
        _ptr(log_beta_new, torch.float32), _ptr(log_tail_new, torch.float32), _ptr(pos_new, torch.int32), int(n_new),
        _ptr(now, torch.int32), _ptr(budget, torch.int64), _ptr(score_out, torch.float32), _ptr(keep_out, torch.uint8),
        _ptr(kept_out, torch.int32), _ptr(thr_key_out), C.byref(dst.c), int(reserve), _stream(stream)),
        "kvtrim_append_compact")


def kvtrim_decode_step(ctx, src, k_new, v_new, log_beta_new, pos_new, n_new, now, budget, score_out, keep_out, kept_out, dst,
                       reserve, q, layer_begin, layer_end, softmax_scale, out, lse=None, thr_key_out=None, log_tail_new=None,
                       evict_hint=0, stream=None):
    _check(ctx, load_library().kvtrim_decode_step(
        ctx.handle, C.byref(src.c), _ptr(k_new, torch.bfloat16), _ptr(v_new, torch.bfloat16),
        _ptr(log_beta_new, torch.float32), _ptr(log_tail_new, torch.float32), _ptr(pos_new, torch.int32), int(n_new),
        _ptr(now, torch.int32), _ptr(budget, torch.int64), _ptr(score_out, torch.float32), _ptr(keep_out, torch.uint8),
        _ptr(kept_out, torch.int32), _ptr(thr_key_out), C.byref(dst.c), int(reserve), _ptr(q, torch.bfloat16),
        int(layer_begin), int(layer_end), float(softmax_scale), _ptr(out, torch.float32), _ptr(lse, torch.float32),
        int(evict_hint), _stream(stream)), "kvtrim_decode_step")


def kvtrim_decode_step_inplace(ctx, cache, k_new, v_new, log_beta_new, pos_new, n_new, now, budget, score_out, keep_out,
                               kept_out, spare, q, layer_begin, layer_end, softmax_scale, out, lse=None, thr_key_out=None,
                               log_tail_new=None, evict_hint=0, stream=None):
    _check(ctx, load_library().kvtrim_decode_step_inplace(
        ctx.handle, C.byref(cache.c), _ptr(k_new, torch.bfloat16), _ptr(v_new, torch.bfloat16),
        _ptr(log_beta_new, torch.float32), _ptr(log_tail_new, torch.float32), _ptr(pos_new, torch.int32), int(n_new),
        _ptr(now, torch.int32), _ptr(budget, torch.int64), _ptr(score_out, torch.float32), _ptr(keep_out, torch.uint8),
        _ptr(kept_out, torch.int32), _ptr(thr_key_out), C.byref(spare.c), _ptr(q, torch.bfloat16),
        int(layer_begin), int(layer_end), float(softmax_scale), _ptr(out, torch.float32), _ptr(lse, torch.float32),
        int(evict_hint), _stream(stream)), "kvtrim_decode_step_inplace")


def kvtrim_paged_build(ctx, src, keep, kept, dst, stream=None):
    _check(ctx, load_library().kvtrim_paged_build(ctx.handle, C.byref(src.c), _ptr(keep, torch.uint8),
                                                  _ptr(kept, torch.int32), C.byref(dst.c), _stream(stream)),
           "kvtrim_paged_build")


def kvtrim_paged_append(ctx, cache, k_new, v_new, log_beta_new, pos_new, log_tail_new=None, n_new=1, stream=None):
    _check(ctx, load_library().kvtrim_paged_append(
        ctx.handle, C.byref(cache.c), _ptr(k_new, torch.bfloat16), _ptr(v_new, torch.bfloat16),
        _ptr(log_beta_new, torch.float32), _ptr(log_tail_new, torch.float32), _ptr(pos_new, torch.int32),
        int(n_new), _stream(stream)), "kvtrim_paged_append")


def kvtrim_paged_score(ctx, cache, now, score_out, stream=None):
    _check(ctx, load_library().kvtrim_paged_score(ctx.handle, C.byref(cache.c), _ptr(now, torch.int32),
                                                  _ptr(score_out, torch.float32), _stream(stream)),
           "kvtrim_paged_score")


def kvtrim_paged_score_select(ctx, cache, now, budget, score_out, keep_out, kept_out, thr_key_out=None, evict_hint=0, stream=None):
    _check(ctx, load_library().kvtrim_paged_score_select(
        ctx.handle, C.byref(cache.c), _ptr(now, torch.int32), _ptr(budget, torch.int64), _ptr(score_out, torch.float32),
        _ptr(keep_out, torch.uint8), _ptr(kept_out, torch.int32), _ptr(thr_key_out), int(evict_hint), _stream(stream)),
        "kvtrim_paged_score_select")


def kvtrim_paged_decode_step(ctx, cache, k_new, v_new, log_beta_new, pos_new, now, budget, score_out, keep_out, kept_out, q,
                             layer_begin, layer_end, softmax_scale, out, lse=None, thr_key_out=None, log_tail_new=None,
                             evict_hint=0, stream=None):
    _check(ctx, load_library().kvtrim_paged_decode_step(
        ctx.handle, C.byref(cache.c), _ptr(k_new, torch.bfloat16), _ptr(v_new, torch.bfloat16),
        _ptr(log_beta_new, torch.float32), _ptr(log_tail_new, torch.float32), _ptr(pos_new, torch.int32),
        _ptr(now, torch.int32), _ptr(budget, torch.int64), _ptr(score_out, torch.float32), _ptr(keep_out, torch.uint8),
        _ptr(kept_out, torch.int32), _ptr(thr_key_out), _ptr(q, torch.bfloat16), int(layer_begin), int(layer_end),
        float(softmax_scale), _ptr(out, torch.float32), _ptr(lse, torch.float32), int(evict_hint), _stream(stream)),
        "kvtrim_paged_decode_step")


def kvtrim_paged_select(ctx, cache, score, budget, keep_out, kept_out, thr_key_out=None, stream=None):
    _check(ctx, load_library().kvtrim_paged_select(
        ctx.handle, C.byref(cache.c), _ptr(score, torch.float32), _ptr(budget, torch.int64),
        _ptr(keep_out, torch.uint8), _ptr(kept_out, torch.int32), _ptr(thr_key_out), _stream(stream)),
        "kvtrim_paged_select")


def kvtrim_paged_evict(ctx, cache, keep, stream=None):
    _check(ctx, load_library().kvtrim_paged_evict(ctx.handle, C.byref(cache.c), _ptr(keep, torch.uint8),
                                                  _stream(stream)), "kvtrim_paged_evict")


def kvtrim_paged_defrag(ctx, cache, stream=None):
    _check(ctx, load_library().kvtrim_paged_defrag(ctx.handle, C.byref(cache.c), _stream(stream)), "kvtrim_paged_defrag")


def kvtrim_paged_attn(ctx, cache, q, layer_begin, layer_end, softmax_scale, out, lse=None, stream=None):
    _check(ctx, load_library().kvtrim_paged_attn(ctx.handle, C.byref(cache.c), _ptr(q, torch.bfloat16),
                                                 int(layer_begin), int(layer_end), float(softmax_scale),
                                                 _ptr(out, torch.float32), _ptr(lse, torch.float32),
                                                 _stream(stream)), "kvtrim_paged_attn")


def kvtrim_gate_scratch_bytes(gate, n_tok, n_layers):
    return int(load_library().kvtrim_gate_scratch_bytes(C.byref(gate.c), int(n_tok), int(n_layers)))


def kvtrim_gate_forward(ctx, gate, x, n_tok, layer_begin, layer_end, horizon, scratch, log_beta_out, log_tail_out=None,
                        stream=None):
    _check(ctx, load_library().kvtrim_gate_forward(
        ctx.handle, C.byref(gate.c), _ptr(x, torch.bfloat16), int(n_tok), int(layer_begin), int(layer_end), int(horizon),
        _ptr(scratch), _ptr(log_beta_out, torch.float32), _ptr(log_tail_out, torch.float32), _stream(stream)),
        "kvtrim_gate_forward")


def kvtrim_gate_prepared_bytes(gate, n_layers, n_kv_heads):
    return int(load_library().kvtrim_gate_prepared_bytes(C.byref(gate.c), int(n_layers), int(n_kv_heads)))


def kvtrim_gate_prepare(ctx, gate, prepared, stream=None):
    _check(ctx, load_library().kvtrim_gate_prepare(ctx.handle, C.byref(gate.c), _ptr(prepared), _stream(stream)),
           "kvtrim_gate_prepare")


def kvtrim_gate_forward_prepared(ctx, gate, prepared, x, n_tok, layer_begin, layer_end, horizon, scratch, log_beta_out,
                                 log_tail_out=None, stream=None):
    _check(ctx, load_library().kvtrim_gate_forward_prepared(
        ctx.handle, C.byref(gate.c), _ptr(prepared), _ptr(x, torch.bfloat16), int(n_tok), int(layer_begin), int(layer_end),
        int(horizon), _ptr(scratch), _ptr(log_beta_out, torch.float32), _ptr(log_tail_out, torch.float32), _stream(stream)),
        "kvtrim_gate_forward_prepared")


def kvtrim_kernel_name(kernel_id):
    n = load_library().kvtrim_kernel_name(int(kernel_id))
    return n.decode() if n else None


def kvtrim_profile_begin(ctx, kernel_mask):
    _check(ctx, load_library().kvtrim_profile_begin(ctx.handle, int(kernel_mask)), "kvtrim_profile_begin")


def kvtrim_profile_end(ctx, stream=None):
    """Returns {kernel name: (summed ms, bracketed launches)} for the kernels that were launched."""
    ms = (C.c_double * N_KERNELS)()
    n = (C.c_int64 * N_KERNELS)()
    _check(ctx, load_library().kvtrim_profile_end(ctx.handle, _stream(stream), ms, n), "kvtrim_profile_end")
    return {kvtrim_kernel_name(i): (ms[i], n[i]) for i in range(N_KERNELS) if n[i] > 0}
