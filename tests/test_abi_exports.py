"""CPU-only: the C-ABI library builds/loads and exports every function the header declares."""
import ctypes
import os
import re

import paper_2605_09649_amd as kv
from paper_2605_09649_amd import build as kbuild

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "kvtrim.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(kvtrim_[a-z_]+)\s*\(", text)))


def test_header_declares_the_four_stage_calls():
    names = declared_functions()
    for n in ("kvtrim_score", "kvtrim_select_global", "kvtrim_compact", "kvtrim_decode_attn"):
        assert n in names


def test_library_exports_every_declared_symbol():
    if not os.path.exists(kv.library_path()):
        kbuild.build_lib()
    lib = ctypes.CDLL(kv.library_path())
    names = declared_functions()
    assert len(names) >= 10
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(kv.binding.EXPORTS) == names


def test_workspace_size_is_reported_without_a_gpu_and_rejects_bad_configs():
    assert kv.kvtrim_workspace_bytes(1, 32, 8, 32, 128, 2_097_152 + 512) > 0
    assert kv.kvtrim_workspace_bytes(1, 32, 8, 32, 96, 1000) == 0        # head_dim not 64/128
    assert kv.kvtrim_workspace_bytes(1, 32, 8, 36, 128, 1000) == 0       # Hq not a multiple of Hkv
    assert kv.kvtrim_workspace_bytes(1, 4, 1, 16, 128, 1000) == 0        # group > 8
    assert kv.kvtrim_workspace_bytes(0, 4, 1, 4, 128, 1000) == 0


def test_product_path_does_not_reach_the_oracle():
    pkg = os.path.join(ROOT, "paper_2605_09649_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.replace("no CPU fallback", ""), f


def test_entry_limit_and_kernel_name_table():
    assert kv.kvtrim_workspace_bytes(1, 1, 1, 1, 64, 2 ** 31 - 4096) > 0
    assert kv.kvtrim_workspace_bytes(1, 1, 1, 1, 64, 2 ** 31 - 4095) == 0   # segment entries are indexed with 32-bit integers
    names = [kv.kvtrim_kernel_name(i) for i in range(kv.binding.N_KERNELS)]
    assert all(names) and len(set(names)) == len(names)
    assert kv.kvtrim_kernel_name(kv.binding.N_KERNELS) is None and kv.kvtrim_kernel_name(-1) is None
    header = open(os.path.join(ROOT, "include", "kvtrim.h")).read()
    assert f"#define KVTRIM_N_KERNELS {kv.binding.N_KERNELS}" in header
    assert f"#define KVTRIM_PAGE_SIZE {kv.PAGE_SIZE}" in header
