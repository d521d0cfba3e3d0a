"""The C-ABI library loads and exports every entry point the header declares (no GPU needed)."""
import ctypes
import os
import re

import paper_2602_11543_amd as S

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_header_symbols_are_exported():
    header = open(os.path.join(ROOT, "include", "spes.h")).read()
    names = set(re.findall(r"SPES_API[^;(]*?\b(spes_\w+)\s*\(", header))
    assert {"spes_moe_fwd", "spes_moe_bwd", "spes_expert_merge", "spes_expert_warmup_merge"} <= names
    lib = ctypes.CDLL(S.library_path())
    for n in names:
        assert hasattr(lib, n), n


def test_host_only_queries():
    sh = S.moe_shape(512, 256, 8, 512, 2, S.SPES_F32, 1)
    lay = S.spes_moe_ctx_describe(sh)
    assert lay["total"] == S.spes_moe_ctx_bytes(sh) > 0
    offs = sorted(v for k, v in lay.items() if k != "total")
    assert all(o % 256 == 0 for o in offs) and len(set(offs)) == len(offs)
    assert S.spes_moe_ctx_bytes(S.moe_shape(512, 256, 65, 512, 2, 0, 0)) == 0       # more than 64 experts
    assert S.spes_moe_ctx_bytes(S.moe_shape(512, 250, 8, 512, 2, 0, 0)) == 0        # d_model not a multiple of 8
    assert S.spes_warmup_scratch_bytes(8, 4096) > 0
    assert "aligned" in S.spes_strerror(-3)


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2602_11543_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text, f
