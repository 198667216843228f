"""CPU tests of the group-wise training attention's entry points: exported as declared, struct layout, host-side validation."""
import ctypes
import os
import re

import pytest

from paper_2410_05589_amd import binding as B
from paper_2410_05589_amd import train as TR

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2410_05589_amd.build import build_library
        build_library(verbose=False)
    return B.load_library()


def _code():
    return re.sub(r"/\*.*?\*/", "", open(os.path.join(ROOT, "include", "ps_train.h")).read(), flags=re.S)


def test_declared_symbols_and_struct_layout(lib):
    declared = sorted(set(re.findall(r"\bPS_API\s+[a-z_]+\s+(ps_[a-z_]+)\s*\(", _code())))
    assert declared == sorted(TR.EXPORTED_SYMBOLS)
    for n in declared:
        assert getattr(lib, n) is not None
    body = _code()
    body = body[body.index("typedef struct ps_group_attn_args {"):body.index("} ps_group_attn_args;")]
    names = [n for line in re.findall(r"[^;{]+;", body) for n in re.findall(r"\*?\s*([a-z_]+)\s*[,;]", line)]
    assert names == [f[0] for f in TR.ps_group_attn_args._fields_]


def test_validation_on_the_host(lib):
    def args(**kw):
        a = TR.make_args(1, 64, 4, 8, 8, 64, "bf16", 10000.0)
        for n in ("q", "k_", "v", "out", "workspace"):
            setattr(a, n, 0x100000)
        a.workspace_bytes = 1 << 40
        for k_, v in kw.items():
            setattr(a, k_, v)
        return a
    assert TR.ps_group_attention_workspace_bytes(args()) > 0
    assert TR.ps_group_attention(None, None) == B.PS_ERR_NULL
    for kw in (dict(seqs=0), dict(tokens=0), dict(k=-1), dict(n_kv_heads=3), dict(dtype=5), dict(rope_base=0.0)):
        assert TR.ps_group_attention(args(**kw), None) == B.PS_ERR_SHAPE, kw
        assert TR.ps_group_attention_workspace_bytes(args(**kw)) == 0
    for kw in (dict(head_dim=96), dict(k=16), dict(tokens=1 << 20), dict(k=15, n_heads=32768, n_kv_heads=32768, head_dim=128)):
        assert TR.ps_group_attention(args(**kw), None) == B.PS_ERR_UNSUPPORTED, kw
    for n in ("q", "k_", "v", "out", "workspace"):
        assert TR.ps_group_attention(args(**{n: None}), None) == B.PS_ERR_NULL, n
    need = TR.ps_group_attention_workspace_bytes(args())
    assert TR.ps_group_attention(args(workspace_bytes=need - 1), None) == B.PS_ERR_WORKSPACE
    assert TR.ps_group_attention(args(workspace=0x100010), None) == B.PS_ERR_WORKSPACE
