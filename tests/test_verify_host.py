"""CPU tests of the tree / acceptance-walk entry points: exported as the header declares, struct
layouts match, and host-side validation reports errors before anything touches a device."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2410_05589_amd import binding as B
from paper_2410_05589_amd import verify as VF

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "ps_verify.h")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2410_05589_amd.build import build_library
        build_library(verbose=False)
    return B.load_library()


def _header_code():
    return re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)


def test_every_declared_symbol_is_exported(lib):
    declared = sorted(set(re.findall(r"\bPS_API\s+[a-z_]+\s+(ps_[a-z_]+)\s*\(", _header_code())))
    assert declared == sorted(VF.EXPORTED_SYMBOLS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_struct_layouts_match_header():
    code = _header_code()
    body = code[code.index("typedef struct ps_tree_shape {"):code.index("} ps_tree_shape;")]
    assert re.findall(r"\b([a-z_]+);", body) == [f[0] for f in VF.ps_tree_shape._fields_]
    body = code[code.index("typedef struct ps_verify_args {"):code.index("} ps_verify_args;")]
    names = [n for line in re.findall(r"[^;{]+;", body) for n in re.findall(r"\*?\s*([a-z_]+)\s*[,;]", line)]
    assert names == [f[0] for f in VF.ps_verify_args._fields_]
    assert int(re.search(r"#define PS_TREE_MAX_NODES (\d+)", code).group(1)) == VF.PS_TREE_MAX_NODES


def _args(**kw):
    a = VF.ps_verify_args()
    a.batch, a.rows, a.vocab = 1, 3, 100
    for n in ("tokens", "q", "p", "r", "n_accepted", "path", "out_tokens"):
        setattr(a, n, 0x100000)
    for k, v in kw.items():
        setattr(a, k, v)
    return a


def test_walk_rejects_bad_arguments_on_the_host(lib):
    good = VF.make_tree([-1, 0, 0, 1], [0, 0, 1, 0])
    assert VF.ps_verify_walk(None, _args(), None) == B.PS_ERR_NULL
    assert VF.ps_verify_walk(good, None, None) == B.PS_ERR_NULL
    for n in ("tokens", "q", "p", "r", "n_accepted", "path", "out_tokens"):
        assert VF.ps_verify_walk(good, _args(**{n: None}), None) == B.PS_ERR_NULL, n
    for kw in (dict(batch=0), dict(rows=0), dict(vocab=0), dict(rows=1)):   # rows=1: depth 2 > rows
        assert VF.ps_verify_walk(good, _args(**kw), None) == B.PS_ERR_SHAPE, kw
    # without tokens the walk reads top_ids: both missing, no topk, no ranks, a rank beyond topk
    assert VF.ps_verify_walk(good, _args(tokens=None), None) == B.PS_ERR_NULL
    assert VF.ps_verify_walk(good, _args(tokens=None, top_ids=0x1000, topk=0), None) == B.PS_ERR_SHAPE
    assert VF.ps_verify_walk(VF.make_tree([-1, 0]), _args(tokens=None, top_ids=0x1000, topk=4), None) == B.PS_ERR_NULL
    assert VF.ps_verify_walk(good, _args(tokens=None, top_ids=0x1000, topk=1), None) == B.PS_ERR_SHAPE
    assert VF.ps_verify_walk(good, _args(vocab=1048580), None) == B.PS_ERR_UNSUPPORTED
    assert VF.ps_verify_walk(good, _args(vocab=262145), None) == B.PS_ERR_UNSUPPORTED      # odd: one entry per load
    for parent in ([0, 0], [-1, 1], [-1, -1], [-1, 0, 3], [-1] + [0] * 64, []):
        t = VF.make_tree(np.array(parent, dtype=np.int32), np.zeros(len(parent), dtype=np.int32))
        assert VF.ps_verify_walk(t, _args(rows=64), None) == B.PS_ERR_SHAPE, parent


def test_static_walk_validates_like_the_walk_and_never_falls_back(lib):
    """The entry point that allocates nothing: same argument checks; a batch beyond what the library's own
    exchange memory holds is an error there, not a slower path."""
    good = VF.make_tree([-1, 0, 0, 1], [0, 0, 1, 0])
    assert VF.ps_verify_walk_static(None, _args(), None) == B.PS_ERR_NULL
    assert VF.ps_verify_walk_static(good, None, None) == B.PS_ERR_NULL
    for n in ("tokens", "q", "p", "r", "n_accepted", "path", "out_tokens"):
        assert VF.ps_verify_walk_static(good, _args(**{n: None}), None) == B.PS_ERR_NULL, n
    for kw in (dict(batch=0), dict(rows=0), dict(vocab=0), dict(rows=1)):
        assert VF.ps_verify_walk_static(good, _args(**kw), None) == B.PS_ERR_SHAPE, kw
    assert VF.ps_verify_walk_static(good, _args(vocab=1048580), None) == B.PS_ERR_UNSUPPORTED
    assert VF.ps_verify_walk_static(good, _args(vocab=128256, batch=65), None) == B.PS_ERR_UNSUPPORTED
    assert VF.ps_verify_walk_static(good, _args(vocab=65536, batch=200), None) == B.PS_ERR_UNSUPPORTED


def test_workspace_bytes(lib):
    assert VF.ps_verify_workspace_bytes(8, 32000) == 0          # P stays in registers: nothing to exchange
    assert VF.ps_verify_workspace_bytes(8, 32768) == 0
    assert VF.ps_verify_workspace_bytes(8, 50001) == 0          # odd: one workgroup per sequence
    assert VF.ps_verify_workspace_bytes(0, 128256) == 0
    one, eight = VF.ps_verify_workspace_bytes(1, 128256), VF.ps_verify_workspace_bytes(8, 128256)
    assert one % 256 == 0 and eight % 256 == 0 and 0 < one < eight <= 8 * one
    assert VF.ps_verify_workspace_bytes(64, 128256) == 1065472  # the size of the library's own array (stated in the header)


def test_tree_tokens_rejects_bad_arguments_on_the_host(lib):
    good = VF.make_tree([-1, 0, 0, 1], [0, 0, 1, 0])
    assert VF.ps_tree_tokens(None, 1, 3, 4, 0x1000, 0x1000, None) == B.PS_ERR_NULL
    assert VF.ps_tree_tokens(good, 1, 3, 4, None, 0x1000, None) == B.PS_ERR_NULL
    assert VF.ps_tree_tokens(good, 1, 3, 4, 0x1000, None, None) == B.PS_ERR_NULL
    assert VF.ps_tree_tokens(VF.make_tree([-1, 0]), 1, 3, 4, 0x1000, 0x1000, None) == B.PS_ERR_NULL   # no ranks
    for batch, rows, topk in ((0, 3, 4), (1, 0, 4), (1, 3, 0), (1, 1, 4), (1, 3, 1)):   # (1,1,4): depth 2 > rows; (1,3,1): rank 1 >= topk
        assert VF.ps_tree_tokens(good, batch, rows, topk, 0x1000, 0x1000, None) == B.PS_ERR_SHAPE, (batch, rows, topk)
    bad_rank = VF.make_tree([-1, 0], [0, -1])
    assert VF.ps_tree_tokens(bad_rank, 1, 3, 4, 0x1000, 0x1000, None) == B.PS_ERR_SHAPE
