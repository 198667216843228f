"""CPU tests of the C-ABI library: it loads, exports what the header declares, and its
host-side validation reports errors before touching any device."""
import ctypes
import os
import re

import pytest

from paper_2410_05589_amd import binding as B
from paper_2410_05589_amd.configs import WORKLOADS, small_shape

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2410_05589_amd.build import build_library
        build_library(verbose=False)
    return B.load_library()


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "ps_draft.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ps_draft_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    declared = _declared_functions()
    assert sorted(B.EXPORTED_SYMBOLS) == declared
    for name in declared:
        assert getattr(lib, name) is not None


def test_struct_layouts_match_header():
    # field order of the ctypes mirrors follows the header text
    text = open(os.path.join(ROOT, "include", "ps_draft.h")).read()
    body = text[text.index("typedef struct ps_draft_config {"):text.index("} ps_draft_config;")]
    names = re.findall(r"\b(?:int32_t|float|uint32_t)\s+([a-z_]+);", body)
    assert names == [f[0] for f in B.ps_draft_config._fields_]
    body = text[text.index("typedef struct ps_draft_weights {"):text.index("} ps_draft_weights;")]
    assert re.findall(r"const void\*\s+([a-z_]+);", body) == list(B.WEIGHT_NAMES)
    body = text[text.index("typedef struct ps_draft_step_args {"):text.index("} ps_draft_step_args;")]
    names = re.findall(r"\b(?:int32_t\*?|float\*|const void\*|void\*|const int64_t\*|const int32_t\*)\s+\*?([a-z_]+)[;,]", body)
    fields = [f[0] for f in B.ps_draft_step_args._fields_]
    assert set(fields) <= set(names) | {"v_cache", "top_p", "lse", "probs", "hidden_out"}
    assert ctypes.sizeof(B.ps_draft_config) == 15 * 4


def _cfg(name="c1", **kw):
    wl = WORKLOADS[name]
    c = B.make_config(wl.shape, max_batch=1, max_new=6, max_positions=2048, max_topk=8)
    for k, v in kw.items():
        setattr(c, k, v)
    return c


def test_workspace_bytes_for_the_five_workloads(lib):
    for name, wl in WORKLOADS.items():
        c = B.make_config(wl.shape, max_batch=wl.batch, max_new=max(wl.n_new_mix or (wl.n_new,)),
                          max_positions=4200, max_topk=8, k_max=wl.k)
        n = B.ps_draft_workspace_bytes(c)
        assert n > 0 and n % 256 == 0, name
        assert n < 2 << 30


def test_config_validation(lib):
    assert B.ps_draft_workspace_bytes(_cfg()) > 0
    bad = [dict(hidden=0), dict(n_kv_heads=3), dict(dtype=7), dict(max_batch=0), dict(k_max=-1),
           dict(rope_base=0.0), dict(flags=8), dict(max_positions=3), dict(max_topk=0), dict(rms_eps=-1.0)]
    for kw in bad:
        c = _cfg(**kw)
        assert B.ps_draft_workspace_bytes(c) == 0, kw
        w = B.ps_draft_weights()
        for n in B.WEIGHT_NAMES:
            setattr(w, n, 0x1000)
        st, h = B.ps_draft_init(c, w, 0x100000, 1 << 40, None)
        assert st == B.PS_ERR_CONFIG, kw
    unsupported = [dict(head_dim=96, n_heads=32, n_kv_heads=32), dict(hidden=4100), dict(ffn=11012),
                   dict(max_batch=32), dict(max_topk=33)]
    for kw in unsupported:
        c = _cfg(**kw)
        w = B.ps_draft_weights()
        for n in B.WEIGHT_NAMES:
            setattr(w, n, 0x1000)
        st, h = B.ps_draft_init(c, w, 0x100000, 1 << 40, None)
        assert st == B.PS_ERR_UNSUPPORTED, kw


def test_init_null_and_workspace_errors(lib):
    c = _cfg()
    w = B.ps_draft_weights()
    for n in B.WEIGHT_NAMES:
        setattr(w, n, 0x1000)
    need = B.ps_draft_workspace_bytes(c)
    assert B.ps_draft_init(None, w, 0x100000, need, None)[0] == B.PS_ERR_NULL
    assert B.ps_draft_init(c, None, 0x100000, need, None)[0] == B.PS_ERR_NULL
    assert B.ps_draft_init(c, w, None, need, None)[0] == B.PS_ERR_NULL
    assert B.ps_draft_init(c, w, 0x100000, need - 1, None)[0] == B.PS_ERR_WORKSPACE
    assert B.ps_draft_init(c, w, 0x100010, need, None)[0] == B.PS_ERR_WORKSPACE
    w2 = B.ps_draft_weights()
    for n in B.WEIGHT_NAMES:
        setattr(w2, n, 0x1000)
    w2.w_lm = None
    assert B.ps_draft_init(c, w2, 0x100000, need, None)[0] == B.PS_ERR_NULL
    # g_final may be NULL only without the final norm
    w3 = B.ps_draft_weights()
    for n in B.WEIGHT_NAMES:
        setattr(w3, n, 0x1000)
    w3.g_final = None
    assert B.ps_draft_init(c, w3, 0x100000, need, None)[0] == B.PS_ERR_NULL


def test_step_and_free_with_null_context(lib):
    a = B.ps_draft_step_args()
    assert B.ps_draft_step(None, a, None) == B.PS_ERR_NULL
    B.ps_draft_free(None)


def test_strerror(lib):
    seen = set()
    for st in range(0, -9, -1):
        s = B.ps_draft_strerror(st)
        assert s and s != "unknown status"
        seen.add(s)
    assert len(seen) == 9
    assert B.ps_draft_strerror(-99) == "unknown status"


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", "/nonexistent/libps_draft.so")
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        B.load_library()
