"""CPU tests of the C-ABI library: it loads, exports what the header declares, and its
host-side validation reports errors before touching any device."""
import ctypes
import os
import re

import pytest

from paper_2410_05589_amd import binding as B
from paper_2410_05589_amd import debug as DBG
from paper_2410_05589_amd.configs import WORKLOADS, small_shape

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2410_05589_amd.build import build_library
        build_library(verbose=False)
    return B.load_library()


def _declared_functions(header):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\bPS_API\s+[a-z_ ]+\*?\s+(ps_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    declared = _declared_functions("ps_draft.h")
    assert sorted(B.EXPORTED_SYMBOLS) == declared
    for name in declared:
        assert getattr(lib, name) is not None
    debug = _declared_functions("ps_draft_debug.h")
    assert sorted(DBG.EXPORTED_SYMBOLS) == debug
    for name in debug:
        assert getattr(lib, name) is not None


def test_nothing_else_is_exported(lib):
    """The dynamic symbol table holds exactly the ps_* functions the headers declare."""
    import subprocess
    out = subprocess.run(["nm", "-D", "--defined-only", B.LIB_PATH], stdout=subprocess.PIPE, text=True, check=True).stdout
    exported = sorted(l.split()[-1] for l in out.splitlines() if l.split()[-1].startswith("ps_"))
    declared = sorted(sum((_declared_functions(h) for h in ("ps_draft.h", "ps_verify.h", "ps_draft_debug.h", "ps_train.h")), []))
    assert exported == declared


def test_struct_layouts_match_header():
    # field order of the ctypes mirrors follows the header text
    text = open(os.path.join(ROOT, "include", "ps_draft.h")).read()
    body = text[text.index("typedef struct ps_draft_config {"):text.index("} ps_draft_config;")]
    names = re.findall(r"\b(?:int32_t|float|uint32_t)\s+([a-z_]+);", body)
    assert names == [f[0] for f in B.ps_draft_config._fields_]
    body = text[text.index("typedef struct ps_draft_weights {"):text.index("} ps_draft_weights;")]
    assert re.findall(r"const void\*\s+([a-z_]+);", body) == list(B.WEIGHT_NAMES + B.INPUT_WEIGHT_NAMES)
    body = text[text.index("typedef struct ps_draft_step_args {"):text.index("} ps_draft_step_args;")]
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    names = [n for line in re.findall(r"[^;{]+;", body) for n in re.findall(r"\*?\s*\**([a-z_]+)\s*[,;]", line)]
    assert names == [f[0] for f in B.ps_draft_step_args._fields_]
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


def test_exchange_buffers_the_kernels_cannot_address_are_refused(lib):
    """The kernels use 32-bit byte offsets into every exchange buffer: a legal configuration whose attention
    partials (or any other exchange buffer) would reach 4 GiB is unsupported, not silently wrapped."""
    ok = _cfg(max_batch=4, max_positions=1 << 15)
    assert B.ps_draft_workspace_bytes(ok) > 0
    for kw in (dict(max_batch=4, max_positions=1 << 20), dict(max_positions=(1 << 24) + 1)):
        c = _cfg(**kw)
        assert B.ps_draft_workspace_bytes(c) == 0, kw
        w = B.ps_draft_weights()
        for n in B.WEIGHT_NAMES:
            setattr(w, n, 0x1000)
        assert B.ps_draft_init(c, w, 0x100000, 1 << 44, None)[0] == B.PS_ERR_UNSUPPORTED, kw
        assert DBG.ps_draft_debug_plan(c, 1, 1, 5, 0, 256, 160 * 1024)[0] == B.PS_ERR_UNSUPPORTED, kw


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
    assert B.ps_draft_last_status(None, None) == B.PS_ERR_NULL
    assert DBG.ps_draft_debug_spin_limit(None, 1) == B.PS_ERR_NULL
    assert DBG.ps_measure_stream_read(None, 1024, None) == B.PS_ERR_NULL
    assert DBG.ps_measure_stream_read(0x1000, 1000, None) == B.PS_ERR_SHAPE
    assert DBG.ps_measure_copy(0x1000, 0x2000, 8, None) == B.PS_ERR_SHAPE
    B.ps_draft_free(None)


def test_strerror(lib):
    seen = set()
    for st in range(0, -10, -1):
        s = B.ps_draft_strerror(st)
        assert s and s != "unknown status"
        seen.add(s)
    assert len(seen) == 10
    assert B.ps_draft_strerror(-99) == "unknown status"


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", "/nonexistent/libps_draft.so")
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        B.load_library()


PS_U, PS_WAVES = 8, 8


def _plan(lib, cfg, batch, n_new, k, n_cu=256, lds=160 * 1024, all_rows=0):
    st, plans = DBG.ps_draft_debug_plan(cfg, batch, n_new, k, all_rows, n_cu, lds)
    return (st, plans) if st == B.PS_OK else (st, None)


def _check_plan(cfg, plans, batch, n_new, k, n_cu, lds):
    """What the device code relies on (it has no bounds checks of its own for these)."""
    esz_step = 32 if cfg.dtype == B.PS_BF16 else 16          # elements per 64-byte step
    for ph, d in enumerate(plans):
        tag = (ph, d, batch, n_new, k, n_cu, lds)
        S, KW = 1 << d["s_log"], 1 << d["kw_log"]
        assert d["Kt"] % PS_U == 0 and d["Kt"] * esz_step >= d["K"] > (d["Kt"] - PS_U) * esz_step, tag
        assert 1 <= KW <= PS_WAVES and 1 <= S <= 8, tag
        if ph == 4:
            assert S == 1, tag                                 # the LM head keeps a row's logits in one workgroup
            assert min(n_cu, d["T"]) <= 512, tag               # one thread per workgroup in the final merge
        assert d["Gs"] == n_cu >> d["s_log"] and d["Gs"] >= 1, tag
        assert d["per_round"] == d["Gs"] * (PS_WAVES >> d["kw_log"]), tag
        assert d["rounds"] == -(-d["T"] // d["per_round"]), tag    # every tile is taken exactly once
        ng = d["Kt"] // PS_U
        sizes = [((ng * (s + 1)) >> d["s_log"]) - ((ng * s) >> d["s_log"]) for s in range(S)]
        pg, npc = d["piece_groups"], d["npieces"]
        assert min(sizes) >= 1 and pg >= KW, tag
        for sz in sizes:
            assert -(-sz // pg) == npc, tag                    # the slices walk through their pieces in step
            assert sz - (npc - 1) * pg >= KW, tag              # every piece gives each wavefront of a tile a group
        assert d["lds_bytes"] <= lds, tag
        arrays = 2 if cfg.dtype == B.PS_BF16 else 1
        assert d["lds_bytes"] >= d["rows"] * arrays * pg * PS_U * 64, tag   # the piece of the panel fits


def test_phase_plans_of_the_five_workloads(lib):
    for name, wl in WORKLOADS.items():
        n_max = max(wl.n_new_mix) if wl.n_new_mix else wl.n_new
        cfg = B.make_config(wl.shape, max_batch=wl.batch, max_new=n_max, max_positions=8192, max_topk=wl.topk, k_max=wl.k)
        for n_new in (sorted(set(wl.n_new_mix)) if wl.n_new_mix else [wl.n_new]):
            st, plans = _plan(lib, cfg, wl.batch, n_new, wl.k)
            assert st == B.PS_OK, (name, n_new)
            _check_plan(cfg, plans, wl.batch, n_new, wl.k, 256, 160 * 1024)


def test_attention_plans_of_the_bf16_workloads_and_of_a_sweep(lib):
    """The bf16 attention's blocks (host logic of ps_draft_step): the block sizes the timed workloads were measured
    fastest with; and for random batches on several device sizes what the device code relies on: the blocks cover
    every sequence, merge items exist exactly when some sequence spans several blocks, and a block size is only
    raised while that spares the workgroups a round of units or the merge."""
    import random
    from paper_2410_05589_amd import inputs
    expect = {"c1": (4, 32, 0), "c2": (2, 160, 40), "c4": (4, 192, 40)}
    for name, (nk, units, merges) in expect.items():
        wl = WORKLOADS[name]
        cfg = B.make_config(wl.shape, max_batch=wl.batch, max_new=6, max_positions=8192, max_topk=wl.topk, k_max=wl.k)
        st, ap = DBG.ps_draft_debug_attn_plan(cfg, wl.kv_len, wl.n_new, wl.k, 256)
        assert st == B.PS_OK and (ap["nk"], ap["units"], ap["merge_items"]) == (nk, units, merges), (name, ap)
    wl = WORKLOADS["c3"]
    cfg = B.make_config(wl.shape, max_batch=wl.batch, max_new=1, max_positions=8192, max_topk=wl.topk, k_max=wl.k)
    st, ap = DBG.ps_draft_debug_attn_plan(cfg, inputs.draw_kv_len(wl), wl.n_new, wl.k, 256)
    assert st == B.PS_OK and ap == {"nk": 16, "units": 256, "blocks": 256, "merge_items": 0}, ap
    f32 = B.make_config(WORKLOADS["c0"].shape, max_batch=1, max_new=1, max_positions=128, max_topk=4, k_max=4)
    assert DBG.ps_draft_debug_attn_plan(f32, (64,), 1, 4, 256)[0] == B.PS_ERR_UNSUPPORTED
    rnd = random.Random(11)
    for _ in range(300):
        n_kv = rnd.choice([1, 2, 4, 8])
        grp = rnd.choice([1, 2, 4])
        shape = small_shape("bf16", hidden=n_kv * grp * 64, n_heads=n_kv * grp, n_kv_heads=n_kv, head_dim=64, ffn=1024, vocab=1000)
        n_new, k = rnd.randint(1, 4), rnd.randint(0, 4)
        M = n_new + k
        batch = rnd.randint(1, max(1, min(8, 64 // (grp * M))))
        kv = [rnd.choice([0, 1, 127, 128, 129, rnd.randint(0, 40000)]) for _ in range(batch)]
        cfg = B.make_config(shape, max_batch=batch, max_new=n_new, max_positions=40000 + M, max_topk=8, k_max=max(k, 1))
        n_cu = rnd.choice([256, 304, 80, 7])
        st, ap = DBG.ps_draft_debug_attn_plan(cfg, kv, n_new, k, n_cu)
        assert st == B.PS_OK, (st, kv)
        ch = 128 * ap["nk"]
        assert ap["nk"] in (1, 2, 4, 8, 16)
        nch = [max(1, -(-l // ch)) for l in kv]
        npass = -(-grp * M // 16)
        assert ap["blocks"] == n_kv * sum(nch) and ap["units"] == ap["blocks"] * npass, (ap, kv)
        assert ap["merge_items"] == n_kv * -(-grp * M // 8) * sum(1 for n in nch if n > 1), (ap, kv)
        if ap["nk"] > 1:   # the next smaller size would cost a round of units more, or is the one that needs the merge
            nch2 = [max(1, -(-l // (ch // 2))) for l in kv]
            more_rounds = -(-n_kv * sum(nch2) * npass // n_cu) > -(-ap["units"] // n_cu)
            assert more_rounds or (max(nch2) > 1 and max(nch) == 1) or max(nch2) > 1, (ap, kv)
    assert DBG.ps_draft_debug_attn_plan(cfg, kv, n_new, k, 0)[0] == B.PS_ERR_SHAPE


def test_phase_plans_over_a_sweep_of_shapes_and_devices(lib):
    import random
    rnd = random.Random(7)
    checked = 0
    for _ in range(400):
        dtype = rnd.choice(["bf16", "f32"])
        mul = 32 if dtype == "bf16" else 16
        head_dim = rnd.choice([64, 128])
        n_kv = rnd.choice([1, 2, 4, 8])
        n_heads = n_kv * rnd.choice([1, 2, 4])
        hidden = n_heads * head_dim
        ffn = mul * rnd.randint(1, 500)
        vocab = rnd.randint(16, 200000)
        shape = small_shape(dtype, hidden=hidden, n_heads=n_heads, n_kv_heads=n_kv, head_dim=head_dim, ffn=ffn, vocab=vocab)
        k = rnd.randint(0, 8)
        n_new = rnd.randint(1, 6)
        grp = n_heads // n_kv
        batch = rnd.randint(1, max(1, min(8, 64 // (n_new + k), 64 // (grp * (n_new + k)) if grp * (n_new + k) <= 64 else 1)))
        if grp * (n_new + k) > 64 or batch * (n_new + k) > 64:
            continue
        cfg = B.make_config(shape, max_batch=batch, max_new=n_new, max_positions=4096, max_topk=8, k_max=max(k, 1))
        for n_cu, lds in ((256, 160 * 1024), (256, 64 * 1024), (304, 160 * 1024), (80, 64 * 1024), (7, 96 * 1024)):
            st, plans = _plan(lib, cfg, batch, n_new, k, n_cu=n_cu, lds=lds, all_rows=rnd.randint(0, 1))
            assert st in (B.PS_OK, B.PS_ERR_UNSUPPORTED), (st, hidden, ffn, vocab)
            if st == B.PS_OK:
                _check_plan(cfg, plans, batch, n_new, k, n_cu, lds)
                checked += 1
    assert checked > 500
