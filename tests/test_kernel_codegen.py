"""CPU check of the generated device code (no GPU needed: hipcc cross-compiles to assembly).

The weight-streaming loops of the GEMM phases only reach HBM speed if every wait in them leaves the other
seven weight loads of the wavefront in flight (`s_waitcnt vmcnt(7)`).  Whether the compiler emits that
depends on details far from the loop - e.g. an activation-panel address it can no longer prove to be LDS
becomes a flat load, and then every wait in the loop waits for all loads - so the property is checked on the
assembly of the instantiation the bf16 workloads run."""
import os
import re
import subprocess

import pytest

from paper_2410_05589_amd import build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def asm(tmp_path_factory):
    out = str(tmp_path_factory.mktemp("asm") / "ps_inst_bf16_d128.s")
    cmd = [build.hipcc_path(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fno-gpu-rdc", "-fvisibility=hidden",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-mllvm", "-instcombine-max-copied-from-constant-users=10000",
           "-I", os.path.join(ROOT, "include"), "-I", build.CSRC,
           "-DPS_INST_NAME=bf16_d128", "-DPS_INST_BF16=1", "-DPS_INST_D=128",
           "--cuda-device-only", "-S", "-o", out, os.path.join(build.CSRC, "ps_inst.hip")]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout[-2000:]
    return open(out).read()


def _streaming_loops(text):
    """(kernel, label, mfma count, vmcnt values) of every basic block that branches back to itself and holds
    8 weight loads and at least 16 MFMAs."""
    found = []
    kernel, label, lines = None, None, []

    def close():
        if kernel and label:
            n_mfma = sum("v_mfma" in l for l in lines)
            n_load = sum("global_load_dwordx4" in l for l in lines)
            loops = any(re.search(r"s_cbranch\w+\s+%s\b" % re.escape(label), l) for l in lines)
            if loops and n_mfma >= 16 and n_load == 8:
                found.append((kernel, label, n_mfma, [int(m.group(1)) for l in lines for m in [re.search(r"vmcnt\((\d+)\)", l)] if m]))

    for line in text.splitlines():
        m = re.match(r"^(_Z\w+):", line)
        if m:
            close()
            kernel, label, lines = m.group(1), None, []
            continue
        m = re.match(r"^(\.LBB\d+_\d+):", line)
        if m:
            close()
            label, lines = m.group(1), []
            continue
        lines.append(line)
    close()
    return found


def test_streaming_loops_keep_seven_weight_loads_in_flight(asm):
    loops = _streaming_loops(asm)
    fused = [l for l in loops if "fused_kernel" in l[0]]
    # the persistent kernel: four variants (1..4 column tiles of rows) x five GEMM phases
    assert len(fused) == 20, [(l[0], l[1]) for l in fused]
    for kernel, label, n_mfma, waits in loops:
        assert waits and all(w == 7 for w in waits), (kernel, label, waits)


def test_no_flat_loads_and_no_spills_in_the_kernels_the_workloads_use(asm):
    assert "flat_load" not in asm
    meta = re.findall(r"\.name:\s+(\S+)\n(?:.*\n)*?\s+\.vgpr_spill_count:\s+(\d+)", asm)
    spills = {n: int(v) for n, v in meta}
    for n, v in spills.items():
        if "fused_kernel" in n and "ELi4EEv" not in n:      # (64 rows = four column tiles is the one variant that spills)
            assert v == 0, (n, v)


def test_attention_loop_keeps_the_next_key_groups_in_flight(asm):
    """bf16 attention: while a wavefront works on two groups of keys, the K and V rows of the next two (16 loads)
    must stay in flight: every wait inside the loop over key groups leaves at least 8 loads outstanding.  (Requests
    under a condition would make the compiler wait for all of them.)"""
    text = asm[asm.index("_Z12attn2_kernel"):]
    text = text[:text.index("s_endpgm")]
    loops = {}          # header label -> lines of all the blocks of that (inner) loop
    cur = None
    for line in text.splitlines():
        m = re.match(r"^\.L(BB\d+_\d+):\s*(;.*)?$", line)
        if m:
            note = m.group(2) or ""
            h = re.search(r"in Loop: Header=(BB\d+_\d+) Depth=2", note)
            cur = h.group(1) if h else (m.group(1) if "Parent Loop" in note and "Depth=1" in note else None)
            continue
        if cur:
            loops.setdefault(cur, []).append(line)
    found = []
    for header, body in loops.items():
        n_mfma = sum("v_mfma" in l for l in body)
        n_load = sum("global_load_dwordx4" in l for l in body)
        if n_mfma >= 40 and n_load >= 16:
            found.append((header, [int(m.group(1)) for l in body for m in [re.search(r"vmcnt\((\d+)\)", l)] if m]))
    assert len(found) == 1, found
    assert found[0][1] and min(found[0][1]) >= 8, found


def test_training_attention_kernel_fits_four_workgroups_per_compute_unit(tmp_path):
    """The bf16 training attention runs four workgroups (16 wavefronts) per compute unit: at most 128 vector
    registers per lane and 40 KiB of LDS per workgroup, no flat loads (LDS addresses stay LDS addresses), and
    only a handful of spilled registers (loop-invariant values)."""
    out = str(tmp_path / "ps_train.s")
    cmd = [build.hipcc_path(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fno-gpu-rdc", "-fvisibility=hidden",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-mllvm", "-instcombine-max-copied-from-constant-users=10000",
           "-I", os.path.join(ROOT, "include"), "-I", build.CSRC,
           "--cuda-device-only", "-S", "-o", out, os.path.join(build.CSRC, "ps_train.hip")]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout[-2000:]
    text = open(out).read()
    assert "flat_load" not in text
    seen = 0
    for m in re.finditer(r"\.group_segment_fixed_size:\s+(\d+)\n(?:.*\n)*?\s+\.name:\s+(\S+)\n(?:.*\n)*?\s+\.vgpr_count:\s+(\d+)\n\s+\.vgpr_spill_count:\s+(\d+)", text):
        lds, name, vgpr, spill = int(m.group(1)), m.group(2), int(m.group(3)), int(m.group(4))
        if "ga_attn_bf16_kernel" in name:
            seen += 1
            assert vgpr <= 128 and lds <= 40 * 1024 and spill <= 4, (name, vgpr, lds, spill)
    assert seen == 2        # head_dim 64 and 128
