"""Static check of the hand-counted waits in the direct-load down-projection GEMM.

That kernel issues its channel-number loads and LDS fragment reads as inline assembly, so the compiler neither waits
for them nor knows that their destination registers are written late.  The test compiles the kernel to assembly and
replays the instruction stream with the hardware's in-order counters (vmcnt for vector-memory loads, lgkmcnt for LDS
reads): between a load's issue and the wait that retires it, no instruction may read or write its destination
registers (a use would see stale data; a reuse as a temporary would be overwritten when the data lands).
"""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "paper_2602_06822_amd", "csrc", "pop_down_gemm.hip")
KERNEL = "_ZN3pop20down_gemm_dma_kernel"


def _regs(tok):
    out = set()
    for m in re.finditer(r"v\[(\d+):(\d+)\]", tok):
        out.update(range(int(m.group(1)), int(m.group(2)) + 1))
    for m in re.finditer(r"(?<![\w\[:])v(\d+)\b", tok):
        out.add(int(m.group(1)))
    return out


def replay(lines):
    """Returns (number of loads seen, list of offending instructions)."""
    vmq, lgq, bad, n_loads = [], [], [], 0
    for raw in lines:
        line = raw.strip()
        if not line or line[0] in ";.":
            continue
        op = line.split()[0]
        parts = [a.strip() for a in line[len(op):].split(",")]
        if op == "s_waitcnt":
            for name, queue in (("vmcnt", vmq), ("lgkmcnt", lgq)):
                m = re.search(name + r"\((\d+)\)", line)
                if m:
                    del queue[:max(0, len(queue) - int(m.group(1)))]
            continue
        dst = _regs(parts[0]) if parts else set()
        src = set().union(*[_regs(a) for a in parts[1:]]) if len(parts) > 1 else set()
        if op.startswith(("global_store", "ds_write")):
            src, dst = src | dst, set()
        pending = set().union(*vmq, *lgq) if (vmq or lgq) else set()
        if op.startswith("global_load_lds"):          # direct load: no register result
            if (src | dst) & pending:
                bad.append(line)
            vmq.append(set())
        elif op.startswith("global_load"):
            if src & pending:
                bad.append(line)
            vmq.append(dst)
            n_loads += 1
        elif op.startswith("ds_read"):
            if src & pending:
                bad.append(line)
            lgq.append(dst)
            n_loads += 1
        elif op.startswith(("s_load", "s_buffer_load")):
            lgq.append(set())
        elif (src | dst) & pending:
            bad.append(line)
    return n_loads, bad


def test_replay_flags_a_planted_hazard():
    ok = ["global_load_dword v5, v[6:7], off", "s_waitcnt vmcnt(0)", "v_add_u32_e32 v1, v5, v2"]
    assert replay(ok) == (1, [])
    early = ["global_load_dword v5, v[6:7], off", "v_add_u32_e32 v1, v5, v2", "s_waitcnt vmcnt(0)"]
    assert replay(early)[1] == ["v_add_u32_e32 v1, v5, v2"]
    reused = ["ds_read_b128 v[8:11], v3", "ds_read_b128 v[12:15], v4", "s_waitcnt lgkmcnt(1)",
              "v_mov_b32_e32 v12, 0", "v_mov_b32_e32 v8, 0"]
    assert replay(reused)[1] == ["v_mov_b32_e32 v12, 0"]


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="needs hipcc")
def test_direct_load_gemm_touches_no_register_with_a_load_in_flight(tmp_path):
    out = tmp_path / "down_gemm.s"
    cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-I", os.path.join(ROOT, "include"), "-I", os.path.dirname(SRC), "-S",
           "--cuda-device-only", SRC, "-o", str(out)]
    subprocess.run(cmd, check=True, capture_output=True, timeout=600)
    text = out.read_text()
    start = text.index(":", text.index(KERNEL))
    body = text[start:text.index(".Lfunc_end", start)].split("\n")
    n_loads, bad = replay(body)
    assert n_loads > 100, "the kernel's inline-assembly loads were not found"
    assert not bad, bad[:5]
