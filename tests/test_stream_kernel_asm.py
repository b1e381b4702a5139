"""The persistent 3x3 kernel issues its residual loads as inline asm whose destination registers
hold no data until a later wait; a compiler that copied or read such a register earlier would
silently compute with stale values.  This test compiles the kernel's source for gfx950 (no GPU
needed) and scans the generated assembly: between each such load and the wait that has it landed
no instruction may touch its destination registers."""
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_1904_08368_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def _regs(code):
    out = set()
    for m in re.finditer(r"v\[(\d+):(\d+)\]|\bv(\d+)\b", code):
        out |= set(range(int(m.group(1)), int(m.group(2)) + 1)) if m.group(1) else {int(m.group(3))}
    return out


@pytest.mark.timeout(300)
def test_async_load_registers_untouched_until_their_wait(tmp_path):
    if not os.path.exists(HIPCC):
        pytest.skip("no hipcc")
    flags = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-x", "hip", "-Xclang", "-target-feature", "-Xclang",
             "-packed-fp32-ops", "-w", "--cuda-device-only", "-S"]
    asm = str(tmp_path / "conv_stream.s")
    r = subprocess.run([HIPCC, *flags, os.path.join(CSRC, "conv_stream.hip"), "-o", asm], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = open(asm).read().split("\n")
    fa, checked, bad = None, 0, []
    for i, raw in enumerate(lines):
        l = raw.strip()
        m = re.match(r"_ZN5relay.*stream_kernelILb\dE(?:Li\d+E){7}Li(\d+)EEEv[^:]*:", l)
        if m:
            fa = int(m.group(1))        # the kernel's look-ahead: its last template argument
        m = re.match(r"buffer_load_dword(x2)?\s+(\S+),", l)
        if not m or " lds" in l:
            continue
        assert fa is not None
        dst = _regs(m.group(2))
        checked += 1
        barriers, j = 0, i + 1
        # the loads are issued in front of a step's barrier; the wait that covers them sits in front of the
        # barrier `fa` steps later (or is the full wait behind the loop)
        while j < len(lines) and barriers < fa:
            t = lines[j].strip()
            if t.startswith("s_barrier"):
                barriers += 1
            elif t.startswith("s_endpgm") or t.startswith("s_waitcnt vmcnt(0)"):
                break
            elif t and t[0] not in ";." and not re.match(r"buffer_load_dword(x2)?\s", t):
                code = t.split(";")[0]
                if _regs(code) & dst:
                    bad.append((i + 1, j + 1, code))
            j += 1
    assert checked >= 8 * 6, checked          # six instantiations (fp16 / int8 x three variants, two chunk lengths each)
    assert not bad, bad[:5]
