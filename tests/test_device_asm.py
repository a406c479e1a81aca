"""The one place where the library issues loads the compiler does not track: the 16-byte agent-scope
loads of the split merge (inline assembly, because the language's atomic loads stop at 8 bytes).  Their
destination registers may only be touched after the explicit wait that follows them.  This test compiles
the attention source to device assembly with the library's own flags and checks exactly that, for every
kernel instance, so a compiler that schedules differently is caught on the host."""
import os
import re
import shutil
import subprocess

import pytest

from paper_2602_03152_amd import build as B


@pytest.mark.skipif(shutil.which(B.HIPCC) is None and not os.path.exists(B.HIPCC), reason="no hipcc")
def test_untracked_loads_are_waited_for_before_any_use(tmp_path):
    out = tmp_path / "attend_dev.s"
    flags = [f for f in B.FLAGS if f != "-fPIC"]
    p = subprocess.run([B.HIPCC, *flags, "--cuda-device-only", "-S", os.path.join(B.CSRC, "attend.hip"), "-o", str(out)],
                       stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert p.returncode == 0, p.stdout[-2000:]
    pending, loads, waits, touches = set(), 0, 0, []
    in_asm = False
    for ln, line in enumerate(out.read_text().split("\n"), 1):
        if "ASMSTART" in line:
            in_asm = True
            continue
        if "ASMEND" in line:
            in_asm = False
            continue
        if in_asm:
            m = re.search(r"global_load_dwordx4 v\[(\d+):(\d+)\].*\bsc1\b", line)
            if m:
                pending.update(range(int(m.group(1)), int(m.group(2)) + 1))
                loads += 1
            elif "s_waitcnt vmcnt(0)" in line:
                pending.clear()
                waits += 1
            continue
        if "s_endpgm" in line:
            assert not pending, "kernel ends with unwaited loads (line %d)" % ln
        if pending and re.match(r"\s+(v_|ds_|global_|flat_|buffer_|scratch_)", line):
            regs = set()
            for a, b in re.findall(r"v\[(\d+):(\d+)\]", line):
                regs.update(range(int(a), int(b) + 1))
            regs.update(int(a) for a in re.findall(r"\bv(\d+)\b", line))
            if regs & pending:
                touches.append((ln, line.strip()))
    assert loads > 0 and waits > 0, "the merge no longer uses the 16-byte agent-scope loads: drop this test"
    assert not touches, touches[:5]
