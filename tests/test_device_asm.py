"""The one place where the library issues loads the compiler does not track: the 16-byte agent-scope
loads of the split merge (inline assembly, because the language's atomic loads stop at 8 bytes).  Their
destination registers may only be touched after the explicit wait that follows them.  The build itself
checks that in the generated assembly (paper_2602_03152_amd/build.py, check_untracked_loads); here the
checker is pinned on small listings - it must find a planted violation on a side path and must not
flag a block that merely follows the loads in the text - and run on the real sources."""
import os
import shutil

import pytest

from paper_2602_03152_amd import build as B

GOOD = """
kern:
\tv_mov_b32_e32 v1, v0
\t;;#ASMSTART
\tglobal_load_dwordx4 v[4:7], v[2:3], off sc1
\t;;#ASMEND
\ts_cbranch_execz .LBB0_2
\tv_add_u32_e32 v9, v1, v1
.LBB0_2:
\t;;#ASMSTART
\ts_waitcnt vmcnt(0)
\t;;#ASMEND
\tv_add_f32_e32 v8, v4, v5
\ts_branch .LBB0_4
.LBB0_3:
\tv_mov_b32_e32 v4, 0
.LBB0_4:
\ts_endpgm
"""


def test_checker_follows_the_control_flow_graph():
    loads, waits, bad = B.check_untracked_loads(GOOD)
    assert (loads, waits, bad) == (1, 1, [])          # .LBB0_3 touches v4 but is not reachable from the load
    planted = GOOD.replace("\tv_add_u32_e32 v9, v1, v1", "\tv_add_u32_e32 v9, v6, v1")   # side path reads v6 early
    assert [b[1] for b in B.check_untracked_loads(planted)[2]] == ["v_add_u32_e32 v9, v6, v1"]
    unwaited = GOOD.replace("\ts_waitcnt vmcnt(0)", "\ts_nop 0")
    assert B.check_untracked_loads(unwaited)[2]


@pytest.mark.skipif(shutil.which(B.HIPCC) is None and not os.path.exists(B.HIPCC), reason="no hipcc")
@pytest.mark.parametrize("source", B.ASM_CHECKED)
def test_untracked_loads_are_waited_for_before_any_use(tmp_path, source):
    B._check_asm(source, (), str(tmp_path), False)       # raises on a violation


def test_build_falls_back_to_counted_loads_when_the_check_fails(monkeypatch, tmp_path):
    """A toolchain on which the check of the hand-placed loads fails must not end in a broken library:
    build() then compiles everything again with the compiler-counted loads.  Host logic only: the
    compiler runs are recorded, not executed."""
    runs, checks = [], []

    def fake_check(source, extra_flags, bdir, verbose):
        checks.append(tuple(extra_flags))
        if B.TRACKED_FLAG not in extra_flags:
            raise B.UntrackedLoadsTouched("%s: planted" % source)

    monkeypatch.setattr(B, "_run", lambda cmd, verbose: runs.append(list(cmd)))
    monkeypatch.setattr(B, "_check_asm", fake_check)
    monkeypatch.setattr(B, "BUILD", str(tmp_path))
    B.build(verbose=False)
    assert any(B.TRACKED_FLAG not in c for c in checks) and any(B.TRACKED_FLAG in c for c in checks)
    link = runs[-1]
    assert "-shared" in link
    second_round = runs[[i for i, c in enumerate(runs) if "-shared" not in c and B.TRACKED_FLAG in c][0]:]
    compiles = [c for c in second_round if "-c" in c]
    assert len(compiles) == len(B.SOURCES) and all(B.TRACKED_FLAG in c for c in compiles)
