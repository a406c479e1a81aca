"""The library's host code - argument validation, workspace carve-up, launch plans, list checker - under
AddressSanitizer and UndefinedBehaviorSanitizer: paper_2602_03152_amd/build.py builds the sources with the
sanitizers on the host side only (device code unchanged) into a stand-alone exerciser of the C ABI
(csrc/abi_host_check.cpp) and runs it; no GPU is needed or touched."""
import os
import shutil
import subprocess

import pytest

from paper_2602_03152_amd import build as B


@pytest.mark.skipif(shutil.which(B.HIPCC) is None and not os.path.exists(B.HIPCC), reason="no hipcc")
def test_abi_host_code_is_clean_under_asan_and_ubsan():
    exe = B.build_sanitized(verbose=False, run=True)       # raises on a failed check or a sanitizer report
    syms = subprocess.run(["nm", "-D", exe], stdout=subprocess.PIPE, text=True).stdout
    assert "__asan_init" in syms and "__ubsan_handle" in syms, "the exerciser is not instrumented"
