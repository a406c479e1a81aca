"""Builds libfasa.so (the C-ABI HIP library) in-tree for gfx950 with hipcc.

    python -m paper_2602_03152_amd.build

Objects go to paper_2602_03152_amd/_build/, the library to paper_2602_03152_amd/libfasa.so.

    python -m paper_2602_03152_amd.build --sanitize

compiles the same sources with AddressSanitizer and UndefinedBehaviorSanitizer on the HOST side (the
device code is untouched) into paper_2602_03152_amd/fasa_abi_host_check, a stand-alone program
(csrc/abi_host_check.cpp) that walks the argument validation of every entry point and the pure host
functions (workspace sizes, launch plans, list checker) without a GPU, and runs it: any sanitizer
report fails the build (tests/test_host_sanitizers.py does the same).

    python -m paper_2602_03152_amd.build --trace

builds a second library, paper_2602_03152_amd/libfasa_trace.so, with device-side stage timers compiled
in (-DFASA_TRACE): the selection and attention kernels then print, for row 0, how long each of their
phases took (units of 10 ns, from the constant 100 MHz counter).  `FASA_LIB=<path> python bench.py
--stage-timers` runs a few steps on it.  For phase breakdowns only: the printing itself costs
microseconds, so a traced library says nothing about step times.
"""
from __future__ import annotations

import os
import re
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
BUILD = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libfasa.so")
LIB_TRACE = os.path.join(PKG, "libfasa_trace.so")
FLOORS = os.path.join(PKG, "fasa_floors")      # stand-alone measurement program (csrc/floors.hip)
SOURCES = ["api.hip", "pack.hip", "score.hip", "topk.hip", "attend.hip", "fused.hip", "offload.hip", "calib.hip"]

HIPCC = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950",
    # packed-FP32 VALU forms stay off for every kernel of this library
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-attributes",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in p.stdout.splitlines()
                    if "packed-fp32-ops" not in l and "is not a recognized feature" not in l)
    if p.returncode != 0:
        raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), p.stdout))
    if verbose and out.strip():
        print(out, flush=True)


# Sources whose merge of split partials issues loads the compiler does not count (inline assembly:
# 16-byte loads with the sc1 bit, csrc/attend_common.h).  Their destination registers may only be
# touched after the explicit wait that follows them; check_untracked_loads() verifies that in the
# generated device assembly, along every path of the control-flow graph, and build() refuses to link a
# library for which it does not hold.
ASM_CHECKED = ["attend.hip", "fused.hip"]


def check_untracked_loads(asm_text: str):
    """Returns (loads, waits, violations) for one device assembly listing.  A violation is
    (line number, instruction): an instruction that reads or writes a register which an inline-assembly
    `global_load_dwordx4 ... sc1` has as its destination while no `s_waitcnt vmcnt(0)` of the same
    inline assembly has been passed since, on some path from the load."""
    lines = asm_text.split("\n")
    # ---- basic blocks of every function: split at labels and after branches ----
    blocks, cur = [], None            # block = dict(label, items=[(ln, kind, payload)], succ=[labels], fall=bool)
    label_re = re.compile(r"^([.\w$]+):")
    in_asm = False

    def new_block(label):
        nonlocal cur
        cur = {"label": label, "items": [], "succ": [], "fall": True}
        blocks.append(cur)

    new_block(None)
    for ln, line in enumerate(lines, 1):
        m = label_re.match(line)
        if m and not in_asm:
            new_block(m.group(1))
            continue
        text = line.strip()
        if "ASMSTART" in text:
            in_asm = True
            continue
        if "ASMEND" in text:
            in_asm = False
            continue
        if not text or text.startswith((";", ".", "//")):
            continue
        if in_asm:
            m = re.search(r"global_load_dwordx4 v\[(\d+):(\d+)\].*\bsc1\b", text)
            if m:
                cur["items"].append((ln, "load", set(range(int(m.group(1)), int(m.group(2)) + 1))))
            elif "s_waitcnt vmcnt(0)" in text:
                cur["items"].append((ln, "wait", None))
            continue
        op = text.split()[0]
        if op.startswith("s_cbranch"):
            cur["succ"].append(text.split()[-1])
            nxt = {"label": None, "items": [], "succ": [], "fall": True}
            cur["next_is_split"] = True
            blocks.append(nxt)
            cur = nxt
            continue
        if op == "s_branch":
            cur["succ"].append(text.split()[-1])
            cur["fall"] = False
            new_block(None)
            continue
        if op in ("s_endpgm", "s_setpc_b64"):
            cur["items"].append((ln, "end", text))
            cur["fall"] = False
            new_block(None)
            continue
        if re.match(r"(v_|ds_|global_|flat_|buffer_|scratch_)", op):
            regs = set()
            for a, b in re.findall(r"v\[(\d+):(\d+)\]", text):
                regs.update(range(int(a), int(b) + 1))
            regs.update(int(a) for a in re.findall(r"\bv(\d+)\b", text))
            if regs:
                cur["items"].append((ln, "use", (regs, text)))
    by_label = {b["label"]: i for i, b in enumerate(blocks) if b["label"]}
    succ = []
    for i, b in enumerate(blocks):
        out = [by_label[l] for l in b["succ"] if l in by_label]
        if b["fall"] and i + 1 < len(blocks):
            out.append(i + 1)
        succ.append(out)
    # ---- forward data flow: registers with a load in flight at block entry (union over predecessors) ----
    entry = [set() for _ in blocks]
    work = list(range(len(blocks)))
    loads = waits = 0
    while work:
        i = work.pop()
        pend = set(entry[i])
        for _, kind, payload in blocks[i]["items"]:
            if kind == "load":
                pend |= payload
            elif kind == "wait":
                pend = set()
        for j in succ[i]:
            if not pend <= entry[j]:
                entry[j] |= pend
                work.append(j)
    violations = []
    for i, b in enumerate(blocks):
        pend = set(entry[i])
        for ln, kind, payload in b["items"]:
            if kind == "load":
                pend |= payload
                loads += 1
            elif kind == "wait":
                pend = set()
                waits += 1
            elif kind == "end":
                if pend:
                    violations.append((ln, "kernel ends with unwaited loads"))
            elif pend and (payload[0] & pend):
                violations.append((ln, payload[1]))
    return loads, waits, violations


def _check_asm(source, extra_flags, bdir, verbose):
    out = os.path.join(bdir, source.replace(".hip", "_dev.s"))
    flags = [f for f in FLAGS if f != "-fPIC"]
    _run([HIPCC, *flags, *extra_flags, "--cuda-device-only", "-S", os.path.join(CSRC, source), "-o", out], verbose)
    loads, waits, bad = check_untracked_loads(open(out).read())
    if TRACKED_FLAG in extra_flags:
        if loads:
            raise RuntimeError("%s: inline-assembly sc1 loads in a build that asked for none" % source)
        return
    if loads == 0 or waits == 0:
        raise RuntimeError("%s: no inline-assembly sc1 loads found: remove it from ASM_CHECKED" % source)
    if bad:
        raise UntrackedLoadsTouched("%s: registers of uncounted loads are touched before their wait: %s" % (source, bad[:5]))


TRACKED_FLAG = "-DFASA_MERGE_LOADS_TRACKED"


class UntrackedLoadsTouched(RuntimeError):
    """The compiler moved a use of a hand-placed load's destination above its wait."""


HOST_CHECK = os.path.join(PKG, "fasa_abi_host_check")
SANITIZE = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
            "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]


def build_sanitized(verbose: bool = True, run: bool = True) -> str:
    """Host-sanitized build of the library's sources into the ABI exerciser; runs it unless run=False.
    Raises on a compile error, a failed check or a sanitizer report."""
    bdir = os.path.join(BUILD, "sanitize")
    os.makedirs(bdir, exist_ok=True)
    flags = [f for f in FLAGS if f != "-O3"] + ["-O1"] + SANITIZE
    objs = [os.path.join(bdir, s.replace(".hip", ".o")) for s in SOURCES]
    cmds = [[HIPCC, *flags, "-c", os.path.join(CSRC, s), "-o", o] for s, o in zip(SOURCES, objs)]
    main_o = os.path.join(bdir, "abi_host_check.o")
    cmds.append([HIPCC, *flags, "-x", "hip", "-c", os.path.join(CSRC, "abi_host_check.cpp"), "-o", main_o])
    with ThreadPoolExecutor(max_workers=8) as ex:
        for fut in [ex.submit(_run, c, verbose) for c in cmds]:
            fut.result()
    _run([HIPCC, "--offload-arch=gfx950", *SANITIZE, "-o", HOST_CHECK, main_o, *objs], verbose)
    if run:
        env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0:exitcode=23",
                   UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
        p = subprocess.run([HOST_CHECK], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env)
        if verbose:
            print(p.stdout, flush=True)
        if p.returncode != 0 or "all checks passed" not in p.stdout or "runtime error" in p.stdout or "ERROR: AddressSanitizer" in p.stdout:
            raise RuntimeError("sanitized ABI check failed (exit %d):\n%s" % (p.returncode, p.stdout[-4000:]))
    return HOST_CHECK


def build(verbose: bool = True, extra_flags=(), trace: bool = False) -> str:
    """Compiles every source and links the library.  If the assembly check of the hand-placed 16-byte
    loads fails (a toolchain that schedules differently), everything is rebuilt with the compiler-counted
    8-byte loads instead (TRACKED_FLAG; `--tracked-merge-loads` asks for that build directly)."""
    try:
        return _build(verbose, tuple(extra_flags), trace)
    except UntrackedLoadsTouched as e:
        print("build: %s\nbuild: falling back to compiler-counted merge loads (%s)" % (e, TRACKED_FLAG), flush=True)
        return _build(verbose, (*extra_flags, TRACKED_FLAG), trace)


def _build(verbose, extra_flags, trace) -> str:
    lib, bdir = LIB, BUILD
    if trace:
        lib, bdir, extra_flags = LIB_TRACE, os.path.join(BUILD, "trace"), (*extra_flags, "-DFASA_TRACE")
    os.makedirs(bdir, exist_ok=True)
    objs = [os.path.join(bdir, s.replace(".hip", ".o")) for s in SOURCES]
    cmds = [[HIPCC, *FLAGS, *extra_flags, "-c", os.path.join(CSRC, s), "-o", o] for s, o in zip(SOURCES, objs)]
    if not extra_flags:   # the floors program does not depend on the library's compile-time switches
        cmds.append([HIPCC, "-O3", "-std=c++17", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang",
                     "-packed-fp32-ops", os.path.join(CSRC, "floors.hip"), "-o", FLOORS])
    jobs = [lambda c=c: _run(c, verbose) for c in cmds]
    jobs += [lambda f=f: _check_asm(f, tuple(extra_flags), bdir, verbose) for f in ASM_CHECKED]
    with ThreadPoolExecutor(max_workers=8) as ex:
        for fut in [ex.submit(j) for j in jobs]:
            fut.result()
    _run([HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", lib, *objs], verbose)
    return lib


if __name__ == "__main__":
    if "--sanitize" in sys.argv:
        print("built and ran", build_sanitized(verbose="-q" not in sys.argv))
    else:
        flags = (TRACKED_FLAG,) if "--tracked-merge-loads" in sys.argv else ()
        print("built", build(verbose="-q" not in sys.argv, extra_flags=flags, trace="--trace" in sys.argv))
