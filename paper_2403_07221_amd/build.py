"""Builds the C-ABI library (hand-written HIP for gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
from pathlib import Path

PKG = Path(__file__).resolve().parent
ROOT = PKG.parent
SRC = PKG / "csrc" / "lookupffn.hip"
LIB = PKG / "liblookupffn.so"
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

N_PARTS = 17         # csrc/lookupffn.hip compiles as parts 0 .. 16 (-DLFFN_PART=i), linked together
SLOW_FIRST = [10, 11, 8, 9, 6, 5]   # the wide BH kernels take the longest: start them first
OBJ_DIR = PKG / "_build"
# Per-part compiler settings.  Part 16 is the staged gather's plain 13-slot, 128-byte-slice kernel: with the
# instruction scheduler set to favour instruction-level parallelism it measured 4 % faster (93.5 against 97.4 us
# for 16384 tokens x 96 tables, alternating runs on one machine); the 64-byte-slice kernels measured 4 % slower
# with it, so they stay with the default.
PART_FLAGS = {16: ["-mllvm", "-amdgpu-sched-strategy=max-ilp"]}

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-ffp-contract=off",                                        # butterflies must stay add/sub
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",  # no packed-fp32 code generation
    "-Wall", "-Wno-unused-command-line-argument", "-Wno-unused-function",
    f"-I{ROOT / 'include'}", f"-I{PKG / 'csrc'}",
]
_NOISE = "is not a recognized feature for this target"


def _quiet(stderr: str) -> str:
    return "\n".join(l for l in stderr.splitlines() if _NOISE not in l)


def build_library(verbose: bool = False, jobs: int | None = None, only_parts=None) -> Path:
    """Compile the parts of csrc/lookupffn.hip side by side and link liblookupffn.so (always recompiles).

    `only_parts` (development aid; `python -m paper_2403_07221_amd.build 0 12`): recompile just these parts and
    link them with the other parts' objects kept from the last such build in _build/ (a part whose object is
    missing is compiled too).  The objects are then kept -- a part whose sources changed since must be named again, or
    the link takes its stale object; a plain call compiles everything, keeps nothing and drops the kept objects."""
    jobs = jobs or max(1, min(os.cpu_count() or 1, int(os.environ.get("MAX_JOBS", "16"))))
    OBJ_DIR.mkdir(exist_ok=True)
    keep = only_parts is not None
    tag = "dev" if keep else str(os.getpid())
    objs = [OBJ_DIR / f"lookupffn_part{i}.{tag}.o" for i in range(N_PARTS)]
    cmds = [[HIPCC, *FLAGS, *PART_FLAGS.get(i, []), f"-DLFFN_PART={i}", "-c", "-o", str(objs[i]), str(SRC)]
            for i in range(N_PARTS)]
    tmp = LIB.with_suffix(f".so.tmp{os.getpid()}")
    try:
        order = SLOW_FIRST + [i for i in range(N_PARTS) if i not in SLOW_FIRST]
        if keep:
            order = [i for i in order if i in set(only_parts) or not objs[i].exists()]
        todo, running, errors = [(i, cmds[i]) for i in order], [], []
        while todo or running:
            while todo and len(running) < jobs:
                i, cmd = todo.pop(0)
                if verbose:
                    print(" ".join(cmd), flush=True)
                running.append((i, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True)))
            i, proc = running.pop(0)
            _, err = proc.communicate()
            if proc.returncode != 0:
                errors.append(f"part {i}:\n{_quiet(err)}")
            elif verbose and _quiet(err).strip():
                print(_quiet(err), file=sys.stderr)
        if errors:
            raise RuntimeError("hipcc failed:\n" + "\n".join(errors))
        link = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", str(tmp), *map(str, objs)]
        if verbose:
            print(" ".join(link), flush=True)
        r = subprocess.run(link, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"link failed:\n{_quiet(r.stderr)}")
        os.replace(tmp, LIB)
    finally:
        if not keep:
            # a full build also drops the objects a partial build kept: they no longer match the sources
            for o in [*objs, *OBJ_DIR.glob("lookupffn_part*.dev.o")]:
                o.unlink(missing_ok=True)
        tmp.unlink(missing_ok=True)
    return LIB


if __name__ == "__main__":
    parts = [int(a) for a in sys.argv[1:]]
    print(build_library(verbose=not parts, only_parts=parts or None))
