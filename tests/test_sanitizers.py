"""Sanitizer runs on the CPU (no GPU, no device code): the oracle, and the host side of the C-ABI library
(validation, size queries, planning arithmetic), each built with AddressSanitizer and
UndefinedBehaviorSanitizer and driven by a small C program under tests/sanitize/."""
import os
import shutil
import subprocess
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent
SAN = ROOT / "tests" / "sanitize"
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
CLANG = "/opt/rocm/lib/llvm/bin/clang"      # the host compiler hipcc drives: links the host-only objects
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")


def run(cmd, **kw):
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    assert p.returncode == 0, f"{' '.join(map(str, cmd))}\n{p.stdout[-4000:]}"
    return p.stdout


def test_oracle_under_asan_and_ubsan(tmp_path):
    exe = tmp_path / "oracle_san"
    run(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
         "-fno-omit-frame-pointer", "-o", str(exe), str(SAN / "oracle_driver.c"), str(ROOT / "oracle" / "lookupffn_oracle.c"),
         "-lm"])
    out = run([str(exe)], env=ENV, timeout=600)
    assert "oracle ran clean" in out and "runtime error" not in out and "AddressSanitizer" not in out


@pytest.mark.skipif(not (shutil.which(HIPCC) and shutil.which(CLANG)), reason="hipcc / clang not found")
def test_library_host_code_under_asan_and_ubsan(tmp_path):
    """Host pass only (--cuda-host-only: the kernels get their launch stubs, no device code is generated);
    the sanitizer flags go to the host compiler.  The host object refers to the device-code bundle that a
    full build embeds; an empty bundle stands in for it (nothing here launches a kernel)."""
    inc = ["-I" + str(ROOT / "include"), "-I" + str(ROOT / "paper_2403_07221_amd" / "csrc")]
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined"]
    obj = tmp_path / "lookupffn_host.o"
    run([HIPCC, "--cuda-host-only", "-O1", "-g", "-std=c++17", "-fPIC", "-fno-omit-frame-pointer", *san,
         "-Wno-unused-command-line-argument", *inc, "-c", "-o", str(obj),
         str(ROOT / "paper_2403_07221_amd" / "csrc" / "lookupffn.hip")], timeout=900)
    undefined = [l.split()[-1] for l in run(["nm", "-u", str(obj)]).splitlines() if "__hip_fatbin_" in l]
    assert len(undefined) == 1, undefined
    stub = tmp_path / "empty_bundle.c"
    stub.write_text(
        "/* an offload bundle with no entries: the magic string and a zero count */\n"
        f"const unsigned char {undefined[0]}[4096] __attribute__((section(\".hip_fatbin\"), aligned(4096))) =\n"
        "    \"__CLANG_OFFLOAD_BUNDLE__\";\n")
    lib = tmp_path / "liblookupffn_san.so"
    host_san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"]
    run([CLANG + "++", "-shared", "-fPIC", *host_san, "-o", str(lib), str(obj), "-x", "c", str(stub),
         "-L/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib"], timeout=300)
    exe = tmp_path / "host_san"
    run([CLANG, "-O1", "-g", *host_san, *inc, "-o", str(exe), str(SAN / "host_driver.c"), str(lib),
         "-Wl,-rpath," + str(tmp_path)], timeout=300)
    out = run([str(exe)], env=ENV, timeout=300)
    assert "host code ran clean" in out and "runtime error" not in out and "AddressSanitizer" not in out
