"""Host-side sanitizer builds (CPU only; the GPU side is never run under a sanitizer).

1. The oracle's C source with AddressSanitizer + UndefinedBehaviorSanitizer behind a driver that calls every
   function on heap blocks of exactly the documented sizes (tests/sanitize_oracle_main.c).
2. The product library with its host code (argument checks, launch plans, length bookkeeping) compiled with
   UndefinedBehaviorSanitizer, with the argument-error tests of the C ABI run against it in a child
   process; a report aborts the child.  (AddressSanitizer needs its runtime first in the process, which a Python
   host does not give; the oracle's driver is a program of its own and has it.)"""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
TESTS = os.path.join(ROOT, "tests")


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    exe = str(tmp_path / "oracle_san")
    cmd = [gcc, "-O1", "-g", "-std=c11", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-o", exe, os.path.join(TESTS, "sanitize_oracle_main.c"),
           os.path.join(ROOT, "oracle", "vs_oracle.c"), "-lm"]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and "ok" in r.stdout, r.stdout[-2000:] + r.stderr[-4000:]


def test_library_host_code_under_undefined_behaviour_sanitizer(tmp_path):
    from paper_2503_09387_amd import build
    if not os.path.exists(build.HIPCC):
        pytest.skip("no hipcc")
    build.generate()
    rt = subprocess.run([build.HIPCC, "--print-file-name=libclang_rt.ubsan_standalone-x86_64.so"], capture_output=True,
                        text=True).stdout.strip()
    if not os.path.isabs(rt) or not os.path.exists(rt):
        pytest.skip("the compiler ships no shared UBSan runtime")
    lib = str(tmp_path / "libvideoscan_host_ubsan.so")
    flags = [f for f in build.FLAGS if f != "-O3"]
    # (device code is compiled along, unsanitized and never run here: a host-only object refers to the embedded
    # device binary and would not load)
    cmd = [build.HIPCC] + flags + ["-O1", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
                                   "-fno-sanitize-recover=undefined", "-shared-libsan",
                                   "-Wl,-rpath," + os.path.dirname(rt), "-o", lib] + build.sources()
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    child = (
        "import sys\n"
        f"sys.path[:0] = [{ROOT!r}, {TESTS!r}]\n"
        "from paper_2503_09387_amd import binding\n"
        f"binding.lib_path = lambda: {lib!r}\n"
        "import pytest\n"
        f"sys.exit(pytest.main(['-x', '-q', '-p', 'no:cacheprovider', {os.path.join(TESTS, 'test_boundary.py')!r}, "
        "'-k', 'argument_errors or workspace or tuning or exports']))\n")
    r = subprocess.run([sys.executable, "-c", child], capture_output=True, text=True, timeout=600, cwd=ROOT)
    assert r.returncode == 0 and "passed" in r.stdout, r.stdout[-3000:] + r.stderr[-3000:]
    assert "runtime error" not in r.stderr, r.stderr[-3000:]
