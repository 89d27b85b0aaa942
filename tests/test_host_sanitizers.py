"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only, no GPU involved).

The fp64 oracle (C), the scheduling model and the launch-plan arithmetic (C++, the host parts of the
library that index arrays by computed sizes) are compiled with ``-fsanitize=address,undefined`` into one
program with ``tests/sanitize_host.cpp``, which drives every exported function over ragged, empty and
boundary-sized inputs in exactly-sized buffers and checks hand-derived values and invariants.  The
sanitizer runtimes are linked statically, so nothing has to be preloaded."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2602_11812_amd", "csrc")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]


@pytest.fixture(scope="module")
def program(tmp_path_factory):
    if not (shutil.which("gcc") and shutil.which("g++")):
        pytest.skip("no host compiler")
    out = tmp_path_factory.mktemp("sanitize")
    objs = []
    units = [("gcc", ["-std=c99"], os.path.join(ROOT, "oracle", "egtp_oracle.c")),
             ("g++", ["-std=c++17"], os.path.join(CSRC, "sched.cpp")),
             ("g++", ["-std=c++17"], os.path.join(CSRC, "k1_plan.cpp")),
             ("g++", ["-std=c++17"], os.path.join(ROOT, "tests", "sanitize_host.cpp"))]
    for cc, std, src in units:
        obj = str(out / (os.path.basename(src) + ".o"))
        subprocess.run([cc, *std, *SAN, "-Wall", "-Wno-unknown-pragmas", "-c", src, "-o", obj], check=True)
        objs.append(obj)
    exe = str(out / "sanitize_host")
    subprocess.run(["g++", *SAN, "-static-libasan", "-static-libubsan", "-o", exe, *objs, "-lm"], check=True)
    return exe


def test_host_code_is_clean_under_asan_and_ubsan(program):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:halt_on_error=1", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    r = subprocess.run([program], capture_output=True, text=True, env=env, timeout=600)
    report = r.stdout + r.stderr
    assert r.returncode == 0, report[-4000:]
    assert "AddressSanitizer" not in report and "runtime error" not in report and "LeakSanitizer" not in report, report[-4000:]
    assert "host checks passed" in r.stdout


def test_the_sanitizers_are_armed(program, tmp_path):
    """The same flags do catch a planted heap overflow (in a throw-away program, not in the library)."""
    src = tmp_path / "planted.c"
    src.write_text("#include <stdlib.h>\nint main(void){volatile int *p = malloc(4 * sizeof(int)); int i = 4; p[i] = 1; return p[0];}\n")
    exe = str(tmp_path / "planted")
    subprocess.run(["gcc", *SAN, "-static-libasan", "-static-libubsan", "-o", exe, str(src)], check=True)
    r = subprocess.run([exe], capture_output=True, text=True)
    assert r.returncode != 0 and ("AddressSanitizer" in r.stderr or "runtime error" in r.stderr)
