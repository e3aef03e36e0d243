"""Host sanitizers over the CPU-side code (no GPU, no GPU sanitizer): the C oracle and the CPU build of the HIP
library's device bit logic are compiled with -fsanitize=address,undefined (gcc / g++, runtime linked statically) into
one small program, tests/sanitize/san_main.cpp, which runs a reduced pin set through both, compares them element by
element and exercises the oracle's array entry points on empty, tiny and ragged arrays."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
FLAGS = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"]


@pytest.mark.skipif(shutil.which("gcc") is None or shutil.which("g++") is None, reason="needs gcc and g++")
def test_oracle_and_device_logic_are_clean_under_asan_and_ubsan(tmp_path):
    objs = []
    for cc, src, extra in (
            ("gcc", os.path.join(ROOT, "oracle", "hif8_oracle.c"), ["-fopenmp", "-ffp-contract=off", "-fno-fast-math"]),
            ("g++", os.path.join(HERE, "devfn_host", "devfn_host.cpp"), ["-std=c++17", "-ffp-contract=off"]),
            ("g++", os.path.join(HERE, "sanitize", "san_main.cpp"), ["-std=c++17"])):
        obj = str(tmp_path / (os.path.basename(src) + ".o"))
        subprocess.run([cc] + FLAGS + extra + ["-c", src, "-o", obj], check=True)
        objs.append(obj)
    exe = str(tmp_path / "san_main")
    subprocess.run(["g++", "-fsanitize=address,undefined", "-static-libasan", "-fopenmp"] + objs + ["-o", exe, "-lm"], check=True)
    syms = subprocess.run(["nm", exe], stdout=subprocess.PIPE, text=True, check=True).stdout
    assert "__asan_init" in syms and "__ubsan_handle" in syms, "the sanitizer runtimes are not linked in"
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1", OMP_NUM_THREADS="4")
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stdout[-4000:]
    assert "sanitize OK" in r.stdout and "0 mismatches" in r.stdout, r.stdout[-2000:]
