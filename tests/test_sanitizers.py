"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only): the C oracle, driven through
its pins, and the plain C client of the library's ABI."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1"]


def runtime(name):
    path = subprocess.check_output(["gcc", "-print-file-name=" + name], text=True).strip()
    if not os.path.isabs(path):
        pytest.skip("gcc has no %s" % name)
    return path


def san_env(**extra):
    env = dict(os.environ)
    # the sanitizer runtime has to come first among the preloaded libraries; whatever is preloaded already stays
    env["LD_PRELOAD"] = " ".join([runtime("libasan.so")] + ([env["LD_PRELOAD"]] if env.get("LD_PRELOAD") else []))
    # the Python interpreter itself is not instrumented: its arena allocator is not a leak of ours
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:exitcode=99"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1:exitcode=98"
    env.update(extra)
    return env


def test_oracle_pins_under_asan_and_ubsan(tmp_path):
    lib = tmp_path / "liboracle_san.so"
    subprocess.check_call(["gcc"] + SAN + ["-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra",
                                           os.path.join(ROOT, "oracle", "la2_oracle.c"), "-o", str(lib), "-lm"])
    res = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                          "-p", "no:cacheprovider"],
                         cwd=ROOT, env=san_env(LA2_ORACLE_LIB=str(lib), OMP_NUM_THREADS="4"),
                         stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=900)
    assert res.returncode == 0, res.stdout[-4000:]
    assert "passed" in res.stdout and "ERROR: AddressSanitizer" not in res.stdout and "runtime error" not in res.stdout


def test_abi_client_under_asan_and_ubsan(tmp_path):
    from paper_2401_04658_amd import binding
    if not os.path.exists(binding.lib_path()):
        from paper_2401_04658_amd.build import build
        build()
    exe = tmp_path / "abi_client_san"
    libdir = os.path.dirname(binding.lib_path())
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror"] + SAN +
                          ["-I", os.path.join(ROOT, "include"), os.path.join(ROOT, "tests", "abi_client.c"), "-o", str(exe),
                           "-L", libdir, "-l:libla2.so", "-Wl,-rpath," + libdir])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:exitcode=99", UBSAN_OPTIONS="halt_on_error=1:exitcode=98")
    res = subprocess.run([str(exe)], env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    assert res.returncode == 0 and "abi client ok" in res.stdout, (res.returncode, res.stdout[-3000:])
