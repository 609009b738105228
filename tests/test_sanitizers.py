"""CPU sanitizer tier: the oracle's C source and the library's host-only sources (the BatchNorm fold and
the version / status / size helpers) are rebuilt with AddressSanitizer and UndefinedBehaviorSanitizer, and
the oracle pins and the exhaustive fold tests run against those builds in a child process.  Any report
(an out-of-bounds access, a signed overflow, a misaligned or invalid shift, ...) ends the child with a
non-zero status.  Device code is not instrumented: sanitizers run on host code only.
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ORACLE_SRC = os.path.join(ROOT, "oracle", "bnn_oracle.c")
CSRC = os.path.join(ROOT, "paper_1602_02830_amd", "csrc")
INCLUDE = os.path.join(ROOT, "include")

SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]


def _asan_runtime():
    path = subprocess.run(["gcc", "-print-file-name=libasan.so"], stdout=subprocess.PIPE, text=True, check=True).stdout.strip()
    if not os.path.isabs(path) or not os.path.exists(path):
        pytest.skip("this compiler ships no AddressSanitizer runtime")
    return os.path.realpath(path)


def _build_oracle(so_path, src=ORACLE_SRC):
    subprocess.run(["gcc", *SAN, "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-std=c99", "-Wall", "-Wextra",
                    "-shared", "-fPIC", src, "-o", so_path, "-lm"], check=True)
    return so_path


def _build_host_sources(so_path):
    """bn_fold.cpp and api.cpp are the library's host-only translation units (no HIP in them)."""
    subprocess.run(["g++", *SAN, "-std=c++17", "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra", f"-I{INCLUDE}",
                    "-shared", "-fPIC", os.path.join(CSRC, "bn_fold.cpp"), os.path.join(CSRC, "api.cpp"), "-o", so_path],
                   check=True)
    return so_path


def _run_child(pytest_args, **extra_env):
    """pytest in a child process whose first loaded library is the sanitizer runtime (an instrumented
    shared object cannot be loaded into an uninstrumented process otherwise)."""
    preload = _asan_runtime()
    if os.environ.get("LD_PRELOAD"):
        preload += ":" + os.environ["LD_PRELOAD"]
    env = dict(os.environ, LD_PRELOAD=preload, OMP_NUM_THREADS="2",
               # Python itself is not leak-clean; the link-order check is for preloads the environment adds.
               ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0:abort_on_error=0:exitcode=86",
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1:exitcode=87", **extra_env)
    # -s: a sanitizer report is written to the process's own stderr right before it exits, which pytest's
    # capture would swallow.
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-s", "-p", "no:cacheprovider", *pytest_args], env=env,
                       cwd=ROOT, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    return r.returncode, r.stdout


def _assert_clean(rc, out):
    assert rc == 0, out[-3000:]
    assert "AddressSanitizer" not in out and "runtime error:" not in out, out[-3000:]


def test_oracle_pins_under_address_and_ub_sanitizers(tmp_path):
    so = _build_oracle(str(tmp_path / "oracle_san.so"))
    rc, out = _run_child([os.path.join("tests", "test_oracle_pins.py")], BNN_ORACLE_LIB=so)
    _assert_clean(rc, out)
    assert " passed" in out


def test_fold_and_size_helpers_under_address_and_ub_sanitizers(tmp_path):
    """The exhaustive check of bnn_bn_fold (every integer s in [-K, K], every channel) with BOTH sides
    instrumented: the fold from the sanitizer build of the host sources, the float BatchNorm + Sign
    from the sanitizer build of the oracle."""
    oracle_so = _build_oracle(str(tmp_path / "oracle_san.so"))
    host_so = _build_host_sources(str(tmp_path / "host_san.so"))
    rc, out = _run_child([os.path.join("tests", "test_host_logic.py"), "-k", "fold or words_per_row"],
                         BNN_ORACLE_LIB=oracle_so, BNN_HOST_LIB=host_so)
    _assert_clean(rc, out)
    assert " passed" in out


def test_the_sanitizers_are_live(tmp_path):
    """Control: an out-of-bounds write planted in a copy of the oracle (the packer writes one word past
    each row) must end the same child run with a sanitizer report."""
    text = open(ORACLE_SRC).read()
    old = "words[r * kw + k / 32] |= (uint32_t)1 << (k % 32);"
    assert text.count(old) == 1
    src = tmp_path / "oracle_oob.c"
    src.write_text(text.replace(old, "words[(r + 1) * kw + k / 32] |= (uint32_t)1 << (k % 32);"))
    so = _build_oracle(str(tmp_path / "oracle_oob.so"), str(src))
    rc, out = _run_child([os.path.join("tests", "test_oracle_pins.py"), "-k", "pack"], BNN_ORACLE_LIB=so)
    assert rc == 86 and "AddressSanitizer" in out, out[-2000:]
