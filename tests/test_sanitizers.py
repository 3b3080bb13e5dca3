"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only; nothing here touches a GPU).

The host part of the library (pack, unpack, schedule, static-scheduler search: pmpd_host.cpp) and the C
oracle are each compiled with -fsanitize=address,undefined into a small program with a driver from
tests/sanitize/ and run.  The programs are stand-alone (sanitizer runtimes linked statically) so that the
runtime is first in the process whatever the environment preloads; a report from either sanitizer ends
the program with a non-zero status (-fno-sanitize-recover)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan", "-g", "-O1",
       "-fno-omit-frame-pointer"]


def _build_and_run(tmp_path, compiler, sources, extra, name):
    if shutil.which(compiler) is None:
        pytest.skip(f"{compiler} not installed")
    exe = str(tmp_path / name)
    cmd = [compiler, *SAN, *extra, "-o", exe, *sources]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1", OMP_NUM_THREADS="4")
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=300)
    assert run.returncode == 0, run.stdout[-4000:]
    assert f"{name}: ok" in run.stdout


def test_host_library_under_asan_and_ubsan(tmp_path):
    src = [os.path.join(ROOT, "tests", "sanitize", "host_driver.cpp"),
           os.path.join(ROOT, "paper_2410_13461_amd", "csrc", "pmpd_host.cpp")]
    inc = ["-std=c++17", "-pthread", "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(ROOT, "paper_2410_13461_amd", "csrc")]
    _build_and_run(tmp_path, "g++", src, inc, "host_driver")


def test_oracle_under_asan_and_ubsan(tmp_path):
    src = [os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"), os.path.join(ROOT, "oracle", "pmpd_oracle.c")]
    _build_and_run(tmp_path, "gcc", src, ["-std=c11", "-fopenmp", "-lm"], "oracle_driver")


def test_sum_words_of_the_ordered_step(tmp_path):
    """part_word / sum_value / whole_word as the kernels use them, compiled for the host: small negative
    parts, the clamp, NaN, 31 parts at either limit, order independence."""
    src = [os.path.join(ROOT, "tests", "sanitize", "sumword_driver.cpp")]
    _build_and_run(tmp_path, "g++", src, ["-std=c++17", "-I" + os.path.join(ROOT, "paper_2410_13461_amd", "csrc")], "sumword_driver")


def test_prefill_deal_covers_every_item_once(tmp_path):
    """pf_grid / pf_share as the prefill launcher and kernel use them, compiled for the host: every (item, token block)
    taken exactly once, shares balanced to one item, one token block per XCD in the XCD-aware deal."""
    src = [os.path.join(ROOT, "tests", "sanitize", "deal_driver.cpp")]
    _build_and_run(tmp_path, "g++", src, ["-std=c++17", "-I" + os.path.join(ROOT, "paper_2410_13461_amd", "csrc")], "deal_driver")
