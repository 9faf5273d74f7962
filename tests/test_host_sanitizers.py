"""The library's host code (tree selection and its thread pool, the baseline policy, the product
forest, Algorithm 1 layer by layer, the cost-model fit) and the oracle's C routine under the
host sanitizers: tests/sanitize/host_driver.cpp built with -fsanitize=address,undefined and with
-fsanitize=thread (batches of 0 .. 256 sequences, four caller threads at once), and
tests/sanitize/oracle_driver.c built with -fsanitize=address,undefined.  A sanitizer report of
any kind fails the test.  (GPU code is not built here: no sanitizer runs on the device.)"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2604_09731_amd", "csrc")
DRIVERS = os.path.join(ROOT, "tests", "sanitize")
HOST_SOURCES = [os.path.join(DRIVERS, "host_driver.cpp"), os.path.join(CSRC, "smart_select.cpp"),
                os.path.join(CSRC, "smart_cost_model.cpp")]
REPORTS = ("ERROR: AddressSanitizer", "ERROR: LeakSanitizer", "runtime error:", "WARNING: ThreadSanitizer",
           "ThreadSanitizer:")


def _build_and_run(tmp_path, compiler, flags, sources, name, libs=()):
    exe = os.path.join(str(tmp_path), name)
    cmd = [compiler, "-O1", "-g", "-fno-omit-frame-pointer", "-ffp-contract=off", *flags, "-I", os.path.join(ROOT, "include"),
           *sources, "-pthread", *libs, "-o", exe]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    env = dict(os.environ)
    env.pop("LD_PRELOAD", None)          # a sanitizer's runtime has to be the first library loaded
    r = subprocess.run([exe], capture_output=True, text=True, timeout=600, env=env)
    text = r.stdout + r.stderr
    for marker in REPORTS:
        assert marker not in text, text[-4000:]
    assert r.returncode == 0, text[-4000:]
    return text


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_host_code_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    out = _build_and_run(tmp_path, "g++", ["-std=c++17", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"],
                         HOST_SOURCES, "host_asan")
    assert "host driver ok" in out


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_selection_thread_pool_under_thread_sanitizer(tmp_path):
    out = _build_and_run(tmp_path, "g++", ["-std=c++17", "-fsanitize=thread"], HOST_SOURCES, "host_tsan")
    assert "host driver ok" in out


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_c_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    out = _build_and_run(tmp_path, "gcc", ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fopenmp"],
                         [os.path.join(DRIVERS, "oracle_driver.c"), os.path.join(ROOT, "oracle", "tree_attention_ref.c")],
                         "oracle_asan", libs=("-lm",))
    assert "oracle driver ok" in out
