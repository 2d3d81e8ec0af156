"""CPU sanitizer runs of the host-side code (no GPU needed).

* AddressSanitizer + UndefinedBehaviorSanitizer: the C oracle (oracle/fc_oracle.c) and the input generator's C part
  (workloads/fill.c) are rebuilt with -fsanitize=address,undefined and the oracle's pin battery plus the workload tests
  run against those builds in a child process (the sanitizer runtime has to be loaded before the interpreter starts).
* ThreadSanitizer: the scatter pool of the DMA evict transmitter (csrc/scatter_pool.h: publish / in-order completion /
  wait / buffer reuse) is built without any GPU runtime, with a mocked "block has landed" signal, and run under
  -fsanitize=thread (tests/tsan_scatter_pool.cpp checks ordering and the final table as well), and so are the host
  threads of the DMA miss path (csrc/gather_pool.h, tests/tsan_gather_pool.cpp).
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _have(cmd):
    try:
        return subprocess.run(cmd, capture_output=True).returncode == 0
    except OSError:
        return False


def test_oracle_and_fill_under_asan_ubsan(tmp_path):
    libasan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(libasan) or not os.path.exists(libasan):
        pytest.skip("no libasan in this toolchain")
    flags = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
             "-ffp-contract=off", "-shared", "-fPIC"]
    oracle_so, fill_so = str(tmp_path / "libfc_oracle_san.so"), str(tmp_path / "libfc_fill_san.so")
    subprocess.check_call(["gcc", "-std=c11", "-fno-fast-math", *flags, os.path.join(ROOT, "oracle", "fc_oracle.c"), "-o", oracle_so])
    subprocess.check_call(["gcc", "-fopenmp", *flags, os.path.join(ROOT, "workloads", "fill.c"), "-o", fill_so, "-lm"])
    env = dict(os.environ, FC_ORACLE_LIB=oracle_so, FC_FILL_LIB=fill_so,
               LD_PRELOAD=" ".join(x for x in (libasan, os.environ.get("LD_PRELOAD", "")) if x),
               ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0:abort_on_error=0:halt_on_error=1",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1", OMP_NUM_THREADS="4")
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        "tests/test_oracle_pins.py", "tests/test_oracle_dirty.py", "tests/test_workloads.py"],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert "AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr, tail
    assert " passed" in r.stdout, tail


def test_gather_pool_under_tsan(tmp_path):
    """The host threads of the DMA miss path (csrc/gather_pool.h) with mocked copies: every row gathered once and sent once,
    a chunk sent only when complete, one arrival mark per job and after every send, failures reported once."""
    exe = str(tmp_path / "tsan_gather_pool")
    src = os.path.join(ROOT, "tests", "tsan_gather_pool.cpp")
    inc = os.path.join(ROOT, "paper_2208_05321_amd", "csrc")
    c = subprocess.run(["g++", "-std=c++17", "-O1", "-g", "-fsanitize=thread", "-pthread", "-I", inc, src, "-o", exe],
                       capture_output=True, text=True)
    if c.returncode != 0 and "tsan" in c.stderr.lower():
        pytest.skip("no libtsan in this toolchain")
    assert c.returncode == 0, c.stderr[-2000:]
    for jobs, threads in ((200, 6), (120, 3), (60, 1)):
        r = subprocess.run([exe, str(jobs), str(threads)], capture_output=True, text=True, timeout=300,
                           env=dict(os.environ, TSAN_OPTIONS="halt_on_error=1"))
        if "unexpected memory mapping" in r.stderr:
            pytest.skip("ThreadSanitizer cannot map its shadow memory on this kernel")
        assert r.returncode == 0 and "ThreadSanitizer" not in r.stderr, (r.stdout + r.stderr)[-3000:]
        assert r.stdout.startswith("ok:")


def test_scatter_pool_under_tsan(tmp_path):
    exe = str(tmp_path / "tsan_scatter_pool")
    src = os.path.join(ROOT, "tests", "tsan_scatter_pool.cpp")
    inc = os.path.join(ROOT, "paper_2208_05321_amd", "csrc")
    c = subprocess.run(["g++", "-std=c++17", "-O1", "-g", "-fsanitize=thread", "-pthread", "-I", inc, src, "-o", exe],
                       capture_output=True, text=True)
    if c.returncode != 0 and "tsan" in c.stderr.lower():
        pytest.skip("no libtsan in this toolchain")
    assert c.returncode == 0, c.stderr[-2000:]
    for blocks, threads in ((400, 8), (150, 3), (60, 1)):
        r = subprocess.run([exe, str(blocks), str(threads)], capture_output=True, text=True, timeout=300,
                           env=dict(os.environ, TSAN_OPTIONS="halt_on_error=1"))
        if "unexpected memory mapping" in r.stderr:
            pytest.skip("ThreadSanitizer cannot map its shadow memory on this kernel")
        assert r.returncode == 0 and "ThreadSanitizer" not in r.stderr, (r.stdout + r.stderr)[-3000:]
        assert r.stdout.startswith("ok:")
