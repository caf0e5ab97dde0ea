"""Host code under sanitizers: the library's pool state machine (pool_core.cpp) and the oracle
(ellm_oracle.c), built from source with AddressSanitizer + UndefinedBehaviorSanitizer and, for the
oracle's threaded decode, ThreadSanitizer, and driven in lock step by tests/sanitize_walk.cpp; the
mapper thread of driver-mapped pools (map_queue.hpp) with a stand-in for the driver, under both
(tests/sanitize_mapq.cpp). Device code is not covered: sanitizers for it do not exist on the target boxes."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2506_15155_amd", "csrc")


def _build(tmp, name, san):
    gcc, gxx = shutil.which("gcc"), shutil.which("g++")
    if not gcc or not gxx:
        pytest.skip("no host compiler")
    obj = os.path.join(tmp, name + "_orc.o")
    exe = os.path.join(tmp, name)
    common = ["-g", "-O1", "-fsanitize=" + san, "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"]
    subprocess.run([gcc, "-std=c11", *common, "-c", os.path.join(ROOT, "oracle", "ellm_oracle.c"), "-o", obj], check=True)
    subprocess.run([gxx, "-std=c++17", *common, "-I", CSRC, os.path.join(ROOT, "tests", "sanitize_walk.cpp"),
                    os.path.join(CSRC, "pool_core.cpp"), obj, "-lpthread", "-lm", "-o", exe], check=True)
    return exe


def _run(exe, *args):
    r = subprocess.run([exe, *map(str, args)], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    assert "states equal throughout" in r.stdout


def test_address_and_undefined_behaviour(tmp_path):
    exe = _build(str(tmp_path), "walk_asan", "address,undefined")
    for seed in (1, 2, 3, 4):       # seed 4: tokens per chunk not a power of two, slack bytes in the chunk
        _run(exe, seed, 2500)


def test_threads_of_the_oracle_decode(tmp_path):
    exe = _build(str(tmp_path), "walk_tsan", "thread")
    _run(exe, 5, 1200, 4)


@pytest.mark.parametrize("san", ["thread", "address,undefined"])
def test_mapper_thread_of_driver_mapped_pools(tmp_path, san):
    gxx = shutil.which("g++")
    if not gxx:
        pytest.skip("no host compiler")
    exe = os.path.join(str(tmp_path), "mapq")
    subprocess.run([gxx, "-std=c++17", "-g", "-O1", "-fsanitize=" + san, "-fno-sanitize-recover=all",
                    "-fno-omit-frame-pointer", "-I", CSRC, os.path.join(ROOT, "tests", "sanitize_mapq.cpp"),
                    "-lpthread", "-o", exe], check=True)
    for seed in (1, 2, 3):
        r = subprocess.run([exe, str(seed), "600"], capture_output=True, text=True, timeout=300)
        assert r.returncode == 0 and "mapper queue behaves" in r.stdout, r.stdout[-2000:] + r.stderr[-4000:]
