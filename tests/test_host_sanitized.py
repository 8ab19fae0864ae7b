"""The scheduler's host logic (paged KV allocator, admission, growing pages, preemption, the
prompt queue's books) compiled for the CPU with the address and undefined-behaviour sanitizers
and driven through random walks: tests/host/sched_driver.cpp includes the very headers the
library is built from (csrc/host_sched.h, csrc/page_pool.h), which contain no GPU code."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    cxx = shutil.which("g++")
    if not cxx:
        pytest.skip("no host C++ compiler")
    out = str(tmp_path_factory.mktemp("sched") / "sched_driver")
    cmd = [cxx, "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
           "-static-libasan", "-static-libubsan", "-fno-sanitize-recover=all", "-Wall", "-Wextra", "-Werror",
           os.path.join(ROOT, "tests", "host", "sched_driver.cpp"), "-o", out]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr
    return out


@pytest.mark.parametrize("chunk", [0, 48], ids=["whole-prompts", "chunked"])
@pytest.mark.parametrize("grow", [0, 1], ids=["reserve-all", "growing-pages"])
@pytest.mark.parametrize("pages,slots,prompts", [(40, 12, 60), (14, 6, 40), (200, 24, 120)],
                         ids=["tight", "tiny-pool", "roomy"])
def test_scheduler_random_walk_under_sanitizers(driver, grow, pages, slots, prompts, chunk):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    preempted = sent_back = 0
    for seed in range(1, 9):
        res = subprocess.run([driver, str(seed), str(grow), str(pages), str(slots), str(prompts), str(chunk)],
                             capture_output=True, text=True, env=env, timeout=120)
        assert res.returncode == 0, f"seed {seed}:\n{res.stdout}\n{res.stderr}"
        assert "ERROR" not in res.stderr and "runtime error" not in res.stderr, res.stderr
        print(res.stdout.strip())
        preempted += int(res.stdout.split(" preemptions")[0].split()[-1])
        if chunk:
            assert int(res.stdout.split("chunked: ")[1].split()[0]) > 0
            sent_back += int(res.stdout.split("prompt rows, ")[1].split()[0])
    if chunk and grow:
        assert sent_back > 0          # half-cached prompts gave way and started over
    if grow and pages <= 40:
        assert preempted > 0          # the tight pools do run out and prompts do give way
    if not grow:
        assert preempted == 0
