"""The stage runtime's host logic on the CPU (no GPU): the message admission of Alg. 2's receive loop, the stash
slots under pipeline_limit (Sec. 3.3), duplicate / surplus messages, the per-wait time limit, the weight-gradient
groups, the optimizer's bucket plan (Sec. 5.2) and the chunk -> lowest-layer gate of the overlapped step (Sec. 5.3).
tests/host/host_logic_test.cpp drives paper_2110_13005_amd/csrc/host_logic.h (the header stage.cpp takes these
decisions from) with a simulated event layer; it is built and run twice: with the address + undefined-behaviour
sanitizers and with the thread sanitizer."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "host", "host_logic_test.cpp")


def _build_and_run(tmp_path, name, flags):
    gxx = shutil.which("g++")
    if not gxx:
        pytest.skip("no g++")
    exe = str(tmp_path / name)
    cmd = [gxx, "-std=c++17", "-O1", "-g", "-Wall", "-Wextra", "-Werror", *flags, SRC, "-o", exe, "-pthread"]
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1",
               TSAN_OPTIONS="halt_on_error=1")
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
    assert r.returncode == 0, (r.stdout + r.stderr)[-3000:]
    assert "all checks passed" in r.stdout
    assert "runtime error" not in r.stderr and "Sanitizer" not in r.stderr, r.stderr[-3000:]


def test_host_logic_address_and_undefined_behaviour_sanitizers(tmp_path):
    _build_and_run(tmp_path, "hl_asan", ["-fsanitize=address,undefined", "-fno-sanitize-recover=all"])


def test_host_logic_thread_sanitizer(tmp_path):
    _build_and_run(tmp_path, "hl_tsan", ["-fsanitize=thread"])


def test_stage_runtime_takes_its_decisions_from_the_tested_header():
    """stage.cpp must call the functions the CPU tests exercise, not private copies of them."""
    src = open(os.path.join(os.path.dirname(HERE), "paper_2110_13005_amd", "csrc", "stage.cpp")).read()
    for fn in ("host::choose_message", "host::admit_forward", "host::commit_forward", "host::admit_backward",
               "host::commit_backward", "host::wgrad_action", "host::release_awaiting", "host::check_post",
               "host::stream_index", "host::WaitClock", "host::bucket_plan", "host::chunk_span", "host::lowest_layer"):
        assert fn in src, fn
