"""The host state machine of a task (cursor, launch-ahead bound, preemption gate: csrc/task_core.h,
the code fp_prefill_advance / fp_preempt / fp_resume / fp_prefill_cursor run on) built for the CPU
with a stand-in device and raced under ThreadSanitizer: signals against a running advance, against
completion, against idle tasks, with the cursor polled from a third thread (Section 5.1: the
scheduler signals, the worker checks between operators and acknowledges)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "tests", "host", "task_core_race.cpp")


def _build(tmp_path, sanitize: bool) -> str:
    cxx = shutil.which("g++") or shutil.which("c++")
    if cxx is None:
        pytest.skip("no host C++ compiler")
    exe = str(tmp_path / ("race_tsan" if sanitize else "race_plain"))
    cmd = [cxx, "-std=c++17", "-O1", "-g", SRC, "-o", exe, "-lpthread"]
    if sanitize:
        cmd.insert(1, "-fsanitize=thread")
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0 and sanitize and "tsan" in r.stdout.lower():
        pytest.skip("ThreadSanitizer runtime not installed")
    assert r.returncode == 0, r.stdout
    return exe


def test_state_machine_invariants_plain_build(tmp_path):
    r = subprocess.run([_build(tmp_path, False), "120"], stdout=subprocess.PIPE, stderr=subprocess.STDOUT,
                       text=True, timeout=120)
    assert r.returncode == 0, r.stdout
    assert "OK" in r.stdout


def test_state_machine_is_race_free_under_thread_sanitizer(tmp_path):
    env = dict(os.environ, TSAN_OPTIONS="halt_on_error=1 exitcode=66")
    r = subprocess.run([_build(tmp_path, True), "120"], stdout=subprocess.PIPE, stderr=subprocess.STDOUT,
                       text=True, timeout=300, env=env)
    assert "ThreadSanitizer" not in r.stdout, r.stdout
    assert r.returncode == 0, r.stdout
    assert "OK" in r.stdout
