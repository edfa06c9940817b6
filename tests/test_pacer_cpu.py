"""Host logic of the chunk-command issue pacing (no GPU): spacing of consecutive commands by the previous command's
link time, and the upward-only ratchet of the link rate from sustained windows."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def harness(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("pacer") / "pacer_harness")
    subprocess.check_call(["g++", "-std=c++17", "-O1", "-Wall", "-Werror", "-I",
                           os.path.join(ROOT, "paper_2604_26557_amd", "csrc"),
                           os.path.join(ROOT, "tests", "pacer_harness.cpp"), "-o", exe])
    return exe


def _run(exe, *args):
    out = subprocess.check_output([exe, *map(str, args)], text=True)
    vals = {}
    for line in out.splitlines():
        k, *v = line.split()
        vals.setdefault(k, []).append(v)
    return vals


def test_spacing_is_the_previous_commands_link_time(harness):
    r = _run(harness, 50e9, 3, 56e9)
    assert r["enabled"] == [["1"]]
    assert float(r["due_first"][0][0]) < 0                      # nothing before the first command
    bytes_ = 512 * 1024
    tau = bytes_ / (1.02 * 50e9)                                 # 2 % headroom over the measured rate
    assert float(r["due_second"][0][0]) == pytest.approx(1.0 + tau, abs=1e-12 * 2)
    # the second command had twice the bytes: the third waits twice as long after it
    assert float(r["due_third"][0][0]) == pytest.approx(1.0 + tau + 2 * tau, abs=1e-12 * 2)
    # two free slots (the queue has fallen behind): half the spacing, so that it fills up again
    assert float(r["due_third_behind"][0][0]) == pytest.approx(1.0 + tau + tau, abs=1e-12 * 2)
    # the copy-kernel engine's setting: no catch-up
    assert float(r["due_third_behind_no_catch_up"][0][0]) == pytest.approx(1.0 + tau + 2 * tau, abs=1e-12 * 2)


@pytest.mark.parametrize("depth", [2, 3, 8])
def test_rate_ratchets_up_after_three_windows_and_never_down(harness, depth):
    r = _run(harness, 50e9, depth, 56e9)
    rates = [float(v[1]) for v in r["rate_after_window"]]
    above = [int(v[3]) for v in r["rate_after_window"]]
    # the first harvest only opens a window; windows 0 and 1 count up, window 2 moves the rate to what was sustained
    assert rates[0] == 50e9 and rates[1] == 50e9 and above[:2] == [1, 2]
    assert rates[2] == pytest.approx(56e9, rel=1e-6) and above[2] == 0
    assert all(b >= a for a, b in zip(rates, rates[1:]))
    assert rates[-1] == pytest.approx(56e9, rel=1e-6)            # sustained = rate: no further movement
    # a link slower than the measured rate never pulls it down
    r = _run(harness, 50e9, depth, 30e9)
    assert all(float(v[1]) == 50e9 for v in r["rate_after_window"])


def test_unwaited_completions_do_not_end_a_window_and_switches(harness):
    r = _run(harness, 50e9, 3, 56e9)
    assert float(r["rate_unwaited"][0][0]) == 10e9
    assert r["enabled_no_rate"] == [["0"]] and r["enabled_depth1"] == [["0"]] and r["enabled_off"] == [["0"]]
