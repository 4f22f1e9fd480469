"""The dynamic scheduler's ready-queue protocol, emulated on the CPU with one thread per workgroup
(tests/dyn_queue_emulation.cpp): exactly-once execution, drained counters and termination over several
launches, including the early push (a task is pushed once the producers of all its events are dispatched)
and a task that waits on two events.  The device kernel has its own GPU tests; this one checks the protocol
where a mistake in it shows as a failed count or a time-out instead of a hung GPU."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))


def test_ready_queue_protocol_terminates_and_runs_every_task_once(tmp_path):
    exe = tmp_path / "dyn_emul"
    subprocess.check_call(["g++", "-O2", "-std=c++17", "-pthread", "-o", str(exe),
                           os.path.join(HERE, "dyn_queue_emulation.cpp")])
    for n, wgs in ((1, 16), (5, 3), (37, 64)):
        out = subprocess.run([str(exe), str(n), str(wgs)], capture_output=True, text=True, timeout=120)
        assert out.returncode == 0, out.stdout + out.stderr
        assert out.stdout.count(": ok") == 3
    # data-dependent update and trigger (run-time counts, indptr ranges, surplus tasks that are never released)
    for n, wgs, groups, surplus in ((1, 4, 1, 0), (24, 16, 5, 7), (40, 64, 3, 1)):
        out = subprocess.run([str(exe), str(n), str(wgs), str(groups), str(surplus)], capture_output=True, text=True,
                             timeout=120)
        assert out.returncode == 0, out.stdout + out.stderr
        assert out.stdout.count(": ok") == 3


def test_dispatch_loop_bound_ends_a_loop_that_repeats_its_task(tmp_path):
    """The defect that once hung the device loop (a workgroup whose pop never runs, so it repeats one task),
    planted here on the CPU: the loop's own iteration bound must end the run with an error, not spin."""
    exe = tmp_path / "dyn_emul"
    subprocess.check_call(["g++", "-O2", "-std=c++17", "-pthread", "-o", str(exe),
                           os.path.join(HERE, "dyn_queue_emulation.cpp")])
    out = subprocess.run([str(exe), "9", "8"], capture_output=True, text=True, timeout=120,
                         env=dict(os.environ, STALE_WG="2"))
    assert out.returncode == 3, out.stdout + out.stderr
    assert "drained on the loop bound" in out.stdout
