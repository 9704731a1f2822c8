"""The bounds-checked host emulator is what stands between a planner mistake and a GPU memory fault (the GPU
fuzz test runs every random plan through it before any launch).  Shown on the CPU with a planted mistake: the
planner is built host-only twice, as it is and from a copy whose lowering shifts every target offset by one
16-byte unit; the emulator accepts the first and refuses the second with LIVER_E_HIP (the code for an access
that would fault on the device) instead of touching memory outside a buffer."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2605_22014_amd", "csrc")
GOOD = "v.b_off = (uint64_t)(d.dst_off * eb);"
PLANTED = "v.b_off = (uint64_t)(d.dst_off * eb) + 16;"


def _build_and_run(tmp_path, planner_source, tag):
    exe = str(tmp_path / f"guard_{tag}")
    cmd = ["g++", "-std=c++17", "-O1", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC, planner_source,
           os.path.join(CSRC, "emulate.cpp"), os.path.join(ROOT, "tests", "emulator_guard_main.cpp"), "-o", exe]
    build = subprocess.run(cmd, capture_output=True, text=True)
    assert build.returncode == 0, build.stderr[-3000:]
    run = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert run.returncode == 0, (run.stdout, run.stderr[-2000:])
    return run.stdout


def test_emulator_accepts_the_planner_and_refuses_a_planted_offset_error(tmp_path):
    text = open(os.path.join(CSRC, "planner.cpp")).read()
    assert text.count(GOOD) == 1, "the lowering statement this test mutates has changed"
    assert "verdict: 0" in _build_and_run(tmp_path, os.path.join(CSRC, "planner.cpp"), "good")
    mutant = tmp_path / "planner_mutant.cpp"
    mutant.write_text(text.replace(GOOD, PLANTED))
    out = _build_and_run(tmp_path, str(mutant), "mutant")
    assert "verdict: -4" in out, out                      # LIVER_E_HIP: "this access would fault on the device"


def test_gpu_fuzz_guard_rejects_a_result_that_differs_from_the_oracle():
    """The guard of the GPU fuzz test (proven_on_host) also compares the emulated result with the oracle's: a
    mistake planted in the ORACLE's expectation is reported by it, on the CPU, as it would be before a launch."""
    import numpy as np
    import pytest
    import oracle
    import paper_2605_22014_amd as lv
    from interp import lv_objects
    from util import make_world, tiny_state
    from test_gpu_fuzz import proven_on_host
    spec = oracle.ModelSpec(n_layers=2, hidden=32, n_q_heads=4, n_kv_heads=2, ffn=64, vocab=64, glu=True)
    src, dst = oracle.Layout(2, 1, 2, 8), oracle.Layout(1, 2, 1, 8)
    world = make_world(spec, src, tiny_state(spec, seed=7))
    want = oracle.reshard_state(spec, src, dst, world)
    plan = lv.liver_plan_create(*lv_objects(spec, src, dst), 1024)
    proven_on_host(plan, world, want)
    key = sorted(want)[3]
    want[key] = want[key].copy()
    want[key][5] ^= 1
    with pytest.raises(AssertionError, match="host emulation"):
        proven_on_host(plan, world, want)
