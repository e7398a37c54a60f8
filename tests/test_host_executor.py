"""The planner and the executor (csrc/graph.cpp, plan.cpp, engine.hip) built for the HOST with
g++ under AddressSanitizer and UBSan against a stand-in for the HIP runtime (tests/hoststub):
whole iterations of the real instruction-issue code run without a GPU, and the stand-in checks
every event use (alive, recorded in this iteration, timed where a time is read), every copy's
address range and every tensor pointer handed to a kernel launcher.

Covers the combination that is refused on the GPU - event timing of plans that swap more than
24 GiB per iteration (ResNet-152, minibatch 224 / 256, every map swapped, re-planned between
iterations) - with the limit lifted at compile time, and the guard itself: with the limit in
place such a step must return ACC_ESTATE before anything is issued."""
import os
import subprocess

import numpy as np
import pytest

import synth as S

HERE = os.path.dirname(os.path.abspath(__file__))
STUB = os.path.join(HERE, "hoststub")
CSRC = os.path.join(HERE, "..", "paper_1901_06773_amd", "csrc")


@pytest.fixture(scope="module")
def binaries(tmp_path_factory):
    out = tmp_path_factory.mktemp("hoststub")
    srcs = [os.path.join(CSRC, f) for f in ("graph.cpp", "plan.cpp", "engine.hip")] + \
           [os.path.join(STUB, f) for f in ("stub_runtime.cpp", "executor_check.cpp")]
    built = {}
    procs = []
    for name, extra in (("limit", []), ("nolimit", ["-DACC_MAX_TIMED_SWAP_BYTES=((size_t)1<<50)"])):
        exe = str(out / f"executor_check_{name}")
        cmd = ["g++", "-std=c++17", "-g", "-O1", "-fsanitize=address,undefined", "-fno-omit-frame-pointer",
               "-fno-sanitize-recover=undefined", "-I", STUB] + extra + ["-x", "c++"] + srcs + ["-o", exe]
        procs.append((exe, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        built[name] = exe
    for exe, p in procs:
        log, _ = p.communicate()
        assert p.returncode == 0, log[-3000:]
    return built, out


def spec_file(out, net):
    path = str(out / f"{net.name}.bin")
    a = net.as_array()
    with open(path, "wb") as f:
        np.array([a.shape[0], net.in_c, net.in_h, net.in_w], np.int32).tofile(f)
        a.tofile(f)
    return path


def run(exe, spec, scenario):
    p = subprocess.run([exe, spec, scenario], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    return p.returncode, p.stdout


def test_the_stand_in_sees_planted_mistakes(binaries):
    built, out = binaries
    rc, log = run(built["limit"], spec_file(out, S.bottleneck_unit()), "selftest")
    assert rc == 0 and "RESULT: planted mistakes seen" in log, log


def test_timed_iterations_that_swap_every_map_of_resnet152_are_clean_on_the_host(binaries):
    built, out = binaries
    rc, log = run(built["nolimit"], spec_file(out, S.resnet152()), "timed_swap_all")
    assert rc == 0 and "RESULT: clean" in log and "ERROR" not in log, log[-3000:]
    assert "k=256 swapped 310 maps, 40.92 GiB each way" in log
    assert "leaked_events 0" in log


def test_event_timing_above_the_limit_is_refused_before_anything_is_issued(binaries):
    built, out = binaries
    rc, log = run(built["limit"], spec_file(out, S.resnet152()), "guard")
    assert rc == 0 and "guard: status -6" in log and "guard: issued records 0 copies 0 launches 0 events 0" in log, log[-3000:]
    assert "RESULT: clean" in log


def test_graph_mode_records_once_per_plan_and_replays(binaries):
    built, out = binaries
    rc, log = run(built["limit"], spec_file(out, S.resnet152()), "graph")
    assert rc == 0 and "RESULT: clean" in log and "ERROR" not in log, log[-3000:]
    assert "three replays 3 launches and 4 graph launches in all" in log


@pytest.mark.parametrize("net", ["resnet152", "resnet34", "vgg16"])
def test_planner_chosen_swaps_are_clean_on_the_host(binaries, net):
    built, out = binaries
    rc, log = run(built["limit"], spec_file(out, getattr(S, net)()), "dynamic")
    assert rc == 0 and "RESULT: clean" in log and "ERROR" not in log, log[-3000:]
