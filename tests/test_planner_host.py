"""Host-side tests of the C-ABI library that need no GPU: the integer planner against the
brute-force oracle and the hand-worked plans, error codes, and exported symbols."""
import json
import os
import random
import re
import subprocess

import pytest

from oracle import plan_oracle
from paper_2601_11589_amd import api

from test_plan_oracle import load_cases, random_case


def strip(plan):
    return {k: plan[k] for k in ("cls", "bucket", "batches", "longs")}


@pytest.mark.parametrize("case", load_cases(), ids=lambda c: c["name"])
def test_planner_matches_hand_worked_plans(case):
    p = case["params"]
    got = api.laps_plan_buckets(p["short_max_len"], p["len_buckets"], p["depths"], p["token_budget"], p["long_chunk"],
                                case["new_len"], case["prefix_len"])
    assert strip(got) == {k: case[k] for k in ("cls", "bucket", "batches", "longs")}


def test_planner_matches_brute_force_bit_exact():
    rng = random.Random(2601_11589)
    for _ in range(400):
        c = random_case(rng)
        want = plan_oracle.plan_buckets(**c)
        got = api.laps_plan_buckets(**c)
        assert strip(got) == want, c
        # per-request back references agree with the batch lists
        for b, batch in enumerate(got["batches"]):
            for r, i in enumerate(batch["req_ids"]):
                assert got["req_batch"][i] == b and got["req_row"][i] == r
        for lg in got["longs"]:
            assert got["req_batch"][lg["req_id"]] == -1


def test_planner_non_power_of_two_depth_grids_against_brute_force():
    rng = random.Random(7)
    for _ in range(200):
        depths = sorted(rng.sample(range(1, 13), rng.randint(1, 5)))
        n = rng.randint(1, 10)
        c = dict(short_max_len=8, len_buckets=[8], depths=depths, token_budget=8 * rng.choice(depths + [12, 20]),
                 long_chunk=64, new_len=[rng.randint(1, 8) for _ in range(n)], prefix_len=[0] * n)
        assert strip(api.laps_plan_buckets(**c)) == plan_oracle.plan_buckets(**c), c


def test_planner_large_input_invariants():
    rng = random.Random(3)
    n = 20000
    new_len = [rng.choice([1, 7, 16, 17, 33, 64, 65, 900, 5000]) for _ in range(n)]
    got = api.laps_plan_buckets(64, [16, 32, 64], [1, 2, 4, 8, 16, 32, 64], 1024, 2048, new_len, [0] * n)
    seen = sorted(i for b in got["batches"] for i in b["req_ids"]) + sorted(l["req_id"] for l in got["longs"])
    assert sorted(seen) == list(range(n))
    for b in got["batches"]:
        assert b["depth"] * b["len_bucket"] <= 1024 and len(b["req_ids"]) <= b["depth"]
    for lg in got["longs"]:
        assert sum(lg["chunks"]) == new_len[lg["req_id"]]


@pytest.mark.parametrize("kw", [
    dict(len_buckets=[16, 16]), dict(len_buckets=[32, 16]), dict(depths=[2, 1]), dict(depths=[0, 1]),
    dict(token_budget=0), dict(long_chunk=0), dict(short_max_len=0), dict(short_max_len=65),
    dict(new_len=[0, 3]), dict(prefix_len=[-1, 0]), dict(len_buckets=[]), dict(depths=[]),
])
def test_planner_rejects_bad_arguments(kw):
    base = dict(short_max_len=64, len_buckets=[16, 32, 64], depths=[1, 2, 4], token_budget=128, long_chunk=2048,
                new_len=[5, 70], prefix_len=[0, 0])
    base.update(kw)
    with pytest.raises(api.LapsError) as e:
        api.laps_plan_buckets(**base)
    assert "error -1" in str(e.value)


def test_planner_empty_request_list():
    got = api.laps_plan_buckets(64, [16, 32, 64], [1, 2], 128, 2048, [], [])
    assert strip(got) == {"cls": [], "bucket": [], "batches": [], "longs": []}


def test_library_exports_every_declared_symbol(repo_root):
    header = open(os.path.join(repo_root, "include", "laps.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(laps_[a-z0-9_]+)\s*\(", header))
    assert len(declared) >= 35
    out = subprocess.run(["nm", "-D", "--defined-only", api.LIB_PATH], capture_output=True, text=True, check=True).stdout
    exported = {line.split()[-1] for line in out.splitlines() if " T " in line}
    missing = sorted(declared - exported)
    assert not missing, missing
    lib = api.lib()
    for name in declared:
        assert hasattr(lib, name)
    assert lib.laps_version().decode().startswith("laps-gfx950")


def test_null_handles_are_rejected_without_touching_the_gpu():
    """Entry points that take a context or a graph return LAPS_EINVAL (-1) on a NULL handle before any HIP call."""
    import ctypes as C
    lib = api.lib()
    assert lib.laps_ctx_set_pool_pages(None, C.c_int32(8)) == -1
    assert b"pool_pages" in lib.laps_last_error()
    assert lib.laps_prof_enable(None, C.c_int32(1)) == -1
    assert lib.laps_graph_replay(None, None) == -1
    assert lib.laps_graph_stage(None, C.c_int32(0), None, None, None, None, C.c_int32(0), None) == -1
    assert lib.laps_workspace_bytes(None, C.c_int32(8), C.c_int32(1)) == 0
    assert lib.laps_graph_device_bytes(None) == 0
    lib.laps_graph_destroy(None)
    lib.laps_ctx_destroy(None)
    assert lib.laps_plan_n_batches(None) == 0 and lib.laps_plan_n_long(None) == 0 and lib.laps_plan_n_requests(None) == 0
    assert not lib.laps_plan_batch_depth(None) and not lib.laps_plan_long_chunk_len(None)
    lib.laps_plan_free(None)


def test_planner_under_address_and_ub_sanitizers(repo_root, tmp_path):
    """Host code only: the planner and a random-input driver built with -fsanitize=address,undefined."""
    exe = str(tmp_path / "planner_san")
    src = [os.path.join(repo_root, "paper_2601_11589_amd", "csrc", "planner.cpp"),
           os.path.join(repo_root, "tests", "planner_sanitize_driver.cpp")]
    build = subprocess.run(["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                            "-o", exe] + src, capture_output=True, text=True)
    assert build.returncode == 0, build.stderr
    env = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert run.returncode == 0 and run.stdout.strip().endswith("OK"), (run.stdout[-500:], run.stderr[-2000:])


def test_host_objects_under_address_and_ub_sanitizers(repo_root, tmp_path):
    """Host code only: the AWD state machine, the pool controller, the latency-model helpers and the fixed-window rule, driven by seeded
    random event loops, built with -fsanitize=address,undefined."""
    exe = str(tmp_path / "host_san")
    csrc = os.path.join(repo_root, "paper_2601_11589_amd", "csrc")
    src = [os.path.join(csrc, f) for f in ("awd.cpp", "pool_ctrl.cpp", "latency_model.cpp", "window.cpp")] + \
          [os.path.join(repo_root, "tests", "host_objects_sanitize_driver.cpp")]
    build = subprocess.run(["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                            "-o", exe] + src, capture_output=True, text=True)
    assert build.returncode == 0, build.stderr
    env = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=180)
    assert run.returncode == 0 and run.stdout.strip().endswith("OK"), (run.stdout[-500:], run.stderr[-2000:])


def test_public_header_is_plain_c99(repo_root, tmp_path):
    """The boundary is a C ABI: the header must compile as C99 with no C++ or torch types in it, and a C program
    linked against the library must be able to call a host entry point."""
    src = tmp_path / "hdr.c"
    src.write_text(f'#include "{os.path.join(repo_root, "include", "laps.h")}"\n'
                   "#include <stdio.h>\n"
                   "int main(void) {\n"
                   "    int32_t lb[2] = {16, 32}, dp[3] = {1, 2, 4}, nl[3] = {5, 20, 100}, pl[3] = {0, 7, 0};\n"
                   "    laps_plan_params p = {32, 2, lb, 3, dp, 64, 64};\n"
                   "    laps_plan* plan = 0;\n"
                   "    if (laps_plan_buckets(&p, 3, nl, pl, &plan) != LAPS_OK) return 1;\n"
                   "    printf(\"%d %d %f\\n\", laps_plan_n_batches(plan), laps_plan_n_long(plan), laps_lm_boundary_prefill(1.0, 2.0, 10.0));\n"
                   "    laps_plan_free(plan);\n"
                   "    return 0;\n"
                   "}\n")
    exe = str(tmp_path / "hdr")
    libdir = os.path.join(repo_root, "paper_2601_11589_amd")
    build = subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", str(src), "-o", exe,
                            f"-L{libdir}", "-llaps", f"-Wl,-rpath,{libdir}"], capture_output=True, text=True)
    assert build.returncode == 0, build.stderr
    run = subprocess.run([exe], capture_output=True, text=True, timeout=60)
    assert run.returncode == 0 and run.stdout.split() == ["2", "1", "8.000000"], (run.stdout, run.stderr)
