"""AddressSanitizer / UndefinedBehaviorSanitizer builds of the host-side code: the launch
planner (which decides every offset and block count the kernels trust) and the CPU oracle.
Both run as standalone programs, so no GPU and no Python extension is involved."""
import os
import subprocess

import pytest

from paper_2307_02047_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan",
       "-g", "-O1", "-fno-omit-frame-pointer"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1")


@pytest.fixture(scope="module")
def plan_driver(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("san") / "plan_driver")
    csrc = os.path.join(ROOT, "paper_2307_02047_amd", "csrc")
    subprocess.run(["g++", "-std=c++17", "-Wall", "-Wextra", *SAN, "-I", os.path.join(ROOT, "include"), "-I", csrc,
                    os.path.join(ROOT, "tests", "sanitize", "plan_driver.cpp"), os.path.join(csrc, "came_plan.cpp"),
                    "-o", exe], check=True)
    return exe


def _plan(exe, tmp_path, descs, tile_rows=0, algo=0, group_elements=0, momentum=0, vector_rule=0, resident=0, tile_rows3=0):
    f = tmp_path / "descs.txt"
    f.write_text("".join(f"{r} {c} {nd} {dt}\n" for r, c, nd, dt in descs))
    res = subprocess.run([exe, str(f), str(tile_rows), str(algo), str(group_elements), str(momentum), str(vector_rule),
                          str(resident), str(tile_rows3)],
                         capture_output=True, text=True, env=ENV)
    assert res.returncode == 0, res.stderr[-2000:]
    return [int(x) for x in res.stdout.split()]


def _descs(w):
    return [(s[0], s[1], 2, w.grad_dtype) if len(s) == 2 else (s[0], 1, 1, w.grad_dtype) for s in w.shapes]


@pytest.mark.parametrize("make", W.CONFIGS, ids=lambda f: f.__name__)
def test_planner_on_the_named_workloads(plan_driver, tmp_path, make):
    w = make()
    for kw in ({}, {"momentum": 1}, {"tile_rows": 4 if w.n_params < 10 ** 9 else 64, "group_elements": 10 ** 7},
               {"tile_rows3": 4 if w.n_params < 10 ** 9 else 64}, {"tile_rows3": 1024, "tile_rows": 16 if w.n_params < 10 ** 9 else 64},
               {"resident": 2}, {"resident": 2, "tile_rows": 4 if w.n_params < 10 ** 9 else 64, "group_elements": 10 ** 7},
               {"resident": 2, "momentum": 1, "group_elements": 3 * 10 ** 7}):
        rc, state, scratch, items, fins, groups = _plan(plan_driver, tmp_path, _descs(w), **kw)
        assert rc == 0 and state >= (2 if kw.get("momentum") else 4) * w.n_params and items > 0 and groups >= 1


def test_planner_on_degenerate_descriptors(plan_driver, tmp_path):
    ok = [(1, 1, 2, 0), (1, 8, 2, 1), (8, 1, 2, 0), (2, 768, 2, 0), (5, 768, 2, 1), (33, 256, 2, 0), (1, 1280, 2, 1),
          (4, 4104, 2, 1), (1, 1, 1, 0), (16385, 1, 1, 1),
          (10 ** 9, 1, 1, 0)]
    for tr in (0, 4, 1024):
        for res in (0, 2):
            assert _plan(plan_driver, tmp_path, ok, tile_rows=tr, resident=res)[0] == 0
    huge = [(1 << 18, 1 << 20, 2, 1)]  # 2^38 elements: fine in tall tiles, too many 4-row tiles for 32-bit tables
    assert _plan(plan_driver, tmp_path, huge, tile_rows=1024)[0] == 0
    assert _plan(plan_driver, tmp_path, huge, tile_rows=4)[0] == -1
    # matrices at and around the on-chip limit of 512 tiles of 16 x 512
    edge = [(16 * 512, 512, 2, 0), (16 * 512 + 1, 512, 2, 1), (16, 512 * 512, 2, 0), (17, 512 * 512, 2, 1), (8192, 520, 2, 0),
            (40, 1032, 2, 1), (512,  1, 1, 0)]
    for kw in ({}, {"momentum": 1}, {"group_elements": 1}, {"algo": 1}):
        assert _plan(plan_driver, tmp_path, edge, resident=2, **kw)[0] == 0, kw
    bad = [[], [(0, 5, 2, 0)], [(5, 0, 2, 0)], [(-1, 5, 2, 0)], [(5, 5, 3, 0)], [(5, 5, 0, 0)], [(5, 2, 1, 0)],
           [(5, 5, 2, 7)], [((1 << 40) + 1, 1, 2, 0)], [(1 << 40, 1 << 40, 2, 0)], [(1 << 30, 1 << 30, 2, 0)],
           [((1 << 38) + 1, 1, 1, 0)], [(1 << 40, 64, 2, 0)] * 2]
    for descs in bad:
        assert _plan(plan_driver, tmp_path, descs)[0] == -1, descs
    # a plan whose tile table would not fit 32-bit indices: 2^40 rows of 4-row tiles
    assert _plan(plan_driver, tmp_path, [(1 << 40, 8, 2, 0)], tile_rows=4)[0] == -1
    for kw in ({"tile_rows": 3}, {"tile_rows": 2048}, {"algo": 2}, {"group_elements": -1}, {"momentum": 2}, {"vector_rule": 2},
               {"resident": 3}, {"resident": -1}, {"tile_rows3": 6}, {"tile_rows3": 1028}):
        assert _plan(plan_driver, tmp_path, [(8, 8, 2, 0)], **kw)[0] == -1, kw


def test_oracle_under_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_driver")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", *SAN, os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"),
                    os.path.join(ROOT, "oracle", "came_oracle.c"), "-o", exe, "-lm"], check=True)
    res = subprocess.run([exe], capture_output=True, text=True, env=ENV)
    assert res.returncode == 0, res.stderr[-2000:]
    assert res.stdout.startswith("checksum ") and "nan" not in res.stdout
