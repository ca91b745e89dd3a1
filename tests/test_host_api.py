"""Host-side behaviour of the C-ABI library that needs no GPU: it loads, exports
every symbol include/came.h declares, sizes and plans the state as Algorithm 2
requires, and turns every invalid argument into an error code."""
import ctypes
import os
import re

import pytest

import paper_2307_02047_amd as P
from paper_2307_02047_amd import binding as B
from paper_2307_02047_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "came.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(came_[a-z_0-9]+)\s*\(", header))
    assert declared == set(B.EXPORTS), declared ^ set(B.EXPORTS)
    lib = P.load_library()
    for name in declared:
        assert getattr(lib, name) is not None


def test_state_size_is_nm_plus_2n_plus_2m():
    """Section 3.1 / 3.3: O(n+m) factored statistics beside the momentum."""
    pad = lambda x: (x + 63) // 64 * 64
    for (n, m) in [(256, 512), (2, 768), (30522, 768), (7, 13)]:
        sb, _ = P.state_size([(n, m)], [0])
        assert sb == 4 * (pad(n * m) + 2 * pad(n) + 2 * pad(m))
        assert sb >= 4 * (n * m + 2 * (n + m))
    sb, _ = P.state_size([(4096,)], [1])
    assert sb == 4 * 3 * 4096


@pytest.mark.parametrize("make,params,mats,vecs", [
    (W.single_matrix, 131_584, 1, 1), (W.bert_base, 108_890_112, 75, 120),
    (W.gpt2_medium, 354_821_120, 98, 192), (W.bert_large, 334_090_240, 147, 240),
    (W.llama_7b, 6_738_415_616, 226, 65)])
def test_plan_of_the_named_workloads(make, params, mats, vecs):
    w = make()
    q = P.plan_query(w.shapes, [w.grad_dtype] * len(w.shapes), resident=P.RESIDENT_OFF)  # the streaming plan
    assert (q["elements"], q["matrices"], q["vectors"]) == (params, mats, vecs)
    tr, tc = q["tile_rows"], q["tile_cols"]
    def tiles(n, m):
        if m % tc == tc // 2:  # folded: swept as ceil(n/2) rows of 2m columns, all tiles full width
            return -(-(-(-n // 2)) // tr) * (2 * m // tc)
        return -(-n // tr) * -(-m // tc)
    want = sum(tiles(*s) for s in w.shapes if len(s) == 2) + vecs  # all vectors are short
    assert q["sweep_items"] == want
    assert q["finalize_items"] == sum(-(-s[0] // 256) + -(-s[1] // 64) for s in w.shapes if len(s) == 2)
    sb, wb = P.state_size(w.shapes, [w.grad_dtype] * len(w.shapes), resident=P.RESIDENT_OFF)
    assert sb >= 4 * sum((s[0] * s[1] + 2 * (s[0] + s[1])) if len(s) == 2 else 3 * s[0] for s in w.shapes)
    assert wb < 0.25 * sb or wb < (1 << 20)  # scratch stays a fraction of the state


def test_which_matrices_take_the_on_chip_path():
    """A matrix qualifies when its ceil(rows/16) * ceil(cols/512) tiles fit the 512 co-resident
    workgroups, its rows are 16-byte aligned and Algorithm 2 is selected; the traffic the plan
    reports prices those at 8 + grad_bytes + 2*momentum_bytes per element."""
    fits = lambda s: len(s) == 2 and s[1] % 8 == 0 and -(-s[0] // 16) * -(-s[1] // 512) <= 512
    for make in (W.single_matrix, W.bert_base, W.gpt2_medium, W.bert_large, W.llama_7b):
        w = make()
        dt = [w.grad_dtype] * len(w.shapes)
        assert P.plan_traffic(w.shapes, dt)["resident_matrices"] == 0  # off unless asked for
        t = P.plan_traffic(w.shapes, dt, resident=P.RESIDENT_ON)
        want = [s for s in w.shapes if fits(s)]
        assert t["resident_matrices"] == len(want)
        assert t["resident_elements"] == sum(s[0] * s[1] for s in want)
        gb = w.grad_bytes
        saved = (P.algorithmic_bytes(gb, 4, P.ALGO_CAME, 0) - P.algorithmic_bytes(gb, 4, P.ALGO_CAME, 4)) * t["resident_elements"]
        assert t["bytes_per_step_streaming"] - t["bytes_per_step"] == saved
        off = P.plan_traffic(w.shapes, dt, resident=P.RESIDENT_OFF)
        assert off["resident_matrices"] == 0 and off["bytes_per_step"] == off["bytes_per_step_streaming"] == t["bytes_per_step_streaming"]
        ada = P.plan_traffic(w.shapes, dt, algo=P.ALGO_ADAFACTOR, resident=P.RESIDENT_ON)
        assert ada["resident_matrices"] == 0  # Algorithm 1 streams
    assert P.algorithmic_bytes(4, 4, P.ALGO_CAME, 4) == 20.0 and P.algorithmic_bytes(2, 4, P.ALGO_CAME, 4) == 18.0
    # the largest that fits, and the first that does not
    on = dict(resident=P.RESIDENT_ON)
    assert P.plan_traffic([(16 * 512, 512)], [0], **on)["resident_matrices"] == 1
    assert P.plan_traffic([(16 * 512 + 1, 512)], [0], **on)["resident_matrices"] == 0
    assert P.plan_traffic([(64, 520)], [0], **on)["resident_matrices"] == 1 and P.plan_traffic([(64, 516)], [0], **on)["resident_matrices"] == 0


def test_long_vectors_are_chunked():
    """Up to 16384 entries: one work item; beyond: ceil(n / chunk) items with chunk a multiple of
    256, at least 16384, and at most 1024 chunks."""
    for n, items in [(16384, 1), (16385, 2), (50257, 4), (16384 * 1024, 1024), (16384 * 1024 + 1, 1009),
                     (10 ** 9, 1024)]:
        assert P.plan_query([(n,)], [0])["sweep_items"] == items, n


def test_tensors_with_more_than_two_dimensions_merge_their_leading_dimensions():
    assert B.matrix_view_of((6, 50, 520)) == (300, 520)
    assert B.matrix_view_of((2, 3, 4, 5)) == (24, 5)
    assert B.matrix_view_of((7, 9)) == (7, 9) and B.matrix_view_of((11,)) == (11,)
    assert P.state_size([(6, 50, 520)], [0]) == P.state_size([(300, 520)], [0])


def test_bf16_momentum_halves_the_momentum_bytes():
    shapes, dt = [(4096, 4096), (4096,)], [1, 1]
    f32, _ = P.state_size(shapes, dt)
    b16, _ = P.state_size(shapes, dt, momentum_dtype=P.MOMENTUM_BF16)
    assert f32 - b16 == 2 * (4096 * 4096 + 4096)
    with pytest.raises(P.CameError):
        P.state_size(shapes, dt, momentum_dtype=2)
    assert P.algorithmic_bytes(2, 4) == 26 and P.algorithmic_bytes(4, 4) == 32
    assert P.algorithmic_bytes(2, 2) == 20 and P.algorithmic_bytes(4, 2) == 26
    assert P.algorithmic_bytes(2, 4, P.ALGO_ADAFACTOR) == 22 and P.algorithmic_bytes(2, 2, P.ALGO_ADAFACTOR) == 18
    assert [P.algorithmic_bytes(2, 2, P.ALGO_CAME, k) for k in (1, 2, 3)] == [2, 4, 14]
    assert P.algorithmic_bytes(3, 4) == 0 and P.algorithmic_bytes(2, 8) == 0
    for g in (2, 4):
        assert [P.algorithmic_bytes(g, 4, P.ALGO_CAME, k) for k in range(4)] == [20 + 3 * g, g, g + 4, g + 16]


def test_groups_split_the_list():
    shapes = [(256, 512), (512,), (100, 1024), (1024,), (512, 512)]
    assert P.plan_query(shapes, [0] * 5)["groups"] == 1
    assert P.plan_query(shapes, [0] * 5, group_elements=150_000)["groups"] == 3
    assert P.plan_query(shapes, [0] * 5, group_elements=1)["groups"] == 5


def test_algorithmic_bytes():
    """Three-sweep design: g read three times, M read twice and written once,
    theta read and written once -> 20 + 3 sizeof(g) bytes per parameter."""
    assert P.algorithmic_bytes(2) == 26
    assert P.algorithmic_bytes(4) == 32
    for gb in (2, 4):
        assert sum(P.algorithmic_bytes(gb, which=k) for k in (1, 2, 3)) == P.algorithmic_bytes(gb)


def _raw(shapes_rows_cols_ndim_dtype):
    arr = (B._Desc * len(shapes_rows_cols_ndim_dtype))()
    for i, t in enumerate(shapes_rows_cols_ndim_dtype):
        arr[i] = B._Desc(*t)
    return arr


@pytest.mark.parametrize("desc", [(0, 4, 2, 0), (4, 0, 2, 0), (-1, 4, 2, 0), (4, 4, 3, 0), (4, 4, 0, 0),
                                  (4, 2, 1, 0), (4, 4, 2, 2), (4, 4, 2, -1)])
def test_bad_descriptors_are_rejected(desc):
    lib = P.load_library()
    sb, wb = ctypes.c_size_t(), ctypes.c_size_t()
    rc = lib.came_state_size(_raw([desc]), 1, None, ctypes.byref(sb), ctypes.byref(wb))
    assert rc == -1
    assert lib.came_strerror(rc) == b"invalid argument"


def test_bad_counts_options_and_null_pointers():
    lib = P.load_library()
    sb, wb = ctypes.c_size_t(), ctypes.c_size_t()
    good = _raw([(4, 8, 2, 0)])
    assert lib.came_state_size(good, 0, None, ctypes.byref(sb), ctypes.byref(wb)) == -1
    assert lib.came_state_size(None, 1, None, ctypes.byref(sb), ctypes.byref(wb)) == -1
    assert lib.came_state_size(good, 1, None, None, ctypes.byref(wb)) == -1
    for kw in (dict(tile_rows=3), dict(tile_rows=2), dict(tile_rows=2048), dict(tile_rows3=3), dict(tile_rows3=2048),
               dict(tile_rows3=-4), dict(algo=7), dict(group_elements=-5),
               dict(momentum_dtype=3), dict(vector_rule=2), dict(vector_rule=-1), dict(resident=3), dict(resident=-1),
               dict(resident_wait_us=-1)):
        o = B._options(**kw)
        assert lib.came_state_size(good, 1, ctypes.byref(o), ctypes.byref(sb), ctypes.byref(wb)) == -1, kw
    assert lib.came_state_size(good, 1, None, ctypes.byref(sb), ctypes.byref(wb)) == 0


def test_init_rejects_short_or_misaligned_blobs_before_touching_the_device():
    lib = P.load_library()
    good = _raw([(4, 8, 2, 0)])
    sb, wb = ctypes.c_size_t(), ctypes.c_size_t()
    assert lib.came_state_size(good, 1, None, ctypes.byref(sb), ctypes.byref(wb)) == 0
    ctx = ctypes.c_void_p()
    fake = 0x10000  # never dereferenced: every call below fails validation first
    assert lib.came_init_state(ctypes.byref(ctx), good, 1, None, fake, sb.value - 1, fake, wb.value, None) == -2
    assert lib.came_init_state(ctypes.byref(ctx), good, 1, None, fake, sb.value, fake, wb.value - 1, None) == -2
    assert lib.came_init_state(ctypes.byref(ctx), good, 1, None, fake + 8, sb.value, fake, wb.value, None) == -3
    assert lib.came_init_state(ctypes.byref(ctx), good, 1, None, None, sb.value, fake, wb.value, None) == -1
    assert lib.came_init_state(None, good, 1, None, fake, sb.value, fake, wb.value, None) == -1
    assert not ctx.value
    assert lib.came_step(None, None, None, None, 1e-3, 1, None) == -1
    v = B._View()
    assert lib.came_state_view_get(None, 0, ctypes.byref(v)) == -1
    lib.came_destroy(None)  # no-op
    assert lib.came_last_hip_error(None) == 0
    assert lib.came_strerror(12345) == b"unknown status"


def test_missing_library_fails_loudly(tmp_path):
    with pytest.raises(ImportError):
        P.load_library(str(tmp_path / "nope.so"))


def test_header_is_plain_c_and_the_library_links_from_c(tmp_path):
    """include/came.h compiles as strict C99 and a C program can call the host-only entry points."""
    import subprocess
    src = tmp_path / "use_came.c"
    src.write_text(r'''
#include <stdio.h>
#include "came.h"
int main(void)
{
    came_tensor_desc d[2] = {{4096, 4096, 2, CAME_GRAD_BF16}, {4096, 1, 1, CAME_GRAD_BF16}};
    came_options o = {0};
    size_t state = 0, scratch = 0;
    int rc = came_state_size(d, 2, &o, &state, &scratch);
    if (rc != CAME_OK) { printf("error %s\n", came_strerror(rc)); return 1; }
    o.momentum_dtype = CAME_MOMENTUM_BF16;
    size_t state16 = 0;
    rc = came_state_size(d, 2, &o, &state16, &scratch);
    if (rc != CAME_OK) return 2;
    d[0].ndim = 3;
    if (came_state_size(d, 2, NULL, &state, &scratch) != CAME_EINVAL) return 3;
    printf("%zu %zu %.0f %s\n", state, state16, came_algorithmic_bytes(2, 4, CAME_ALGO_CAME, 0), came_strerror(CAME_EALIGN));
    return 0;
}
''')
    exe = tmp_path / "use_came"
    libdir = os.path.dirname(B._LIB_PATH)
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
                    str(src), "-o", str(exe), "-L", libdir, "-lcame_hip", f"-Wl,-rpath,{libdir}",
                    "-Wl,-rpath,/opt/rocm/lib", "-Wl,--allow-shlib-undefined"], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    f32_state = 4 * (4096 * 4096 + 4 * 4096 + 3 * 4096)
    assert int(out[0]) == f32_state and int(out[1]) == f32_state - 2 * (4096 * 4096 + 4096)
    assert out[2] == "26"
