"""GPU parity of the on-chip path (came_options.resident): the matrices whose tiles all fit on
the chip take one launch in which g and M stay in LDS across the two whole-tensor
dependencies of Algorithm 2 (r_t, c_t before any u_t; RMS(u_t) of Eq. 1 before any u^_t).
Same bar as the streaming path: 1e-5 after one step, 1e-4 after 100, against the CPU oracle."""
import numpy as np
import pytest
import torch

import paper_2307_02047_amd as P
from paper_2307_02047_amd import workloads as W
from parity_util import SideBySide, rel_err_positive, rel_err_signed, to_f64
from test_gpu_parity import TOL_1, TOL_100, _run

pytestmark = pytest.mark.gpu

ON, OFF = P.RESIDENT_ON, P.RESIDENT_OFF

# rows 16-byte aligned (columns a multiple of 8): ragged row blocks (16-row tiles) and ragged
# column blocks (512-column tiles), one row, one tile, the most tiles a matrix may have (512),
# and, for the streaming path in the same launch group, a width that is no multiple of 8 and a
# matrix with one row block too many
ON_CHIP_SHAPES = [(256, 512), (1, 8), (5, 520), (17, 1000), (130, 24), (33, 1536), (300, 1032), (2, 768), (16, 512),
                  (8192, 512), (16, 8 * 512 + 8), (1030, 8)]
STREAMED_SHAPES = [(257, 1031), (8193, 512)]
VECTORS = [(1,), (77,), (512,), (5000,)]


def test_planner_sends_the_expected_matrices_on_chip():
    shapes = ON_CHIP_SHAPES + STREAMED_SHAPES + VECTORS
    t = P.plan_traffic(shapes, [0] * len(shapes), resident=ON)
    assert t["resident_matrices"] == len(ON_CHIP_SHAPES)


def test_single_matrix_and_bias_10_steps_on_chip():
    """The small configuration: its one matrix on chip, the bias rides in the same launch."""
    w = W.single_matrix()
    sbs = SideBySide(w, resident=ON)
    try:
        sbs.opt.profile_enable(True)
        for t in range(1, 11):
            sbs.step()
            sbs.assert_within(TOL_1 if t == 1 else TOL_100, "on chip")
        phases = sbs.opt.profile_read()
        assert phases["resident"][1] == 10, phases          # one on-chip launch per step ...
        assert all(phases[k][1] == 0 for k in phases if k != "resident"), phases  # ... and nothing else
        assert sbs.opt.device_status() == 0
    finally:
        sbs.close()


@pytest.mark.parametrize("momentum", [P.MOMENTUM_F32, P.MOMENTUM_BF16], ids=["m-f32", "m-bf16"])
@pytest.mark.parametrize("dtype", [W.GRAD_F32, W.GRAD_BF16], ids=["g-f32", "g-bf16"])
def test_odd_shapes_on_chip(dtype, momentum):
    """All four kernel variants on ragged tiles; streamed matrices and vectors in the same list."""
    shapes = ON_CHIP_SHAPES + STREAMED_SHAPES + VECTORS
    w = W.Workload("on-chip-odd", shapes, dtype, seed=79, steps=6, grad_kind="normal", scale_range=(1e-4, 1e-1),
                   zero_row_fraction=0.2)
    if momentum == P.MOMENTUM_F32:
        _run(w, 6, TOL_100, check_every=1, resident=ON)
        return
    # bfloat16 momentum: each step from the oracle's state (two free-running trajectories that
    # round M cannot be compared entry by entry), theta and the factored statistics at the one-step bar
    from test_gpu_bf16_momentum import one_step_from_oracle_state
    one_step_from_oracle_state(w, steps=4, resident=ON)


def test_streaming_and_on_chip_agree():
    """Same inputs through both paths: they differ by the order of the partial sums only."""
    shapes = ON_CHIP_SHAPES + VECTORS
    n = len(shapes)
    w = W.Workload("both-paths", shapes, W.GRAD_BF16, seed=83, steps=5, grad_kind="student_t3", scale_range=(1e-4, 1e-1))
    gen = W.Generator(w, device="cuda:0")
    runs = {}
    for mode in (ON, OFF):
        th = [gen.theta0(i) for i in range(n)]
        opt = P.CameStep(shapes, [w.grad_dtype] * n, resident=mode)
        for t in range(1, 6):
            opt.step(th, [gen.grad(i, t) for i in range(n)], P.CameHyper(), w.lr, t)
        torch.cuda.synchronize()
        runs[mode] = (th, [{k: (None if v is None else v.clone()) for k, v in opt.state_view(i).items()} for i in range(n)])
        assert opt.device_status() == 0
        opt.close()
    for i in range(n):
        assert rel_err_signed(to_f64(runs[ON][0][i]), to_f64(runs[OFF][0][i])) <= 2e-5, (i, shapes[i])
        for k in "MrcRC":
            a, b = runs[ON][1][i][k], runs[OFF][1][i][k]
            if a is None:
                continue
            err = rel_err_signed(to_f64(a), to_f64(b)) if k == "M" else rel_err_positive(to_f64(a), to_f64(b))
            assert err <= 2e-5, (i, shapes[i], k, err)
    # vectors take the same code either way
    for i in range(len(ON_CHIP_SHAPES), n):
        assert torch.equal(runs[ON][0][i], runs[OFF][0][i])


def test_bitwise_reproducible_on_chip():
    """No atomics on data and fixed summation orders: two runs give the same bits, whatever
    order the workgroups happen to reach their meetings in."""
    shapes = [(1024, 1024), (300, 1032), (768, 3072), (77,)]
    w = W.Workload("on-chip-repro", shapes, W.GRAD_F32, seed=85, steps=4, grad_kind="normal", scale_range=(1e-3, 1e-1))
    gen = W.Generator(w, device="cuda:0")
    outs = []
    for _ in range(2):
        th = [gen.theta0(i) for i in range(4)]
        opt = P.CameStep(shapes, [0] * 4, resident=ON)
        for t in range(1, 5):
            opt.step(th, [gen.grad(i, t) for i in range(4)], P.CameHyper(), 1e-3, t)
        torch.cuda.synchronize()
        outs.append((th, [{k: (None if v is None else v.clone()) for k, v in opt.state_view(i).items()} for i in range(4)]))
        opt.close()
    for i in range(4):
        assert torch.equal(outs[0][0][i], outs[1][0][i])
        for k in "MrcRC":
            if outs[0][1][i][k] is not None:
                assert torch.equal(outs[0][1][i][k], outs[1][1][i][k]), (i, k)


def test_constant_gradient_on_chip():
    """u^ -> M: the three binary64 sums behind sum U cancel to many digits (see the streaming
    counterpart); the on-chip path forms them per tile and adds them in its own order."""
    w = W.Workload("constant-grad-on-chip", [(200, 520), (96, 1024), (333,)], W.GRAD_F32, seed=81, steps=100,
                   grad_kind="normal", scale_range=(1e-3, 1e-1))
    sbs = SideBySide(w, resident=ON)
    fixed = {}
    real_grad = sbs.gen.grad
    sbs.gen.grad = lambda i, t: fixed.setdefault(i, real_grad(i, 1))
    try:
        for t in range(1, 101):
            sbs.step()
            if t in (1, 10, 30, 60, 100):
                sbs.assert_within(TOL_1 if t == 1 else TOL_100, "constant gradient, on chip")
    finally:
        sbs.close()


@pytest.mark.parametrize("make", [W.bert_base, W.gpt2_medium, W.bert_large], ids=["bert_base", "gpt2_medium", "bert_large"])
def test_one_layer_100_steps_on_chip(make):
    """One transformer layer of each list (every per-layer shape, its vectors included) for the
    stated 100 steps; the full lists run in test_gpu_parity.py with the default plan, which
    sends these same matrices on chip."""
    w = make()
    per_layer = {W.bert_base: 16, W.gpt2_medium: 12, W.bert_large: 16}[make]
    start = len(w.shapes) - per_layer  # the last layer
    idx = list(range(start, len(w.shapes)))
    assert P.plan_traffic([w.shapes[i] for i in idx], [w.grad_dtype] * len(idx), resident=ON)["resident_matrices"] == \
        sum(1 for i in idx if len(w.shapes[i]) == 2)
    sbs = SideBySide(w, indices=idx, resident=ON)
    try:
        for t in range(1, 101):
            sbs.step()
            if t == 1 or t % 25 == 0:
                sbs.assert_within(TOL_1 if t == 1 else TOL_100, "one layer, on chip")
        assert sbs.opt.device_status() == 0
    finally:
        sbs.close()


def test_bf16_copy_weight_decay_and_a_non_finite_entry_on_chip():
    """came_step_bf16_copy, the decoupled weight decay and IEEE propagation of a NaN gradient entry
    (it poisons its own matrix and nothing else) through the on-chip kernel."""
    shapes = [(300, 1032), (64, 2048), (130, 24), (77,)]
    n = len(shapes)
    w = W.Workload("on-chip-options", shapes, W.GRAD_F32, seed=87, steps=3, grad_kind="normal", scale_range=(1e-3, 1e-1))
    h = P.CameHyper(weight_decay=0.05)
    sbs = SideBySide(w, hyper=h, resident=ON)
    copies = [torch.zeros(s, dtype=torch.bfloat16, device="cuda:0") for s in shapes]
    real_step = sbs.opt.step
    sbs.opt.step = lambda th, g, hy, lr, t: real_step(th, g, hy, lr, t, bf16_copies=[copies[0], None, copies[2], copies[3]])
    try:
        for t in range(1, 4):
            sbs.step()
            sbs.assert_within(TOL_1 if t == 1 else TOL_100, "weight decay + bf16 copy, on chip")
        for i in (0, 2, 3):
            assert torch.equal(copies[i].view(torch.int16), sbs.theta[i].to(torch.bfloat16).view(torch.int16))
        assert not copies[1].any()
        # a NaN in tensor 1's gradient: tensor 1 turns non-finite, the others go on as if nothing happened
        clean = [t.clone() for t in sbs.theta]
        g = [sbs.gen.grad(i, 4) for i in range(n)]
        ref = P.CameStep(shapes, [0] * n, resident=ON)
        for i in range(n):
            for k, v in sbs.opt.state_view(i).items():
                if v is not None:
                    ref.state_view(i)[k].copy_(v)
        th_ref = [t.clone() for t in clean]
        ref.step(th_ref, g, h, w.lr, 4)
        g_bad = [x.clone() for x in g]
        g_bad[1][3, 5] = float("nan")
        real_step(sbs.theta, g_bad, h, w.lr, 4)
        torch.cuda.synchronize()
        assert not torch.isfinite(sbs.theta[1]).all()
        for i in (0, 2, 3):
            assert torch.equal(sbs.theta[i], th_ref[i])
        ref.close()
    finally:
        sbs.close()


def test_a_wait_that_runs_out_is_reported_and_nothing_hangs():
    """resident_wait_us = 1: the first workgroups to reach a meeting of a 512-tile matrix give up
    almost at once; the kernel must still end by itself, and the host must hear of it."""
    shapes = [(8192, 512), (4096, 1024)]
    w = W.Workload("on-chip-timeout", shapes, W.GRAD_BF16, seed=89, steps=1, grad_kind="normal", scale_range=(1e-3, 1e-1))
    gen = W.Generator(w, device="cuda:0")
    th = [gen.theta0(i) for i in range(2)]
    g = [gen.grad(i, 1) for i in range(2)]
    opt = P.CameStep(shapes, [1, 1], resident=ON, resident_wait_us=1)
    try:
        opt.step(th, g, P.CameHyper(), 1e-3, 1)
        assert opt.device_status() == P.ETIMEOUT
        with pytest.raises(P.CameError) as e:
            opt.step(th, g, P.CameHyper(), 1e-3, 2)
        assert e.value.status == P.ETIMEOUT
    finally:
        opt.close()
    # the same list with the default limit is fine, also right after the failed launch (its
    # counters were left clean: every workgroup still went through every meeting)
    opt = P.CameStep(shapes, [1, 1], resident=ON)
    try:
        for t in (1, 2):
            opt.step(th, g, P.CameHyper(), 1e-3, t)
        assert opt.device_status() == 0
    finally:
        opt.close()


def test_hip_graph_replay_on_chip():
    """The on-chip launch clears its own counters, so a captured step can be replayed: every
    replay must give exactly what the eager call gives."""
    shapes = [(256, 512), (512,), (300, 1032), (77,)]
    n = len(shapes)
    w = W.Workload("on-chip-graph", shapes, W.GRAD_F32, seed=91, steps=6, grad_kind="normal", scale_range=(1e-3, 1e-1))
    gen = W.Generator(w, device="cuda:0")
    h, lr = P.CameHyper(), 1e-3

    def fresh():
        th = [gen.theta0(i) for i in range(n)]
        gbuf = [torch.empty_like(gen.grad(i, 1)) for i in range(n)]  # fixed addresses, refilled per step
        return th, gbuf, P.CameStep(shapes, [0] * n, resident=ON)

    th_e, g_e, opt_e = fresh()
    for t in range(1, 7):
        for i in range(n):
            g_e[i].copy_(gen.grad(i, t))
        opt_e.step(th_e, g_e, h, lr, t)
    torch.cuda.synchronize()
    th_g, g_g, opt_g = fresh()
    try:
        for i in range(n):
            g_g[i].copy_(gen.grad(i, 1))
        opt_g.step(th_g, g_g, h, lr, 1)  # uploads the pointer table
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                opt_g.step(th_g, g_g, h, lr, 2)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        for t in range(2, 7):
            for i in range(n):
                g_g[i].copy_(gen.grad(i, t))
            graph.replay()
            torch.cuda.synchronize()
            _ = (th_g[0] * 2).sum().item()  # unrelated eager work between replays
        assert opt_g.device_status() == 0
        for a, b in zip(th_e, th_g):
            assert torch.equal(a, b)
        for i in range(n):
            for k in "MrcRC":
                if opt_e.state_view(i)[k] is not None:
                    assert torch.equal(opt_e.state_view(i)[k], opt_g.state_view(i)[k])
    finally:
        opt_e.close()
        opt_g.close()
