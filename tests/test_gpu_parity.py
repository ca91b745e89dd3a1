"""GPU parity: the HIP library (through its C ABI) against the CPU oracle on the
same seeded inputs.  Bar: max relative error 1e-5 after 1 step, 1e-4 after 100
steps (measure defined in parity_util.py)."""
import numpy as np
import pytest
import torch

import paper_2307_02047_amd as P
from paper_2307_02047_amd import workloads as W
from parity_util import SideBySide

pytestmark = pytest.mark.gpu

TOL_1, TOL_100 = 1e-5, 1e-4


def _run(w, steps, tol_end, check_every=None, progress=None, **kw):
    sbs = SideBySide(w, **kw)
    sbs.progress = progress
    try:
        for t in range(1, steps + 1):
            sbs.step()
            if t == 1:
                sbs.assert_within(TOL_1)
            elif t == steps or (check_every and t % check_every == 0):
                sbs.assert_within(tol_end)
    finally:
        sbs.close()


def test_single_matrix_and_bias_10_steps():
    """256x512 matrix + bias of 512, the small configuration, all 10 steps."""
    _run(W.single_matrix(), 10, TOL_100, check_every=1)


@pytest.mark.parametrize("tile_rows", [4, 20, 64, 512])
def test_single_matrix_tile_rows(tile_rows):
    """Same result whatever the row tiling (ragged last row block included)."""
    _run(W.single_matrix(), 3, TOL_100, check_every=1, tile_rows=tile_rows)


@pytest.mark.parametrize("tile_rows3", [4, 12, 100, 1024])
def test_update_sweep_tile_rows(tile_rows3):
    """The update sweep cuts the matrices into row blocks of its own (came_options.tile_rows3),
    independent of the other two sweeps' (here 20): same result whatever their height, ragged
    last block included, on aligned and unaligned widths."""
    shapes = [(256, 512), (333, 1032), (70, 515), (512,)]
    w = W.Workload("update-sweep-tiles", shapes, W.GRAD_BF16, seed=5, steps=3, grad_kind="normal",
                   scale_range=(1e-3, 1e-1), zero_row_fraction=0.1)
    _run(w, 3, TOL_100, check_every=1, tile_rows=20, tile_rows3=tile_rows3)
    # bit-identical to the default height: the per-element arithmetic does not depend on the tiling
    gen = W.Generator(w, device="cuda:0")
    out = []
    for tr3 in (0, tile_rows3):
        th = [gen.theta0(i) for i in range(len(shapes))]
        opt = P.CameStep(shapes, [w.grad_dtype] * len(shapes), tile_rows=20, tile_rows3=tr3)
        try:
            for t in (1, 2):
                opt.step(th, [gen.grad(i, t) for i in range(len(shapes))], P.CameHyper(), w.lr, t)
            torch.cuda.synchronize()
            out.append([x.clone() for x in th] + [opt.state_view(0)["M"].clone()])
        finally:
            opt.close()
    for a, b in zip(*out):
        assert torch.equal(a, b)


def _vocabulary_and_one_per_shape(w):
    """Tensor 0 (the vocabulary matrix: the tallest column reduction of the list) plus the first
    tensor of every other distinct shape, matrices and vectors."""
    seen, check = set(), []
    for k, s in enumerate(w.shapes):
        if s not in seen:
            seen.add(s)
            check.append(k)
    assert check[0] == 0
    return check


@pytest.mark.parametrize("make,follow", [(W.bert_base, "all"), (W.gpt2_medium, "shapes"), (W.bert_large, "shapes")],
                         ids=["bert_base", "gpt2_medium", "bert_large"])
def test_full_list_100_steps(make, follow, capsys):
    """The stated bar on the stated configurations: every tensor of the list in one grouped
    launch, 100 steps, 1e-5 after the first (incl. the first move theta_1 - theta_0 by itself)
    and 1e-4 at steps 25, 50, 75, 100.  The oracle follows every tensor of the BERT-base-shaped
    list; on the two larger lists (where one oracle step of the whole list takes seconds) it
    follows the vocabulary matrix and one tensor of every other distinct shape, while the
    library still updates all of them together."""
    w = make()
    _run(w, 100, TOL_100, check_every=25, check=None if follow == "all" else _vocabulary_and_one_per_shape(w),
         progress=capsys.disabled)  # these take minutes: each check reports when it is made


def test_llama_full_size_sampled():
    """The 6.7B-parameter list in the configuration bench.py times (all tensors,
    default plan); the oracle follows one tensor of every distinct shape."""
    w = W.llama_7b()
    seen, check = set(), []
    for k, s in enumerate(w.shapes):
        if s not in seen and s != (32000, 4096):
            seen.add(s)
            check.append(k)
    check.append(len(w.shapes) - 1)  # LM head 32000 x 4096 (last tensor, after all layers)
    _run(w, 2, TOL_1 * 2, check=check)


ODD_SHAPES = [(1, 1), (1, 8), (8, 1), (3, 5), (2, 768), (5, 768), (3, 256), (5, 520), (7, 1000), (130, 24), (33, 513),
              (257, 1031), (1030, 8), (4, 4104)]


NARROW_SHAPES = [(37, 768), (129, 256), (77, 8), (50, 1160), (1, 264), (2, 128), (3, 640), (261, 768), (1, 768), (2, 256),
                 (70, 1280), (64, 768)]


@pytest.mark.parametrize("momentum", [P.MOMENTUM_F32, P.MOMENTUM_BF16], ids=["m-f32", "m-bf16"])
@pytest.mark.parametrize("dtype", [W.GRAD_F32, W.GRAD_BF16], ids=["g-f32", "g-bf16"])
@pytest.mark.parametrize("algo", [P.ALGO_CAME, P.ALGO_ADAFACTOR], ids=["came", "adafactor"])
def test_last_column_block_of_at_most_256_columns(dtype, momentum, algo):
    """Matrices whose last column block is at most half a tile wide (768 = 512 + 256, 8, 264 = 256 + 8,
    1160 = 2 * 512 + 136 ...: the widths of BERT-base / GPT-2-small shaped layers among them), with odd
    and even row counts and one to several row blocks, through all kernel variants.  Those whose width
    is an odd multiple of 256 (256, 768, 1280) are swept by the update sweep as ceil(n/2) rows of 2m
    columns; an odd row count leaves the last of those rows half empty."""
    w = W.Workload("narrow-tiles", NARROW_SHAPES, dtype, seed=321, steps=5, grad_kind="normal",
                   scale_range=(1e-4, 1e-1), zero_row_fraction=0.2)
    if momentum == P.MOMENTUM_BF16:
        # the stored momentum is rounded: compared one step at a time from the oracle's state
        from test_gpu_bf16_momentum import one_step_from_oracle_state
        one_step_from_oracle_state(w, 4, algo=algo, tile_rows=12, tile_rows3=20)
    else:
        _run(w, 5, TOL_100, check_every=1, algo=algo, tile_rows=12, tile_rows3=20)


@pytest.mark.parametrize("dtype", [W.GRAD_F32, W.GRAD_BF16], ids=["f32", "bf16"])
def test_odd_shapes(dtype):
    """Ragged rows and columns, widths that are not a multiple of 8 (scalar-load
    path), single rows/columns, vectors of awkward lengths."""
    shapes = ODD_SHAPES + [(1,), (7,), (255,), (256,), (257,), (5000,)]
    w = W.Workload("odd-shapes", shapes, dtype, seed=77, steps=5, grad_kind="normal",
                   scale_range=(1e-4, 1e-1), zero_row_fraction=0.3)
    _run(w, 5, TOL_100, check_every=1, tile_rows=8)


@pytest.mark.parametrize("dtype", [W.GRAD_F32, W.GRAD_BF16], ids=["f32", "bf16"])
def test_adafactor_mode_matches_algorithm_1(dtype):
    """CAME_ALGO_ADAFACTOR against the oracle's Algorithm 1 (Adafactor with momentum):
    same r, c, M recursion, theta moves by -eta m_t, R and C stay zero."""
    shapes = [(256, 512), (512,), (300, 1032), (77,), (5, 13), (64, 2048), (1030, 8)]
    w = W.Workload("adafactor", shapes, dtype, seed=21, steps=10, grad_kind="normal", scale_range=(1e-4, 1e-1),
                   zero_row_fraction=0.05, lr=1e-3)
    _run(w, 10, TOL_100, check_every=1, algo=P.ALGO_ADAFACTOR, tile_rows=32)


def test_adafactor_and_came_share_momentum_and_second_moment():
    """Algorithm 1 is Algorithm 2 without the confidence lines: on the same gradients the two
    modes must produce the same M, r, c (they never read theta, R, C)."""
    w = W.Workload("shared", [(300, 1024), (1024,), (130, 24)], W.GRAD_BF16, seed=22, steps=5,
                   grad_kind="normal", scale_range=(1e-3, 1e-1))
    res = []
    for algo in (P.ALGO_CAME, P.ALGO_ADAFACTOR):
        gen = W.Generator(w, device="cuda:0")
        th = [gen.theta0(i) for i in range(3)]
        opt = P.CameStep(w.shapes, [w.grad_dtype] * 3, algo=algo, tile_rows=64)
        for t in range(1, 6):
            opt.step(th, [gen.grad(i, t) for i in range(3)], P.CameHyper(), 1e-3, t)
        torch.cuda.synchronize()
        res.append([opt.state_view(i)[k].clone() for i in range(3) for k in "Mrc" if opt.state_view(i)[k] is not None])
        opt.close()
    for a, b in zip(*res):
        a, b = a.double().cpu().numpy(), b.double().cpu().numpy()
        scale = np.sqrt(np.mean(b * b))
        assert np.max(np.abs(a - b) / (np.abs(b) + scale)) < 1e-6


@pytest.mark.parametrize("dtype", [W.GRAD_F32, W.GRAD_BF16], ids=["f32", "bf16"])
def test_long_vectors_take_the_two_pass_path(dtype):
    """1-D parameters longer than one workgroup's share are cut into chunks and updated in two
    passes; lengths straddle the switch-over (16384) and a chunk boundary."""
    shapes = [(16384,), (16385,), (50257,), (300001,), (64, 512), (5,)]
    w = W.Workload("long-vectors", shapes, dtype, seed=61, steps=4, grad_kind="normal", scale_range=(1e-4, 1e-1))
    _run(w, 4, TOL_100, check_every=1)


def test_transposed_matrix_swaps_row_and_column_statistics():
    """Algorithm 2 is symmetric in rows and columns: g^T, theta^T give theta^T, M^T,
    r <-> c, R <-> C.  On the GPU the row reduction (wave shuffles) and the column
    reduction (LDS + second stage) are different code, so this checks one against the other."""
    n, m = 300, 1048
    dev = "cuda:0"
    gen = torch.Generator(device=dev)
    gen.manual_seed(5)
    th = torch.randn((n, m), generator=gen, device=dev) * 0.02
    tht = th.t().contiguous()
    a = P.CameStep([(n, m)], [0], tile_rows=16)
    b = P.CameStep([(m, n)], [0], tile_rows=16)
    h = P.CameHyper()
    for t in range(1, 4):
        g = torch.randn((n, m), generator=gen, device=dev) * 0.01
        a.step([th], [g], h, 1e-3, t)
        b.step([tht], [g.t().contiguous()], h, 1e-3, t)
    torch.cuda.synchronize()
    va, vb = a.state_view(0), b.state_view(0)
    for x, y in [(th.t(), tht), (va["M"].t(), vb["M"]), (va["r"], vb["c"]), (va["c"], vb["r"]),
                 (va["R"], vb["C"]), (va["C"], vb["R"])]:
        x, y = x.double().cpu().numpy(), y.double().cpu().numpy()
        scale = np.sqrt(np.mean(y * y))
        assert np.max(np.abs(x - y) / (np.abs(y) + scale)) < 5e-6
    a.close(); b.close()


def test_bitwise_reproducible():
    """No data atomics anywhere: two runs from the same inputs agree bit for bit."""
    w = W.Workload("repro", [(700, 1536), (1536,), (64, 520)], W.GRAD_BF16, seed=9, steps=4,
                   grad_kind="normal", scale_range=(1e-3, 1e-1))
    outs = []
    for _ in range(2):
        gen = W.Generator(w, device="cuda:0")
        th = [gen.theta0(i) for i in range(3)]
        opt = P.CameStep(w.shapes, [w.grad_dtype] * 3, tile_rows=32)
        for t in range(1, 5):
            opt.step(th, [gen.grad(i, t) for i in range(3)], P.CameHyper(), 1e-3, t)
        torch.cuda.synchronize()
        outs.append([x.clone() for x in th] + [opt.state_view(0)[k].clone() for k in "MrcRC"])
        opt.close()
    for x, y in zip(*outs):
        assert torch.equal(x, y)


def test_state_checkpoint_round_trip():
    """State is exactly (M, r, c, R, C): 2 steps, copy the state out and into a fresh
    context, 2 more steps == 4 straight steps, bit for bit."""
    w = W.Workload("ckpt", [(300, 1024), (1024,)], W.GRAD_F32, seed=10, steps=4, grad_kind="normal",
                   scale_range=(1e-3, 1e-1))
    gen = W.Generator(w, device="cuda:0")
    h = P.CameHyper()
    th_a = [gen.theta0(i) for i in range(2)]
    a = P.CameStep(w.shapes, [0, 0])
    for t in range(1, 5):
        a.step(th_a, [gen.grad(i, t) for i in range(2)], h, 1e-3, t)
    th_b = [gen.theta0(i) for i in range(2)]
    b1 = P.CameStep(w.shapes, [0, 0])
    for t in range(1, 3):
        b1.step(th_b, [gen.grad(i, t) for i in range(2)], h, 1e-3, t)
    b2 = P.CameStep(w.shapes, [0, 0])
    torch.cuda.synchronize()
    for i in range(2):
        src, dst = b1.state_view(i), b2.state_view(i)
        for k in "MrcRC":
            if src[k] is not None:
                dst[k].copy_(src[k])
    for t in range(3, 5):
        b2.step(th_b, [gen.grad(i, t) for i in range(2)], h, 1e-3, t)
    torch.cuda.synchronize()
    for i in range(2):
        assert torch.equal(th_a[i], th_b[i])
        for k in "MrcRC":
            if a.state_view(i)[k] is not None:
                assert torch.equal(a.state_view(i)[k], b2.state_view(i)[k])
    a.close(); b1.close(); b2.close()


def test_update_sweep_direction_changes_nothing():
    """On short lists the update sweep walks its tiles forwards on a context's 1st, 3rd, ...
    call and backwards on the others.  Steps 2 and 3 taken by a fresh context (its 1st
    and 2nd call) must equal steps 2 and 3 of a context that also took step 1, bit for bit."""
    shapes = [(300, 1024), (1024,), (131, 768), (40, 520), (9, 256)]
    n = len(shapes)
    w = W.Workload("direction", shapes, W.GRAD_BF16, seed=14, steps=3, grad_kind="normal",
                   scale_range=(1e-3, 1e-1))
    gen = W.Generator(w, device="cuda:0")
    h = P.CameHyper()
    dt = [w.grad_dtype] * n
    th_a = [gen.theta0(i) for i in range(n)]
    a = P.CameStep(w.shapes, dt)
    for t in range(1, 4):
        a.step(th_a, [gen.grad(i, t) for i in range(n)], h, 1e-3, t)
    th_b = [gen.theta0(i) for i in range(n)]
    b1 = P.CameStep(w.shapes, dt)
    b1.step(th_b, [gen.grad(i, 1) for i in range(n)], h, 1e-3, 1)
    b2 = P.CameStep(w.shapes, dt)
    torch.cuda.synchronize()
    for i in range(n):
        src, dst = b1.state_view(i), b2.state_view(i)
        for k in "MrcRC":
            if src[k] is not None:
                dst[k].copy_(src[k])
    for t in range(2, 4):
        b2.step(th_b, [gen.grad(i, t) for i in range(n)], h, 1e-3, t)
    torch.cuda.synchronize()
    for i in range(n):
        assert torch.equal(th_a[i], th_b[i])
        for k in "MrcRC":
            if a.state_view(i)[k] is not None:
                assert torch.equal(a.state_view(i)[k], b2.state_view(i)[k])
    a.close(); b1.close(); b2.close()


def test_grouped_launch_equals_single_group():
    """Splitting the list into launch groups changes scheduling only."""
    # (a folded width, 768, and a ragged one, 520, among them: every tile shape in every group)
    shapes = [(256, 512), (512,), (100, 1024), (1024,), (512, 512), (131, 768), (768,), (40, 520)]
    n = len(shapes)
    w = W.Workload("groups", shapes, W.GRAD_BF16, seed=11, steps=3, grad_kind="normal", scale_range=(1e-3, 1e-1))
    res = []
    for ge in (0, 150_000):
        gen = W.Generator(w, device="cuda:0")
        th = [gen.theta0(i) for i in range(n)]
        opt = P.CameStep(w.shapes, [w.grad_dtype] * n, group_elements=ge, tile_rows=16)
        for t in range(1, 4):
            opt.step(th, [gen.grad(i, t) for i in range(n)], P.CameHyper(), 1e-3, t)
        torch.cuda.synchronize()
        res.append(th + [opt.state_view(0)["R"].clone(), opt.state_view(4)["C"].clone(), opt.state_view(5)["C"].clone(),
                         opt.state_view(5)["r"].clone()])
        opt.close()
    for x, y in zip(*res):
        assert torch.equal(x, y)


def test_pointer_table_follows_new_addresses():
    """Gradients handed over in fresh buffers every step (addresses change each call)."""
    w = W.Workload("ptrs", [(64, 512), (512,)], W.GRAD_F32, seed=12, steps=6, grad_kind="normal",
                   scale_range=(1e-2, 1e-1))
    _run(w, 6, TOL_100, check_every=1)


def test_placement_probe_changes_nothing():
    """came_probe_placement rewrites theta and M with their own bits: after some steps,
    probing must leave every parameter and every state array bit-identical, report a
    positive rate, and the following steps must match a run that never probed."""
    w = W.Workload("probe", [(300, 1024), (1024,), (64, 520), (33, 16)], W.GRAD_BF16, seed=31, steps=4,
                   grad_kind="normal", scale_range=(1e-3, 1e-1))
    runs = []
    for probe in (False, True):
        gen = W.Generator(w, device="cuda:0")
        th = [gen.theta0(i) for i in range(4)]
        opt = P.CameStep(w.shapes, [w.grad_dtype] * 4, tile_rows=32, place_against=th if probe else None,
                         placement_spacer_bytes=1 << 20)
        for t in range(1, 5):
            grads = [gen.grad(i, t) for i in range(4)]
            opt.step(th, grads, P.CameHyper(), 1e-3, t)
            if probe and t == 2:
                torch.cuda.synchronize()
                before = [x.clone() for x in th] + [opt.state_view(0)[k].clone() for k in "MrcRC"]
                assert opt.probe_placement(th, repeats=3) > 0
                assert opt.probe_placement(th, grads, repeats=2) > 0   # sweep 2's read streams as well
                after = th + [opt.state_view(0)[k] for k in "MrcRC"]
                for a, b in zip(before, after):
                    assert torch.equal(a, b)
        torch.cuda.synchronize()
        runs.append([x.clone() for x in th] + [opt.state_view(i)["M"].clone() for i in range(4)])
        if probe:
            assert len(opt.placement_log) >= 1 and all(g > 0 for _, g in opt.placement_log)
        opt.close()
    for a, b in zip(*runs):
        assert torch.equal(a, b)


def test_hip_graph_replay_matches_eager():
    """came_step only enqueues kernels (and no memset), so a step with unchanged tensor
    addresses can be captured into a HIP graph.  Every replay must give exactly what the
    eager call gives, with eager work and synchronisations between the replays."""
    w = W.Workload("graph", [(256, 512), (512,), (100, 1032), (77,)], W.GRAD_F32, seed=41, steps=6,
                   grad_kind="normal", scale_range=(1e-3, 1e-1))
    h, lr = P.CameHyper(), 1e-3
    gen = W.Generator(w, device="cuda:0")
    n = len(w.shapes)

    def fresh():
        th = [gen.theta0(i) for i in range(n)]
        gbuf = [torch.empty_like(gen.grad(i, 1)) for i in range(n)]  # fixed addresses, refilled per step
        return th, gbuf, P.CameStep(w.shapes, [w.grad_dtype] * n, tile_rows=32)

    # eager reference
    th_e, g_e, opt_e = fresh()
    for t in range(1, 7):
        for i in range(n):
            g_e[i].copy_(gen.grad(i, t))
        opt_e.step(th_e, g_e, h, lr, t)
    torch.cuda.synchronize()

    # graph: one eager step first (uploads the pointer table), then capture and replay
    th_g, g_g, opt_g = fresh()
    for i in range(n):
        g_g[i].copy_(gen.grad(i, 1))
    opt_g.step(th_g, g_g, h, lr, 1)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for i in range(n):
            g_g[i].copy_(gen.grad(i, 2))
        with torch.cuda.graph(graph, stream=side):
            opt_g.step(th_g, g_g, h, lr, 2)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    # capture does not execute: step 2 happens at the first replay
    for t in range(2, 7):
        for i in range(n):
            g_g[i].copy_(gen.grad(i, t))
        graph.replay()
        torch.cuda.synchronize()
        _ = (th_g[0] * 2).sum().item()  # unrelated eager work between replays
    for a, b in zip(th_e, th_g):
        assert torch.equal(a, b)
    for i in range(n):
        for k in "MrcRC":
            if opt_e.state_view(i)[k] is not None:
                assert torch.equal(opt_e.state_view(i)[k], opt_g.state_view(i)[k])
    opt_e.close(); opt_g.close()


def test_step_rejects_bad_arguments_on_device():
    """Every invalid came_step argument is an error code, nothing is enqueued, state unchanged."""
    import ctypes
    w = W.Workload("bad", [(64, 512), (512,)], W.GRAD_F32, seed=51, steps=1, grad_kind="normal", scale_range=None)
    gen = W.Generator(w, device="cuda:0")
    th = [gen.theta0(i) for i in range(2)]
    g = [gen.grad(i, 1) for i in range(2)]
    opt = P.CameStep(w.shapes, [0, 0])
    opt.step(th, g, P.CameHyper(), 1e-3, 1)
    torch.cuda.synchronize()
    snap = [x.clone() for x in th] + [opt.state_view(0)[k].clone() for k in "MrcRC"]
    bad_hypers = [dict(beta1=1.0), dict(beta2=-0.1), dict(beta3=1.5), dict(eps1=-1e-3), dict(eps2=float("nan")),
                  dict(clip_d=0.0), dict(clip_d=float("inf"))]
    for kw in bad_hypers:
        with pytest.raises(P.CameError) as e:
            opt.step(th, g, P.CameHyper(**kw), 1e-3, 2)
        assert e.value.status == -1, kw
    for lr, step in [(float("nan"), 2), (float("inf"), 2), (1e-3, 0), (1e-3, -5)]:
        with pytest.raises(P.CameError) as e:
            opt.step(th, g, P.CameHyper(), lr, step)
        assert e.value.status == -1
    with pytest.raises(P.CameError) as e:  # misaligned gradient pointer
        opt.step(th, [g[0].view(-1)[1:65 * 512 - 511].view(-1)[: 64 * 512 - 512], g[1]], P.CameHyper(), 1e-3, 2)
    assert e.value.status == -3
    with pytest.raises(P.CameError) as e:  # theta and grad are the same buffer
        opt.step(th, [th[0], g[1]], P.CameHyper(), 1e-3, 2)
    assert e.value.status == -1
    big = torch.zeros(64 * 512 + 512 + 64, dtype=torch.float32, device="cuda:0")
    overlapping = [big[: 64 * 512].view(64, 512), big[64 * 512 - 64: 64 * 512 - 64 + 512]]  # theta[1] starts inside theta[0]
    with pytest.raises(P.CameError) as e:
        opt.step(overlapping, g, P.CameHyper(), 1e-3, 2)
    assert e.value.status == -1
    with pytest.raises(P.CameError) as e:  # a gradient that lies inside a parameter
        opt.step(th, [g[0], th[0].view(-1)[1024:1536]], P.CameHyper(), 1e-3, 2)
    assert e.value.status == -1
    with pytest.raises(P.CameError) as e:  # a parameter inside the state blob
        opt.step([th[0], opt.state_view(0)["M"].view(-1)[:512]], g, P.CameHyper(), 1e-3, 2)
    assert e.value.status == -1
    shared = [g[0], g[0].view(-1)[:512]]   # two tensors reading one gradient buffer: allowed
    opt2 = P.CameStep(w.shapes, [0, 0])
    t2 = [x.clone() for x in th]
    opt2.step(t2, shared, P.CameHyper(), 1e-3, 1)
    opt2.close()
    torch.cuda.synchronize()
    for a, b in zip(snap, th + [opt.state_view(0)[k] for k in "MrcRC"]):
        assert torch.equal(a, b)
    opt.step(th, g, P.CameHyper(), 1e-3, 2)  # still usable afterwards
    torch.cuda.synchronize()
    assert all(torch.isfinite(x).all() for x in th)
    opt.close()


def test_mixed_gradient_dtypes_in_one_list():
    """A list may mix fp32 and bf16 gradients and aligned / unaligned widths: each kernel variant
    gets its own launch.  Tensors are independent, so the result must equal, bit for bit, what
    single-dtype lists give."""
    shapes = [(128, 1024), (1024,), (96, 520), (40, 13), (300, 512), (77,)]
    dtypes = [W.GRAD_BF16, W.GRAD_F32, W.GRAD_F32, W.GRAD_BF16, W.GRAD_F32, W.GRAD_BF16]
    gens = {d: W.Generator(W.Workload("mixed", shapes, d, seed=71, steps=3, grad_kind="normal",
                                      scale_range=(1e-3, 1e-1)), device="cuda:0") for d in (0, 1)}
    h = P.CameHyper()

    def run(idx):
        th = [gens[dtypes[i]].theta0(i) for i in idx]
        opt = P.CameStep([shapes[i] for i in idx], [dtypes[i] for i in idx], tile_rows=32)
        for t in range(1, 4):
            opt.step(th, [gens[dtypes[i]].grad(i, t) for i in idx], h, 1e-3, t)
        torch.cuda.synchronize()
        out = {i: [th[k].clone()] + [opt.state_view(k)[q].clone() for q in "MrcRC" if opt.state_view(k)[q] is not None]
               for k, i in enumerate(idx)}
        opt.close()
        return out

    mixed = run(list(range(6)))
    for d in (0, 1):
        single = run([i for i in range(6) if dtypes[i] == d])
        for i, arrs in single.items():
            for a, b in zip(arrs, mixed[i]):
                assert torch.equal(a, b), (i, d)


def test_constant_gradient_where_the_instability_sums_cancel():
    """With the same gradient every step u^ approaches M, so U = (u^ - M)^2 shrinks like
    beta1^(2t) and the three sums sweep 2 forms (kappa^2 sum u^2 - 2 kappa sum u M + sum M^2)
    cancel to many digits.  The fp64 accumulation must keep R, C and theta within the bar."""
    w = W.Workload("constant-grad", [(200, 520), (96, 1024), (333,)], W.GRAD_F32, seed=81, steps=100,
                   grad_kind="normal", scale_range=(1e-3, 1e-1))
    sbs = SideBySide(w, tile_rows=32)
    fixed = {}
    real_grad = sbs.gen.grad
    sbs.gen.grad = lambda i, t: fixed.setdefault(i, real_grad(i, 1))
    try:
        for t in range(1, 101):
            sbs.step()
            if t in (1, 10, 30, 60, 100):
                sbs.assert_within(TOL_1 if t == 1 else TOL_100, "constant gradient")
    finally:
        sbs.close()


@pytest.mark.parametrize("dtype", [W.GRAD_F32, W.GRAD_BF16], ids=["f32", "bf16"])
def test_bf16_parameter_copy_is_the_rounded_parameter(dtype):
    """came_step_bf16_copy: theta, M and all statistics are exactly what came_step gives, and the
    copy is theta_t rounded to nearest even (what torch's .to(bfloat16) does), bit for bit --
    matrices (aligned, ragged, unaligned widths), short and long vectors, and tensors whose
    copy is switched off."""
    shapes = [(256, 512), (512,), (300, 1032), (40, 13), (64, 2048), (20000,), (5, 520)]
    w = W.Workload("copy", shapes, dtype, seed=91, steps=3, grad_kind="normal", scale_range=(1e-3, 1e-1))
    n = len(shapes)
    gen = W.Generator(w, device="cuda:0")
    h = P.CameHyper()
    th_a = [gen.theta0(i) for i in range(n)]
    th_b = [gen.theta0(i) for i in range(n)]
    a = P.CameStep(shapes, [dtype] * n, tile_rows=32)
    b = P.CameStep(shapes, [dtype] * n, tile_rows=32)
    copies = [torch.full(s, float("nan"), dtype=torch.bfloat16, device="cuda:0") for s in shapes]
    skip = {3, 5}  # no copy wanted for these
    arg = [None if i in skip else copies[i] for i in range(n)]
    for t in range(1, 4):
        g = [gen.grad(i, t) for i in range(n)]
        a.step(th_a, g, h, 1e-2, t)
        b.step(th_b, g, h, 1e-2, t, bf16_copies=arg)
    torch.cuda.synchronize()
    for i in range(n):
        assert torch.equal(th_a[i], th_b[i])
        for k in "MrcRC":
            if a.state_view(i)[k] is not None:
                assert torch.equal(a.state_view(i)[k], b.state_view(i)[k])
        if i in skip:
            assert torch.isnan(copies[i].float()).all()  # untouched
        else:
            assert torch.equal(copies[i].view(torch.int16), th_b[i].to(torch.bfloat16).view(torch.int16)), i
    # special values go through the same rounding: NaN stays NaN, infinities and zeros keep their sign
    th = [torch.tensor([[float("inf"), -float("inf"), 0.0, -0.0, 1.0, 3.0e38, 1e-40, -1.5]], device="cuda:0")]
    g0 = [torch.zeros((1, 8), device="cuda:0")]
    c = P.CameStep([(1, 8)], [0])
    out = [torch.zeros((1, 8), dtype=torch.bfloat16, device="cuda:0")]
    c.step(th, g0, h, 1e-3, 1, bf16_copies=out)  # zero gradient: theta unchanged
    torch.cuda.synchronize()
    assert torch.equal(out[0].view(torch.int16), th[0].to(torch.bfloat16).view(torch.int16))
    a.close(); b.close(); c.close()


def test_more_than_two_dimensions_are_merged_leading_dimensions():
    """The binding hands a contiguous (a, b, c) parameter to the library as the (a*b, c) matrix
    it is in memory: same bits as stepping the reshaped tensor."""
    w = W.Workload("nd", [(6, 50, 520)], W.GRAD_F32, seed=95, steps=3, grad_kind="normal", scale_range=(1e-2, 1e-1))
    gen = W.Generator(w, device="cuda:0")
    th3, th2 = gen.theta0(0), gen.theta0(0).reshape(300, 520).clone()
    a, b = P.CameStep([(6, 50, 520)], [0], tile_rows=32), P.CameStep([(300, 520)], [0], tile_rows=32)
    for t in range(1, 4):
        g = gen.grad(0, t)
        a.check_tensors([th3], [g])
        a.step([th3], [g], P.CameHyper(), 1e-3, t)
        b.step([th2], [g.reshape(300, 520).clone()], P.CameHyper(), 1e-3, t)
    torch.cuda.synchronize()
    assert torch.equal(th3.reshape(300, 520), th2)
    va, vb = a.state_view(0), b.state_view(0)
    assert va["M"].shape == (6, 50, 520) and torch.equal(va["M"].reshape(300, 520), vb["M"])
    for k in "rcRC":
        assert torch.equal(va[k], vb[k])
    a.close(); b.close()


def test_decoupled_weight_decay():
    """theta_t = (1 - eta lambda) theta_{t-1} - eta M_t / sqrt(S_t) on matrices and vectors, against the
    oracle (decay, then Algorithm 2); lambda = 0 is bit-identical to a context stepped without the field."""
    w = W.Workload("wd", [(130, 520), (64, 1024), (33, 77), (700,), (20000,)], W.GRAD_BF16, seed=71, steps=20,
                   grad_kind="normal", scale_range=(1e-3, 1e-1))
    _run(w, 20, TOL_100, check_every=5, hyper=P.CameHyper(weight_decay=0.1), tile_rows=32)
    gen = W.Generator(w, device="cuda:0")
    a, b = P.CameStep(w.shapes, [1] * 5, tile_rows=32), P.CameStep(w.shapes, [1] * 5, tile_rows=32)
    ta, tb = [gen.theta0(i) for i in range(5)], [gen.theta0(i) for i in range(5)]
    for t in range(1, 4):
        g = [gen.grad(i, t) for i in range(5)]
        a.step(ta, g, P.CameHyper(), 1e-2, t)
        b.step(tb, g, P.CameHyper(weight_decay=0.5 if t == 3 else 0.0), 1e-2, t)
    torch.cuda.synchronize()
    for k in range(5):
        assert torch.equal(a.state_view(k)["M"], b.state_view(k)["M"])   # the decay does not enter the statistics
        assert not torch.equal(ta[k], tb[k])
    with pytest.raises(P.CameError) as e:
        a.step(ta, g, P.CameHyper(weight_decay=-0.1), 1e-2, 4)
    assert e.value.status == -1
    a.close(); b.close()


@pytest.mark.parametrize("dtype", [W.GRAD_F32, W.GRAD_BF16], ids=["f32", "bf16"])
def test_vectors_updated_by_momentum_only(dtype):
    """Option CAME_VECTOR_MOMENTUM_ONLY: 1-D parameters (short and long) move by -eta M_t and keep s = 0,
    matrices follow Algorithm 2 as before."""
    w = W.Workload("vmo", [(130, 520), (700,), (5,), (40000,), (64, 64)], dtype, seed=72, steps=12,
                   grad_kind="normal", scale_range=(1e-3, 1e-1))
    sbs = SideBySide(w, vector_confidence=False, tile_rows=32)
    try:
        for t in range(1, 13):
            sbs.step()
            sbs.assert_within(TOL_1 if t == 1 else TOL_100)
        for k, s in enumerate(w.shapes):
            if len(s) == 1:
                assert not sbs.opt.state_view(k)["R"].any()
            else:
                assert sbs.opt.state_view(k)["R"].all()
    finally:
        sbs.close()


def test_non_finite_gradient_stays_in_its_tensor():
    """A NaN or Inf in one tensor's gradient propagates through that tensor exactly as Algorithm 2's
    arithmetic does in the oracle (same entries non-finite, the finite ones within tolerance) and
    leaves every other tensor of the grouped launches bit-identical to a clean run."""
    from oracle import came_oracle as O
    from parity_util import to_f64
    shapes = [(70, 520), (64, 1024), (600,), (33, 40), (20000,)]
    w = W.Workload("nonfinite", shapes, W.GRAD_F32, seed=81, steps=2, grad_kind="normal", scale_range=(1e-2, 1e-1))
    gen = W.Generator(w, device="cuda:0")
    clean, dirty = P.CameStep(shapes, [0] * 5, tile_rows=32), P.CameStep(shapes, [0] * 5, tile_rows=32)
    tc, td = [gen.theta0(i) for i in range(5)], [gen.theta0(i) for i in range(5)]
    otl = O.TensorList(shapes, [to_f64(t) for t in td])
    oh = O.Hyper(lr=w.lr)
    for t in (1, 2):
        g = [gen.grad(i, t) for i in range(5)]
        gd = [x.clone() for x in g]
        if t == 2:
            gd[1][5, 700] = float("nan")
            gd[2][17] = float("inf")
        clean.step(tc, g, P.CameHyper(), w.lr, t)
        dirty.step(td, gd, P.CameHyper(), w.lr, t)
        otl.step([to_f64(x) for x in gd], oh)
    torch.cuda.synchronize()
    for k in (0, 3, 4):
        assert torch.equal(tc[k], td[k])
        for q, a in clean.state_view(k).items():
            assert a is None or torch.equal(a, dirty.state_view(k)[q])
    for k in (1, 2):
        sv, st = dirty.state_view(k), otl.state[k]
        pairs = [("theta", to_f64(td[k]), otl.theta[k]), ("M", to_f64(sv["M"]), st.M)]
        if k == 1:
            pairs += [(q, to_f64(sv[q]), getattr(st, q)) for q in "rcRC"]
        else:
            pairs += [("v", to_f64(sv["r"]), st.v), ("s", to_f64(sv["R"]), st.s)]
        for name, got, ref in pairs:
            assert np.array_equal(np.isfinite(got), np.isfinite(ref)), f"tensor {k} {name}: different entries are non-finite"
            fin = np.isfinite(ref)
            if fin.any():
                scale = np.abs(ref[fin]) + np.sqrt(np.mean(ref[fin] ** 2))
                assert np.max(np.abs(got[fin] - ref[fin]) / scale) <= 1e-5, f"tensor {k} {name}"
    assert not torch.isfinite(td[1]).any()            # one NaN reaches the whole matrix through the sum of r
    assert torch.isfinite(td[2]).sum().item() == 599  # the vector loses only the entry that was Inf
    clean.close(); dirty.close()
