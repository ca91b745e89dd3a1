"""GPU parity of the bfloat16-momentum variant (CAME_MOMENTUM_BF16) against the CPU oracle
with the same storage rounding.

Two trajectories that each round M to bfloat16 cannot be compared entry by entry over many
steps: where M_t lands within rounding noise of a bfloat16 tie the binary32 kernel and the
binary64 oracle legitimately store neighbouring values (about one entry in 10^5 per step),
and from then on that entry follows a different, equally valid, path.  So:

  * step by step, both sides start every step from the SAME state -- the oracle's, loaded
    into the library's state blob like a checkpoint -- and one step is compared at the
    one-step bar 1e-5 (theta, r, c, R, C).  Every stored M entry must be a correct rounding
    of the oracle's unrounded M_t up to the binary32 noise of the kernel's own evaluation:
        |stored - M_t| <= spacing/2 + 2^-20 (|beta1 M_{t-1}| + |(1-beta1) u^_t|)
    (2^-20 = 16 binary32 roundings of relative size 2^-24: r, c and their rsqrt, the three
    products of u^, kappa, the momentum sum).  Where the sum cancels to a tiny M_t that
    noise exceeds the spacing, which is why the bound is not simply "one spacing".  The
    share of entries stored differently from the oracle is printed (about 5e-5).
  * free running for many steps: everything the rounding does not reach (r, c) at the
    100-step bar 1e-4, the row/column confidence sums at 1e-4 as well (single entries
    average out), and for theta, M and the unfactored s of vectors at least 99.8 % of the
    entries at 1e-4 (measured: 99.95 %).  The entries beyond that are bounded in size: two
    stored momenta that parted at a tie differ by one bfloat16 spacing (<= 2^-7 |M|) for as
    long as they keep rounding apart (0.9 spacings apart before rounding is 0 or 1 spacing
    after it; when M shrinks into a finer binade the gap it inherited just decays by beta1
    per step), so M may be off by two spacings of the largest |M| that entry has had, and
    theta by at most eta * spacing(M_t) / sqrt(S_t) per step, i.e. by no more than
    T * eta * 2^-7 * max |M / sqrt(S)| after T steps.  An entry that is wrong for any other
    reason breaks one of the two bounds.
"""
import numpy as np
import pytest
import torch

import paper_2307_02047_amd as P
from oracle import came_oracle as O
from paper_2307_02047_amd import workloads as W
from parity_util import rel_err_positive, to_f64

pytestmark = pytest.mark.gpu


def bf16_spacing(y):
    """Distance between neighbouring bfloat16 values at magnitude y (normal range)."""
    y = np.maximum(np.abs(y), 2.0 ** -126)
    return 2.0 ** (np.floor(np.log2(y)) - 7)


def signed_err(x, ref):
    rms = float(np.sqrt(np.mean(ref * ref)))
    return np.abs(x - ref) / (np.abs(ref) + rms)


def oracle_step(otl, grads64, oh, algo):
    """One oracle step with bfloat16 storage of M; returns the unrounded M_t of every tensor."""
    if algo == P.ALGO_CAME:
        otl.step(grads64, oh, nthreads=8)
        exact = [st.M.copy() for st in otl.state]
        for st in otl.state:
            O.store_bf16(st.M)
        return exact
    exact = []
    for pos, g in enumerate(grads64):  # Algorithm 1 per tensor; a vector is its n x 1 matrix
        st, th = otl.state[pos], otl.theta[pos]
        if isinstance(st, O.MatrixState):
            O.adafactor_matrix_step(th, g, st.M, st.r, st.c, oh)
        else:
            if not hasattr(st, "c1"):
                st.c1 = np.zeros(1)
            O.adafactor_matrix_step(th.reshape(-1, 1), g.reshape(-1, 1), st.M.reshape(-1, 1), st.v, st.c1, oh)
        exact.append(st.M.copy())
        O.store_bf16(st.M)
    return exact


def load_oracle_state(opt, theta, otl, algo):
    """The oracle's theta and state into the library's tensors (binary32; M is exactly a bfloat16)."""
    dev = theta[0].device
    f32 = lambda a: torch.from_numpy(np.asarray(a)).to(torch.float32).to(dev)
    for k, st in enumerate(otl.state):
        sv = opt.state_view(k)
        theta[k].copy_(f32(otl.theta[k]))
        M16 = torch.from_numpy(st.M).to(torch.float32).to(torch.bfloat16)
        assert np.array_equal(M16.to(torch.float64).numpy(), st.M), "oracle momentum is not a bfloat16"
        sv["M"].copy_(M16.to(dev))
        if isinstance(st, O.MatrixState):
            sv["r"].copy_(f32(st.r)); sv["c"].copy_(f32(st.c))
            if algo == P.ALGO_CAME:
                sv["R"].copy_(f32(st.R)); sv["C"].copy_(f32(st.C))
        else:
            sv["r"].copy_(f32(st.v))
            if algo == P.ALGO_CAME:
                sv["R"].copy_(f32(st.s))


SHAPES = [(300, 1024), (64, 520), (37, 77), (1, 9), (130, 1), (1000,), (5,), (20000,)]


@pytest.mark.parametrize("algo", [P.ALGO_CAME, P.ALGO_ADAFACTOR], ids=["came", "adafactor"])
@pytest.mark.parametrize("dtype", [W.GRAD_F32, W.GRAD_BF16], ids=["f32", "bf16"])
def test_each_step_from_the_oracles_state(dtype, algo):
    w = W.Workload("mb16", SHAPES, dtype, seed=61, steps=12, grad_kind="normal", scale_range=(1e-4, 1e-1))
    one_step_from_oracle_state(w, 12, algo=algo, tile_rows=32)


def one_step_from_oracle_state(w, steps, algo=P.ALGO_CAME, **opts):
    """Every step starts from the oracle's state; theta and the factored statistics at the
    one-step bar, every stored M entry a correct rounding of the oracle's unrounded M_t."""
    SHAPES, dtype = w.shapes, w.grad_dtype
    gen = W.Generator(w, device="cuda:0")
    n = len(SHAPES)
    opt = P.CameStep(SHAPES, [dtype] * n, algo=algo, momentum_dtype=P.MOMENTUM_BF16, **opts)
    theta = [gen.theta0(i) for i in range(n)]
    otl = O.TensorList(SHAPES, [to_f64(t) for t in theta])
    h, oh = P.CameHyper(), O.Hyper(lr=w.lr)
    try:
        for t in range(1, steps + 1):
            grads = [gen.grad(i, t) for i in range(n)]
            load_oracle_state(opt, theta, otl, algo)
            M_prev = [st.M.copy() for st in otl.state]
            opt.step(theta, grads, h, w.lr, t)
            exact = oracle_step(otl, [to_f64(g) for g in grads], oh, algo)
            torch.cuda.synchronize()
            worst, differ, total = {}, 0, 0
            for k, s in enumerate(SHAPES):
                sv, st = opt.state_view(k), otl.state[k]
                e = {"theta": float(signed_err(to_f64(theta[k]), otl.theta[k]).max())}
                if isinstance(st, O.MatrixState):
                    e["r"] = rel_err_positive(to_f64(sv["r"]), st.r)
                    e["c"] = rel_err_positive(to_f64(sv["c"]), st.c)
                    if algo == P.ALGO_CAME:
                        e["R"] = rel_err_positive(to_f64(sv["R"]), st.R)
                        e["C"] = rel_err_positive(to_f64(sv["C"]), st.C)
                else:
                    e["v"] = rel_err_positive(to_f64(sv["r"]), st.v)
                    if algo == P.ALGO_CAME:
                        e["s"] = rel_err_positive(to_f64(sv["R"]), st.s)
                for q, v in e.items():
                    worst[q] = max(worst.get(q, 0.0), v)
                    assert v <= 1e-5, f"step {t} tensor {s}: {q} error {v:.2e}"
                M = to_f64(sv["M"])
                noise = 2.0 ** -20 * (np.abs(h.beta1 * M_prev[k]) + np.abs(exact[k] - h.beta1 * M_prev[k]))
                allowed = 0.5 * bf16_spacing(np.maximum(np.abs(M), np.abs(exact[k]))) + noise
                bad = np.abs(M - exact[k]) > allowed
                assert not bad.any(), (f"step {t} tensor {s}: {bad.sum()} stored M entries are not a rounding "
                                       f"of the oracle's M_t; first at {np.argwhere(bad)[0]}")
                differ += int((M != st.M).sum())
                total += M.size
            worst["M stored differently"] = differ / total
            print(f"[bf16-M resync] algo {algo} dtype {dtype} step {t}: " +
                  ", ".join(f"{q}={v:.1e}" for q, v in worst.items()), flush=True)
    finally:
        opt.close()


def test_free_running_100_steps():
    w = W.bert_large()
    idx = [1, 3, 4, 8, 9, 10]   # 512x1024, 1024x1024 (x2), 4096x1024 and two vectors
    shapes = [w.shapes[i] for i in idx]
    gen = W.Generator(w, device="cuda:0")
    opt = P.CameStep(shapes, [w.grad_dtype] * len(idx), momentum_dtype=P.MOMENTUM_BF16)
    theta = [gen.theta0(i) for i in idx]
    otl = O.TensorList(shapes, [to_f64(t) for t in theta])
    h, oh = P.CameHyper(), O.Hyper(lr=w.lr)
    T = 100
    move = [0.0] * len(idx)  # per tensor: largest |M_t / sqrt(S_t)| the oracle saw (the size of a step, in units of eta)
    peak = [np.zeros(s) for s in shapes]  # per entry: largest |M_t| so far
    try:
        for t in range(1, T + 1):
            grads = [gen.grad(i, t) for i in idx]
            opt.step(theta, grads, h, w.lr, t)
            otl.step([to_f64(g) for g in grads], oh, nthreads=8, momentum_bf16=True)
            for k, st in enumerate(otl.state):
                if isinstance(st, O.MatrixState):
                    a = np.abs(st.M) / np.sqrt(st.R / st.R.sum())[:, None] / np.sqrt(st.C)[None, :]
                else:
                    a = np.abs(st.M) / np.sqrt(st.s)
                move[k] = max(move[k], float(a.max()))
                np.maximum(peak[k], np.abs(st.M), out=peak[k])
        torch.cuda.synchronize()
        for k, s in enumerate(shapes):
            sv, st = opt.state_view(k), otl.state[k]
            th = to_f64(theta[k])
            assert np.all(np.isfinite(th))
            e_th = signed_err(th, otl.theta[k])
            Mg = to_f64(sv["M"])
            e_M = signed_err(Mg, st.M)
            d_th = float(np.abs(th - otl.theta[k]).max())
            bound_th = T * w.lr * 2.0 ** -7 * move[k]
            d_M = np.abs(Mg - st.M)
            bound_M = 2.0 * bf16_spacing(1.01 * peak[k])
            line = (f"[bf16-M free] {s}: theta >1e-4: {(e_th > 1e-4).mean():.2e}, M >1e-4: {(e_M > 1e-4).mean():.2e}, "
                    f"max |dtheta| {d_th:.2e} (bound {bound_th:.2e}), max |dM| in spacings of the entry's peak |M| "
                    f"{float((d_M / bound_M).max()) * 2.0:.2f} (bound 2)")
            print(line, flush=True)
            few = max(2e-3, 4.0 / th.size)  # 0.2 % of the entries; a 1024-entry vector may have 4
            assert (e_th > 1e-4).mean() <= few and (e_M > 1e-4).mean() <= few, line
            assert d_th <= bound_th, line
            assert not (d_M > bound_M).any(), line
            if len(s) == 2:
                errs = {q: rel_err_positive(to_f64(sv[q]), getattr(st, q)) for q in "rcRC"}
                assert all(v <= 1e-4 for v in errs.values()), errs
            else:
                errs = {"v": rel_err_positive(to_f64(sv["r"]), st.v)}
                assert errs["v"] <= 1e-4
                e_s = np.abs(to_f64(sv["R"]) - st.s) / st.s
                errs["s >1e-4"] = float((e_s > 1e-4).mean())
                assert errs["s >1e-4"] <= few, errs
            print("    " + ", ".join(f"{q}={v:.1e}" for q, v in errs.items()), flush=True)
    finally:
        opt.close()


def test_state_is_smaller_and_views_are_bfloat16():
    shapes = [(300, 1024), (1000,)]
    a = P.CameStep(shapes, [0, 0])
    b = P.CameStep(shapes, [0, 0], momentum_dtype=P.MOMENTUM_BF16)
    try:
        assert a.state_bytes - b.state_bytes == 2 * (300 * 1024) + 2 * 1000 + (4096 - 4000) - (2048 - 2000)
        assert b.state_view(0)["M"].dtype == torch.bfloat16 and b.state_view(0)["M"].shape == (300, 1024)
        assert b.state_view(1)["M"].dtype == torch.bfloat16 and b.state_view(0)["r"].dtype == torch.float32
        assert not b.state_view(0)["M"].any() and not b.state_view(1)["M"].any()
    finally:
        a.close(); b.close()


def test_bf16_copy_together_with_bf16_momentum():
    shapes = [(100, 1024), (33, 24), (700,)]
    w = W.Workload("mb16c", shapes, W.GRAD_BF16, seed=62, steps=3, grad_kind="normal", scale_range=(1e-3, 1e-1))
    gen = W.Generator(w, device="cuda:0")
    a = P.CameStep(shapes, [1] * 3, tile_rows=16, momentum_dtype=P.MOMENTUM_BF16)
    b = P.CameStep(shapes, [1] * 3, tile_rows=16, momentum_dtype=P.MOMENTUM_BF16)
    ta, tb = [gen.theta0(i) for i in range(3)], [gen.theta0(i) for i in range(3)]
    copies = [torch.zeros(s, dtype=torch.bfloat16, device="cuda:0") for s in shapes]
    try:
        for t in range(1, 4):
            g = [gen.grad(i, t) for i in range(3)]
            a.step(ta, g, P.CameHyper(), 1e-3, t, bf16_copies=copies)
            b.step(tb, g, P.CameHyper(), 1e-3, t)
        torch.cuda.synchronize()
        for k in range(3):
            assert torch.equal(ta[k], tb[k]) and torch.equal(copies[k], ta[k].to(torch.bfloat16))
            assert torch.equal(a.state_view(k)["M"], b.state_view(k)["M"])
    finally:
        a.close(); b.close()


def test_llama_full_size_sampled_bf16_momentum():
    """The whole 6.7B-parameter list with a bfloat16 momentum in the launch configuration
    `bench.py --momentum-dtype bf16` times (all tensors, default plan, 512-row tiles); the oracle
    follows one tensor of every distinct shape.  Step 1 starts from the same (zero) state on
    both sides, so it is compared directly; step 2 restarts the sampled tensors from the
    oracle's state."""
    w = W.llama_7b()
    seen, check = set(), []
    for k, s in enumerate(w.shapes):
        if s not in seen and s != (32000, 4096):
            seen.add(s)
            check.append(k)
    check.append(len(w.shapes) - 1)  # LM head 32000 x 4096
    n = len(w.shapes)
    gen = W.Generator(w, device="cuda:0")
    opt = P.CameStep(w.shapes, [w.grad_dtype] * n, momentum_dtype=P.MOMENTUM_BF16)
    theta = [gen.theta0(i) for i in range(n)]
    shapes = [w.shapes[k] for k in check]
    otl = O.TensorList(shapes, [to_f64(theta[k]) for k in check])
    h, oh = P.CameHyper(), O.Hyper(lr=w.lr)

    class Sampled:  # the library's tensors the oracle follows, addressed by the oracle's positions
        def state_view(self, pos):
            return opt.state_view(check[pos])

    try:
        for t in (1, 2):
            grads = [gen.grad(i, t) for i in range(n)]
            if t > 1:
                load_oracle_state(Sampled(), [theta[k] for k in check], otl, P.ALGO_CAME)
            M_prev = [st.M.copy() for st in otl.state]
            opt.step(theta, grads, h, w.lr, t)
            exact = oracle_step(otl, [to_f64(grads[k]) for k in check], oh, P.ALGO_CAME)
            torch.cuda.synchronize()
            del grads
            for pos, k in enumerate(check):
                sv, st = opt.state_view(k), otl.state[pos]
                e = {"theta": float(signed_err(to_f64(theta[k]), otl.theta[pos]).max())}
                if isinstance(st, O.MatrixState):
                    for q in "rcRC":
                        e[q] = rel_err_positive(to_f64(sv[q]), getattr(st, q))
                else:
                    e["v"] = rel_err_positive(to_f64(sv["r"]), st.v)
                    e["s"] = rel_err_positive(to_f64(sv["R"]), st.s)
                assert all(v <= 1e-5 for v in e.values()), f"step {t} tensor {k} {w.shapes[k]}: {e}"
                M = to_f64(sv["M"])
                noise = 2.0 ** -20 * (np.abs(h.beta1 * M_prev[pos]) + np.abs(exact[pos] - h.beta1 * M_prev[pos]))
                allowed = 0.5 * bf16_spacing(np.maximum(np.abs(M), np.abs(exact[pos]))) + noise
                assert not (np.abs(M - exact[pos]) > allowed).any(), f"step {t} tensor {k}: stored M is not a rounding of M_t"
                print(f"[bf16-M llama] step {t} tensor {k} {w.shapes[k]}: " + ", ".join(f"{q}={v:.1e}" for q, v in e.items()) +
                      f", M stored differently {(M != st.M).mean():.1e}", flush=True)
    finally:
        opt.close()
