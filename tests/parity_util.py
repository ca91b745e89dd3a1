"""Runs the HIP library and the CPU oracle side by side on one seeded workload
and compares theta, M, r, c, R, C (v, s for vectors) element by element.

Error measure (stated bar: max relative error 1e-5 after 1 step, 1e-4 after
100 steps, binary32 GPU path against the binary64 oracle):
  * r, c, R, C, v, s are sums of non-negative terms, never near zero relative
    to their scale: plain elementwise |x - ref| / |ref|.
  * theta and M are signed and individual entries can cancel to ~0, where an
    elementwise relative error is meaningless; they use
    |x - ref| / (|ref| + RMS(ref over the tensor)).
  * theta_0 ~ 0.02 is ten times larger than the first step's move, so an error in the last
    line of Algorithm 2 (theta_t = theta_{t-1} - eta m_t / sqrt(S_t)) shows in theta diluted
    ten to twenty times.  After step 1 the move itself, theta_1 - theta_0, is therefore
    compared as well ("dtheta", same measure, same bar).  theta is stored in binary32, so the
    library's theta_1 cannot lie closer to the oracle's than half a binary32 spacing of theta_1
    (up to 3.7e-9 for |theta| < 0.125, which is 2e-6 of a CAME move at eta = 2e-4 and 4e-5 of
    an Algorithm-1 move at eta = 1e-3): that storage rounding is taken off the difference
    before it is divided, so that what is left is the error of the update itself.
The strict elementwise figure max |x - ref| / |ref| of theta and M is printed beside these
(not asserted: it is unbounded wherever an entry passes through zero).
"""
from __future__ import annotations

import numpy as np
import torch

import paper_2307_02047_amd as P
from oracle import came_oracle as O
from paper_2307_02047_amd import workloads as W


def rel_err_positive(x: np.ndarray, ref: np.ndarray) -> float:
    return float(np.max(np.abs(x - ref) / np.abs(ref)))


def rel_err_signed(x: np.ndarray, ref: np.ndarray) -> float:
    rms = float(np.sqrt(np.mean(ref * ref)))
    if rms == 0.0:
        return float(np.max(np.abs(x - ref)))
    return float(np.max(np.abs(x - ref) / (np.abs(ref) + rms)))


def rel_err_move(th: np.ndarray, th_ref: np.ndarray, th0: np.ndarray) -> float:
    """Error of the move theta - theta_0 against the oracle's, beyond the binary32 storage
    rounding of theta: max(0, |d - d_ref| - spacing32(theta)/2) / (|d_ref| + RMS(d_ref))."""
    d, dref = th - th0, th_ref - th0
    big = np.maximum(np.abs(th), np.abs(th_ref)).astype(np.float32)
    half_spacing = 0.5 * np.spacing(big).astype(np.float64)
    excess = np.maximum(np.abs(d - dref) - half_spacing, 0.0)
    rms = float(np.sqrt(np.mean(dref * dref)))
    if rms == 0.0:
        return float(np.max(excess))
    return float(np.max(excess / (np.abs(dref) + rms)))


def rel_err_strict(x: np.ndarray, ref: np.ndarray) -> float:
    """max |x - ref| / |ref| over the entries with ref != 0 (0 if there is none)."""
    nz = ref != 0.0
    if not nz.any():
        return 0.0
    return float(np.max(np.abs(x[nz] - ref[nz]) / np.abs(ref[nz])))


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu").to(torch.float32).numpy().astype(np.float64)


class SideBySide:
    """GPU library on every tensor of `shapes`; oracle on the tensors in `check`."""

    def __init__(self, w: W.Workload, indices=None, check=None, hyper=None, device="cuda:0", algo=0,
                 vector_confidence=True, **opts):
        self.w = w
        self.gen = W.Generator(w, device=device)
        self.idx = list(range(len(w.shapes))) if indices is None else list(indices)
        self.check = list(range(len(self.idx))) if check is None else list(check)  # positions in self.idx
        self.shapes = [w.shapes[i] for i in self.idx]
        self.hyper = hyper or P.CameHyper()
        self.algo = algo  # 0: Algorithm 2 (CAME), 1: Algorithm 1 (Adafactor with momentum)
        self.vector_confidence = vector_confidence  # False: 1-D parameters move by -eta M (option beyond the paper)
        self.opt = P.CameStep(self.shapes, [w.grad_dtype] * len(self.shapes), device=device, algo=algo,
                              vector_rule=P.VECTOR_ALGORITHM2 if vector_confidence else P.VECTOR_MOMENTUM_ONLY, **opts)
        self.theta = [self.gen.theta0(i) for i in self.idx]
        self.otl = O.TensorList([self.shapes[k] for k in self.check], [to_f64(self.theta[k]) for k in self.check])
        self.theta0 = [to_f64(self.theta[k]) for k in self.check]  # for the undiluted check of the first move
        self.strict = {}
        self.t = 0
        # a context manager factory under which the progress line of a check is printed; a long test
        # passes pytest's capsys.disabled so that the line appears when the check is made, not
        # when the test ends
        self.progress = None

    def step(self, nthreads: int = 0):
        self.t += 1
        grads = [self.gen.grad(i, self.t) for i in self.idx]
        self.opt.check_tensors(self.theta, grads)
        self.opt.step(self.theta, grads, self.hyper, self.w.lr, self.t)
        oh = O.Hyper(self.hyper.beta1, self.hyper.beta2, self.hyper.beta3, self.hyper.eps1, self.hyper.eps2,
                     self.hyper.clip_d, self.w.lr)
        og = [to_f64(grads[k]) for k in self.check]
        if self.algo == 0:
            self.otl.step(og, oh, nthreads=nthreads, weight_decay=self.hyper.weight_decay,
                          vector_confidence=self.vector_confidence)
        else:
            assert self.hyper.weight_decay == 0.0
            # Algorithm 1 per tensor; a vector is its n x 1 matrix (then v = r, c is a scalar)
            for pos, g in enumerate(og):
                st, th = self.otl.state[pos], self.otl.theta[pos]
                if isinstance(st, O.MatrixState):
                    O.adafactor_matrix_step(th, g, st.M, st.r, st.c, oh)
                else:
                    if not hasattr(st, "c1"):
                        st.c1 = np.zeros(1)
                    O.adafactor_matrix_step(th.reshape(-1, 1), g.reshape(-1, 1), st.M.reshape(-1, 1), st.v, st.c1, oh)
        torch.cuda.synchronize()

    def errors(self) -> dict:
        """Worst error per quantity over the checked tensors, plus where it occurs."""
        worst = {}

        def upd(name, e, k):
            if name not in worst or e > worst[name][0]:
                worst[name] = (e, self.idx[k], self.shapes[k])

        for pos, k in enumerate(self.check):
            sv = self.opt.state_view(k)
            st = self.otl.state[pos]
            th = to_f64(self.theta[k])
            assert np.all(np.isfinite(th)), f"non-finite theta in tensor {self.idx[k]} {self.shapes[k]}"
            upd("theta", rel_err_signed(th, self.otl.theta[pos]), k)
            if self.t == 1:  # the first move itself, not diluted by theta_0
                upd("dtheta", rel_err_move(th, self.otl.theta[pos], self.theta0[pos]), k)
            Mg = to_f64(sv["M"])
            upd("M", rel_err_signed(Mg, st.M), k)
            self.strict["theta"] = max(self.strict.get("theta", 0.0), rel_err_strict(th, self.otl.theta[pos]))
            self.strict["M"] = max(self.strict.get("M", 0.0), rel_err_strict(Mg, st.M))
            if len(self.shapes[k]) == 2:
                upd("r", rel_err_positive(to_f64(sv["r"]), st.r), k)
                upd("c", rel_err_positive(to_f64(sv["c"]), st.c), k)
                if self.algo == 0:
                    upd("R", rel_err_positive(to_f64(sv["R"]), st.R), k)
                    upd("C", rel_err_positive(to_f64(sv["C"]), st.C), k)
                else:  # Algorithm 1 has no confidence statistics: they must stay untouched
                    assert not sv["R"].any() and not sv["C"].any()
            else:
                upd("v", rel_err_positive(to_f64(sv["r"]), st.v), k)
                if self.algo == 0 and self.vector_confidence:
                    upd("s", rel_err_positive(to_f64(sv["R"]), st.s), k)
                else:
                    assert not sv["R"].any()
        return worst

    def assert_within(self, tol: float, label: str = ""):
        self.strict = {}
        errs = self.errors()
        bad = {k: v for k, v in errs.items() if not (v[0] <= tol)}
        summary = ", ".join(f"{k}={v[0]:.2e}" for k, v in errs.items())
        strict = ", ".join(f"{k}={v:.2e}" for k, v in self.strict.items())
        line = f"[parity] {self.w.name} {label} step {self.t}: {summary}; strict elementwise: {strict}"
        if self.progress is None:
            print(line, flush=True)
        else:
            with self.progress():
                print(line, flush=True)
        assert not bad, f"{self.w.name} step {self.t}: over tolerance {tol:g}: {bad}"
        return errs

    def close(self):
        self.opt.close()
