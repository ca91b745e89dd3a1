"""Pins of the CPU oracle: checks of oracle/came_oracle.c against things the paper
and the mathematics fix, none of which is the oracle itself.

Every check is a plain function taking the loaded oracle library, so that
tests/test_oracle_pins.py can run it on the real oracle (must pass) and
tests/test_oracle_mutations.py can run it on deliberately broken copies of the
oracle source (at least one pin must fail for each planted mistake).

Citations are to the CAME paper: Algorithm 1 (Adafactor), Algorithm 2 (CAME),
Eq. 1 (RMS clipping), Eq. 2 (rank-1 factorisation), Section 3.1 / 3.3.
"""
import json
import os

import numpy as np

from oracle import came_oracle as O

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _rng(seed):
    return np.random.default_rng(seed)


# --------------------------------------------------------------------------- P1
def pin_step1_rank1_reconstruction(lib):
    """Algorithm 2 lines r_t, c_t, v_t with r_0 = c_0 = 0, and Eq. 2: when
    g^2 + eps1 is rank-1 the factored v_1 equals (1-beta2)(g^2+eps1) exactly.
    Observed through u_1 = g / sqrt(v_1): with a huge clip threshold nothing is
    clipped, so M_1 = (1-beta1) g / sqrt((1-beta2)(g^2+eps1)) entry by entry and
    RMS(u_1) follows in closed form."""
    rng = _rng(11)
    n, m = 5, 7
    a = rng.uniform(0.5, 2.0, n)
    b = rng.uniform(0.5, 2.0, m)
    sign = rng.choice([-1.0, 1.0], (n, m))
    # (i) |g| = a_i b_j, eps1 = 0  -> g^2 is rank-1
    g = sign * np.outer(a, b)
    h = O.Hyper(eps1=0.0, clip_d=1e30)
    st = O.MatrixState(n, m)
    th = np.zeros((n, m))
    rms_u, rms_uh = O.matrix_step(th, g, st, h, lib)
    v1 = (1 - h.beta2) * g * g
    np.testing.assert_allclose(st.M, (1 - h.beta1) * g / np.sqrt(v1), rtol=1e-13)
    np.testing.assert_allclose(rms_u, 1 / np.sqrt(1 - h.beta2), rtol=1e-13)
    np.testing.assert_allclose(rms_uh, rms_u, rtol=1e-13)
    # (ii) |g| constant and a LARGE eps1: g^2 + eps1 is a constant matrix (rank-1),
    # so eps1 shows in the result: u = g / sqrt((1-beta2)(g0^2+eps1))
    g0, eps1 = 0.3, 0.7
    g = sign * g0
    h = O.Hyper(eps1=eps1, clip_d=1e30)
    st = O.MatrixState(n, m)
    th = np.zeros((n, m))
    rms_u, _ = O.matrix_step(th, g, st, h, lib)
    u = g / np.sqrt((1 - h.beta2) * (g0 * g0 + eps1))
    np.testing.assert_allclose(st.M, (1 - h.beta1) * u, rtol=1e-13)
    np.testing.assert_allclose(rms_u, abs(u[0, 0]), rtol=1e-13)
    np.testing.assert_allclose(st.r, np.full(n, (1 - h.beta2) * m * (g0 * g0 + eps1)), rtol=1e-13)
    np.testing.assert_allclose(st.c, np.full(m, (1 - h.beta2) * n * (g0 * g0 + eps1)), rtol=1e-13)


# --------------------------------------------------------------------------- P2
def pin_rms_clip(lib):
    """Eq. 1: RMS(u_hat) = min(RMS(u), d); u_hat = u when RMS(u) <= d."""
    rng = _rng(12)
    n, m = 6, 4
    for d in (0.25, 1.0, 10.0, 1e6):
        st = O.MatrixState(n, m)
        th = rng.normal(size=(n, m))
        h = O.Hyper(clip_d=d)
        for _ in range(5):
            g = rng.normal(size=(n, m)) * 10 ** rng.uniform(-4, 0)
            rms_u, rms_uh = O.matrix_step(th, g, st, h, lib)
            np.testing.assert_allclose(rms_uh, min(rms_u, d), rtol=1e-12)
            assert rms_uh <= d * (1 + 1e-12)
    # vector path too
    st = O.VectorState(9)
    th = rng.normal(size=9)
    for d in (0.5, 1e6):
        h = O.Hyper(clip_d=d)
        rms_u, rms_uh = O.vector_step(th, rng.normal(size=9), st, h, lib)
        np.testing.assert_allclose(rms_uh, min(rms_u, d), rtol=1e-12)


# --------------------------------------------------------------------------- P3
def pin_dense_brute_force(lib):
    """Section 3.1 (O(n+m) instead of O(nm)) and Section 3.3 (factorising U_t):
    the factored recursion must reproduce the brute force that stores the full
    EMAs V_t and Ubar_t and factors them with Eq. 2 each step."""
    rng = _rng(13)
    for (n, m) in [(1, 1), (2, 3), (3, 2), (8, 5), (1, 6), (7, 1)]:
        h = O.Hyper(beta1=0.8, beta2=0.95, beta3=0.97, eps1=1e-12, eps2=1e-9, clip_d=1.5, lr=1e-2)
        th_f = rng.normal(size=(n, m))
        th_d = th_f.copy()
        sf, sd = O.MatrixState(n, m), O.DenseState(n, m)
        for t in range(25):
            g = rng.standard_t(3, size=(n, m)) * 10 ** rng.uniform(-3, 0)
            O.matrix_step(th_f, g, sf, h, lib)
            O.dense_step(th_d, g, sd, h, lib)
            for a, b in [(th_f, th_d), (sf.M, sd.M), (sf.r, sd.r), (sf.c, sd.c),
                         (sf.R, sd.R), (sf.C, sd.C)]:
                np.testing.assert_allclose(a, b, rtol=1e-11, atol=0)


# --------------------------------------------------------------------------- P4
def pin_state_size(lib):
    """Section 3.1 / 3.3: the factored statistics take O(n+m) memory: exactly
    2(n+m) numbers (r, c, R, C) beside the n*m momentum; 3n for a vector."""
    for (n, m) in [(256, 512), (2, 768), (30522, 768)]:
        st = O.MatrixState(n, m)
        assert st.factored_elems() == 2 * (n + m)
        assert st.elems() == n * m + 2 * (n + m)
    assert O.VectorState(4096).elems() == 3 * 4096
    tl = O.TensorList([(4, 6), (5,)], [np.zeros((4, 6)), np.zeros(5)])
    assert tl.state_elems() == 4 * 6 + 2 * (4 + 6) + 3 * 5
    # and the C code really touches nothing else: guard values around each array survive
    n, m = 3, 4
    pad = 8
    bufs = {k: np.full(sz + 2 * pad, 123.456) for k, sz in
            dict(theta=n * m, g=n * m, M=n * m, r=n, c=m, R=n, C=m).items()}
    view = {k: b[pad:-pad] for k, b in bufs.items()}
    for k in ("M", "r", "c", "R", "C"):
        view[k][:] = 0
    view["g"][:] = _rng(14).normal(size=n * m)
    st = O.MatrixState(n, m)
    st.M, st.r, st.c, st.R, st.C = (view["M"].reshape(n, m), view["r"], view["c"],
                                    view["R"], view["C"])
    O.matrix_step(view["theta"].reshape(n, m), view["g"].reshape(n, m), st, O.Hyper(), lib)
    for k, b in bufs.items():
        assert np.all(b[:pad] == 123.456) and np.all(b[-pad:] == 123.456), k


# --------------------------------------------------------------------------- P5
def pin_step1_closed_form(lib):
    """Algorithm 2 from zero state with |g| rank-1 and 1/sqrt(1-beta2) >= d:
    u = sign(g)/sqrt(1-beta2) (as eps1 -> 0), u_hat = d sign(g),
    M_1 = (1-beta1) d sign(g), U = beta1^2 d^2,
    R_1 = (1-beta3) m (beta1^2 d^2 + eps2), C_1 = (1-beta3) n (beta1^2 d^2 + eps2),
    theta_1 = theta_0 - eta (1-beta1) d sign(g) / sqrt((1-beta3)(beta1^2 d^2 + eps2)).
    Non-default, clearly visible eps2 so a dropped eps2 shows."""
    rng = _rng(15)
    n, m = 4, 9
    for hyp in (O.Hyper(), O.Hyper(beta1=0.7, beta2=0.9, beta3=0.6, eps1=0.0, eps2=0.5,
                                   clip_d=0.75, lr=3e-2)):
        a = rng.uniform(0.1, 3.0, n)
        b = rng.uniform(0.1, 3.0, m)
        sg = rng.choice([-1.0, 1.0], (n, m))
        g = sg * np.outer(a, b)
        th0 = rng.normal(size=(n, m))
        th = th0.copy()
        st = O.MatrixState(n, m)
        O.matrix_step(th, g, st, hyp, lib)
        b1, b3, d, e2 = hyp.beta1, hyp.beta3, hyp.clip_d, hyp.eps2
        np.testing.assert_allclose(st.M, (1 - b1) * d * sg, rtol=1e-12)
        np.testing.assert_allclose(st.R, np.full(n, (1 - b3) * m * (b1 * b1 * d * d + e2)), rtol=1e-12)
        np.testing.assert_allclose(st.C, np.full(m, (1 - b3) * n * (b1 * b1 * d * d + e2)), rtol=1e-12)
        dth = -hyp.lr * (1 - b1) * d * sg / np.sqrt((1 - b3) * (b1 * b1 * d * d + e2))
        np.testing.assert_allclose(th - th0, dth, rtol=1e-9)
    # defaults: the step is -11.111.. eta sign(g); R_1 = 8.1e-5 m; C_1 = 8.1e-5 n
    hyp = O.Hyper()
    g = rng.choice([-1.0, 1.0], (n, m)) * 0.01
    th = np.zeros((n, m))
    st = O.MatrixState(n, m)
    O.matrix_step(th, g, st, hyp, lib)
    np.testing.assert_allclose(th, -(100.0 / 9.0) * hyp.lr * np.sign(g), rtol=1e-9)
    np.testing.assert_allclose(st.R, 8.1e-5 * m, rtol=1e-9)
    np.testing.assert_allclose(st.C, 8.1e-5 * n, rtol=1e-9)
    # every vector with nonzero entries is rank-1: same closed form on the vector path
    gv = rng.choice([-1.0, 1.0], 13) * rng.uniform(0.5, 2, 13)
    thv = np.zeros(13)
    sv = O.VectorState(13)
    O.vector_step(thv, gv, sv, hyp, lib)
    np.testing.assert_allclose(thv, -(100.0 / 9.0) * hyp.lr * np.sign(gv), rtol=1e-9)
    np.testing.assert_allclose(sv.s, 8.1e-5, rtol=1e-9)
    np.testing.assert_allclose(sv.v, (1 - hyp.beta2) * gv * gv, rtol=1e-12)


def pin_zero_gradient(lib):
    """Algorithm 2 with g = 0 from zero state: u = 0, M = 0, U = 0, so
    r_1 = (1-beta2) m eps1, c_1 = (1-beta2) n eps1, R_1 = (1-beta3) m eps2,
    C_1 = (1-beta3) n eps2 and theta does not move: the eps terms sit INSIDE
    the row/column sums."""
    n, m = 3, 5
    h = O.Hyper()
    th0 = _rng(16).normal(size=(n, m))
    th = th0.copy()
    st = O.MatrixState(n, m)
    O.matrix_step(th, np.zeros((n, m)), st, h, lib)
    np.testing.assert_allclose(st.r, (1 - h.beta2) * m * h.eps1, rtol=1e-12)
    np.testing.assert_allclose(st.c, (1 - h.beta2) * n * h.eps1, rtol=1e-12)
    np.testing.assert_allclose(st.R, (1 - h.beta3) * m * h.eps2, rtol=1e-12)
    np.testing.assert_allclose(st.C, (1 - h.beta3) * n * h.eps2, rtol=1e-12)
    assert np.array_equal(th, th0) and not st.M.any()


# --------------------------------------------------------------------------- P6
def pin_vector_is_nx1_matrix(lib):
    """Our reading for 1-D parameters: Algorithm 2 on an n x 1 matrix (then
    c = sum r, v = r, S = R).  The vector routine must equal the matrix routine
    on n x 1, and (by symmetry of the algorithm in rows/columns) on 1 x n."""
    rng = _rng(17)
    n = 11
    h = O.Hyper(beta1=0.85, beta2=0.97, beta3=0.99, eps1=1e-8, eps2=1e-6, clip_d=0.8, lr=1e-2)
    th0 = rng.normal(size=n)
    tv, tc, tr = th0.copy(), th0.copy().reshape(n, 1), th0.copy().reshape(1, n)
    sv, sc, sr = O.VectorState(n), O.MatrixState(n, 1), O.MatrixState(1, n)
    for _ in range(12):
        g = rng.normal(size=n) * 10 ** rng.uniform(-3, 0)
        O.vector_step(tv, g, sv, h, lib)
        O.matrix_step(tc, g.reshape(n, 1).copy(), sc, h, lib)
        O.matrix_step(tr, g.reshape(1, n).copy(), sr, h, lib)
        np.testing.assert_allclose(tv, tc[:, 0], rtol=1e-12)
        np.testing.assert_allclose(tv, tr[0], rtol=1e-12)
        np.testing.assert_allclose(sv.M, sc.M[:, 0], rtol=1e-12)
        np.testing.assert_allclose(sv.v, sc.r, rtol=1e-12)
        np.testing.assert_allclose(sv.s, sc.R, rtol=1e-12)
        np.testing.assert_allclose(sv.v, sr.c, rtol=1e-12)
        np.testing.assert_allclose(sv.s, sr.C, rtol=1e-12)
        np.testing.assert_allclose(sc.c[0], sc.r.sum(), rtol=1e-12)


# --------------------------------------------------------------------------- P7
def pin_instability_identity(lib):
    """Algorithm 2, momentum and instability lines: u_hat - m_t =
    beta1 (u_hat - m_{t-1}), hence U_t = beta1^2 (u_hat_t - m_{t-1})^2.
    u_hat is recovered from the momentum alone, u_hat = (m_t - beta1 m_{t-1})/(1-beta1),
    and the R, C recursions are re-evaluated from it."""
    rng = _rng(18)
    n, m = 5, 6
    h = O.Hyper(beta1=0.8, beta3=0.9, eps2=1e-3, lr=1e-3)
    th = rng.normal(size=(n, m))
    st = O.MatrixState(n, m)
    for _ in range(8):
        M_old, R_old, C_old = st.M.copy(), st.R.copy(), st.C.copy()
        g = rng.normal(size=(n, m))
        O.matrix_step(th, g, st, h, lib)
        uh = (st.M - h.beta1 * M_old) / (1 - h.beta1)
        U = h.beta1 ** 2 * (uh - M_old) ** 2
        np.testing.assert_allclose(st.R, h.beta3 * R_old + (1 - h.beta3) * (U.sum(1) + m * h.eps2),
                                   rtol=1e-10)
        np.testing.assert_allclose(st.C, h.beta3 * C_old + (1 - h.beta3) * (U.sum(0) + n * h.eps2),
                                   rtol=1e-10)


# --------------------------------------------------------------------------- P8
def pin_sum_and_positivity(lib):
    """Row sums and column sums of one matrix have the same total, so
    sum r = sum c and sum R = sum C at every step; with eps > 0 all are > 0
    even for all-zero rows and columns."""
    rng = _rng(19)
    n, m = 7, 5
    h = O.Hyper()
    th = rng.normal(size=(n, m))
    st = O.MatrixState(n, m)
    for _ in range(10):
        g = rng.normal(size=(n, m))
        g[2, :] = 0.0
        g[:, 3] = 0.0
        O.matrix_step(th, g, st, h, lib)
        np.testing.assert_allclose(st.r.sum(), st.c.sum(), rtol=1e-12)
        np.testing.assert_allclose(st.R.sum(), st.C.sum(), rtol=1e-12)
        for x in (st.r, st.c, st.R, st.C):
            assert np.all(x > 0)
        assert np.all(np.isfinite(th)) and np.all(np.isfinite(st.M))
        assert not st.M[2, :].any() and not st.M[:, 3].any()


# --------------------------------------------------------------------------- P9
def pin_scale_covariance(lib):
    """g -> alpha g with eps1 -> alpha^2 eps1 scales r, c by alpha^2 and leaves
    u, hence M, R, C, theta, unchanged; for alpha a power of two, bit for bit."""
    rng = _rng(20)
    n, m = 6, 8
    alpha = 2.0 ** 7
    h1 = O.Hyper(eps1=1e-12)
    h2 = O.Hyper(eps1=1e-12 * alpha * alpha)
    th1 = rng.normal(size=(n, m))
    th2 = th1.copy()
    s1, s2 = O.MatrixState(n, m), O.MatrixState(n, m)
    for _ in range(6):
        g = rng.normal(size=(n, m))
        O.matrix_step(th1, g, s1, h1, lib)
        O.matrix_step(th2, g * alpha, s2, h2, lib)
        assert np.array_equal(s1.r * alpha * alpha, s2.r)
        assert np.array_equal(s1.c * alpha * alpha, s2.c)
        for a, b in [(s1.M, s2.M), (s1.R, s2.R), (s1.C, s2.C), (th1, th2)]:
            assert np.array_equal(a, b)


# -------------------------------------------------------------------------- P10
def pin_transpose_covariance(lib):
    """Algorithm 2 is symmetric in rows and columns: stepping g^T, theta^T gives
    theta^T, M^T with r <-> c and R <-> C."""
    rng = _rng(21)
    n, m = 4, 9
    h = O.Hyper(lr=1e-2)
    th = rng.normal(size=(n, m))
    tht = np.ascontiguousarray(th.T)
    s, stt = O.MatrixState(n, m), O.MatrixState(m, n)
    for _ in range(6):
        g = rng.normal(size=(n, m))
        O.matrix_step(th, g, s, h, lib)
        O.matrix_step(tht, np.ascontiguousarray(g.T), stt, h, lib)
        np.testing.assert_allclose(th.T, tht, rtol=1e-12)
        np.testing.assert_allclose(s.M.T, stt.M, rtol=1e-12)
        np.testing.assert_allclose(s.r, stt.c, rtol=1e-12)
        np.testing.assert_allclose(s.c, stt.r, rtol=1e-12)
        np.testing.assert_allclose(s.R, stt.C, rtol=1e-12)
        np.testing.assert_allclose(s.C, stt.R, rtol=1e-12)


# -------------------------------------------------------------------------- P11
def pin_permutation_equivariance(lib):
    """Permuting rows and columns of g and theta permutes the result."""
    rng = _rng(22)
    n, m = 6, 7
    pr, pc = rng.permutation(n), rng.permutation(m)
    h = O.Hyper(lr=1e-2)
    th = rng.normal(size=(n, m))
    thp = np.ascontiguousarray(th[pr][:, pc])
    s, sp = O.MatrixState(n, m), O.MatrixState(n, m)
    for _ in range(5):
        g = rng.normal(size=(n, m))
        O.matrix_step(th, g, s, h, lib)
        O.matrix_step(thp, np.ascontiguousarray(g[pr][:, pc]), sp, h, lib)
        np.testing.assert_allclose(th[pr][:, pc], thp, rtol=1e-11)
        np.testing.assert_allclose(s.r[pr], sp.r, rtol=1e-11)
        np.testing.assert_allclose(s.C[pc], sp.C, rtol=1e-11)


# -------------------------------------------------------------------------- P12
def pin_adafactor_subset(lib):
    """Algorithm 1 is Algorithm 2 without the confidence lines: on the same
    gradients M, r, c of both coincide (they never read theta, R or C), and
    Algorithm 1's parameter moves by exactly -eta m_t."""
    rng = _rng(23)
    n, m = 5, 4
    h = O.Hyper(lr=1e-2)
    th_c = rng.normal(size=(n, m))
    th_a = th_c.copy()
    s = O.MatrixState(n, m)
    Ma, ra, ca = np.zeros((n, m)), np.zeros(n), np.zeros(m)
    for _ in range(8):
        g = rng.normal(size=(n, m)) * 0.1
        before = th_a.copy()
        d1 = O.matrix_step(th_c, g, s, h, lib)
        d2 = O.adafactor_matrix_step(th_a, g, Ma, ra, ca, h, lib)
        np.testing.assert_allclose(s.M, Ma, rtol=1e-13)
        np.testing.assert_allclose(s.r, ra, rtol=1e-13)
        np.testing.assert_allclose(s.c, ca, rtol=1e-13)
        np.testing.assert_allclose(d1, d2, rtol=1e-13)
        np.testing.assert_allclose(th_a, before - h.lr * Ma, rtol=1e-13)


# -------------------------------------------------------------------------- P13
def pin_worked_example(lib):
    """Two steps on a 2 x 3 matrix against tests/golden/worked_2x3.json
    (60-digit scalar evaluation of Algorithm 2; r_1, c_1 checkable by hand)."""
    with open(os.path.join(GOLDEN, "worked_2x3.json")) as fh:
        gold = json.load(fh)
    h = O.Hyper(**gold["hyper"])
    th = np.array(gold["theta0"])
    st = O.MatrixState(2, 3)
    for k, stp in enumerate(gold["steps"]):
        rms_u, rms_uh = O.matrix_step(th, np.array(stp["g"]), st, h, lib)
        if k == 0:
            np.testing.assert_allclose(st.r, gold["hand"]["r1"], rtol=1e-12)
            np.testing.assert_allclose(st.c, gold["hand"]["c1"], rtol=1e-12)
            np.testing.assert_allclose(rms_uh, gold["hand"]["rms_uhat_1"], rtol=1e-12)
        np.testing.assert_allclose(rms_u, stp["rms_u"], rtol=1e-12)
        for name, got in (("r", st.r), ("c", st.c), ("R", st.R), ("C", st.C), ("M", st.M),
                          ("theta", th)):
            np.testing.assert_allclose(got, np.array(stp[name]), rtol=1e-12, err_msg=f"step {k+1} {name}")


def pin_list_driver(lib):
    """The tensor-list driver is only a loop over independent tensors
    (Algorithm 2 is stated per parameter): same results as per-tensor calls,
    for any thread count."""
    rng = _rng(24)
    shapes = [(4, 6), (5,), (3, 3), (7,), (1, 8)]
    th0 = [rng.normal(size=s) for s in shapes]
    h = O.Hyper(lr=1e-2)
    lists = [O.TensorList(shapes, [t.copy() for t in th0]) for _ in range(2)]
    single_th = [t.copy() for t in th0]
    single_st = [O.MatrixState(*s) if len(s) == 2 else O.VectorState(s[0]) for s in shapes]
    for _ in range(4):
        grads = [rng.normal(size=s) for s in shapes]
        lists[0].step(grads, h, nthreads=1, lib=lib)
        lists[1].step(grads, h, nthreads=3, lib=lib)
        for i, s in enumerate(shapes):
            if len(s) == 2:
                O.matrix_step(single_th[i], grads[i], single_st[i], h, lib)
            else:
                O.vector_step(single_th[i], grads[i], single_st[i], h, lib)
        for L in lists:
            for i, s in enumerate(shapes):
                assert np.array_equal(L.theta[i], single_th[i])
                assert np.array_equal(L.state[i].M, single_st[i].M)
                if len(s) == 2:
                    assert np.array_equal(L.state[i].R, single_st[i].R)
                    assert np.array_equal(L.state[i].c, single_st[i].c)
                else:
                    assert np.array_equal(L.state[i].s, single_st[i].s)
                    assert np.array_equal(L.state[i].v, single_st[i].v)


# --------------------------------------------------------------------------- bfloat16 momentum storage
def _torch_bf16(x64):
    """float64 -> binary32 -> bfloat16 -> float64 by torch's CPU conversion (a library
    routine independent of the oracle)."""
    import torch
    return torch.from_numpy(np.asarray(x64, dtype=np.float64)).to(torch.float32).to(torch.bfloat16) \
        .to(torch.float64).numpy()


def pin_bf16_rounding_by_hand(lib):
    """bfloat16 format: 8 significant bits, ties to the even significand, subnormal
    spacing 2^-133, overflow to infinity at 2^128.  Cases worked out by hand."""
    r = lambda x: O.round_bf16(x, lib)
    assert r(1.0) == 1.0 and r(-2.5) == -2.5 and r(0.0) == 0.0
    assert r(1.0 + 2.0 ** -8) == 1.0                       # tie: 1.0000000|1 -> even below
    assert r(1.0 + 3.0 * 2.0 ** -8) == 1.0 + 2.0 ** -6     # tie: 1.0000001|1 -> even above
    assert r(1.0 + 2.0 ** -8 + 2.0 ** -20) == 1.0 + 2.0 ** -7   # just above the tie
    assert r(-(1.0 + 2.0 ** -8 - 2.0 ** -20)) == -1.0           # just below the tie
    assert r(3.0 * 2.0 ** -10 + 2.0 ** -17) == 3.0 * 2.0 ** -10  # a quarter step: stays
    assert r(0.5 * 2.0 ** -133) == 0.0                     # tie between 0 and the smallest subnormal
    assert r(1.5 * 2.0 ** -133) == 2.0 ** -132             # tie between 1 and 2 steps -> even
    assert r(0.75 * 2.0 ** -133) == 2.0 ** -133
    assert r((2.0 - 2.0 ** -7) * 2.0 ** 127) == (2.0 - 2.0 ** -7) * 2.0 ** 127   # largest bfloat16
    assert r((2.0 - 2.0 ** -8) * 2.0 ** 127) == np.inf     # tie between it and 2^128 -> even = 2^128 = inf
    assert r(-3.4e38) == -np.inf
    assert np.isnan(r(np.nan)) and r(np.inf) == np.inf
    # a double that is not a binary32: goes through binary32 first.  1 + 2^-8 + 2^-40 rounds to
    # the binary32 1 + 2^-8 (a tie for bfloat16 -> 1.0), although it lies above the tie itself.
    assert r(1.0 + 2.0 ** -8 + 2.0 ** -40) == 1.0


def pin_bf16_rounding_matches_library(lib):
    """Same rounding as torch's float32 -> bfloat16 conversion on random bit patterns of
    every exponent, on exact ties, on subnormals and around the overflow threshold."""
    rng = _rng(31)
    bits = rng.integers(0, 2 ** 32, size=200000, dtype=np.uint64).astype(np.uint32)
    ties = (rng.integers(0, 2 ** 16, size=20000, dtype=np.uint64).astype(np.uint32) << np.uint32(16)) | np.uint32(0x8000)
    near = ties + rng.integers(-1, 2, size=ties.size).astype(np.int64).astype(np.uint32)
    sub = rng.integers(0, 2 ** 23, size=20000, dtype=np.uint64).astype(np.uint32)      # binary32 subnormals
    top = np.uint32(0x7f7f0000) + rng.integers(0, 2 ** 16, size=2000, dtype=np.uint64).astype(np.uint32)
    allbits = np.concatenate([bits, ties, near, sub, sub | np.uint32(0x80000000), top])
    x32 = allbits.view(np.float32)
    x = x32[np.isfinite(x32)].astype(np.float64)
    got = x.copy()
    O.store_bf16(got, lib)
    want = _torch_bf16(x)
    assert np.array_equal(got, want)
    assert np.array_equal(np.signbit(got), np.signbit(want))
    # doubles between binary32 values
    y = rng.normal(size=50000) * np.exp(rng.uniform(-80, 80, size=50000))
    got = y.copy()
    O.store_bf16(got, lib)
    assert np.array_equal(got, _torch_bf16(y))


def pin_bf16_momentum_mode(lib):
    """The stored momentum is rounded AFTER the step: theta, r, c, R, C of a step are those of
    Algorithm 2 run from the stored m_{t-1}; only the m handed to the next step is rounded.
    Checked against the plain list driver with torch doing the rounding between steps."""
    rng = _rng(32)
    shapes = [(5, 7), (9,), (3, 4)]
    th0 = [rng.normal(size=s) * 0.1 for s in shapes]
    h = O.Hyper(lr=1e-2)
    A = O.TensorList(shapes, [t.copy() for t in th0])
    B = O.TensorList(shapes, [t.copy() for t in th0])
    for step in range(4):
        grads = [rng.normal(size=s) for s in shapes]
        A.step(grads, h, lib=lib, momentum_bf16=True)
        B.step(grads, h, lib=lib)
        for i, s in enumerate(shapes):
            assert np.array_equal(A.theta[i], B.theta[i]), f"step {step}: theta must come from the unrounded m_t"
            B.state[i].M[...] = _torch_bf16(B.state[i].M)
            assert np.array_equal(A.state[i].M, B.state[i].M)
            if len(s) == 2:
                for k in "rcRC":
                    assert np.array_equal(getattr(A.state[i], k), getattr(B.state[i], k))
            else:
                assert np.array_equal(A.state[i].v, B.state[i].v) and np.array_equal(A.state[i].s, B.state[i].s)
    # and the rounding does change something (the mode is not a no-op)
    C = O.TensorList(shapes, [t.copy() for t in th0])
    rng2 = _rng(32)
    [rng2.normal(size=s) for s in shapes]
    g = [rng2.normal(size=s) for s in shapes]
    C.step(g, h, lib=lib)
    assert not np.array_equal(C.state[0].M, _torch_bf16(C.state[0].M))


# --------------------------------------------------------------------------- options beyond the paper
def pin_weight_decay(lib):
    """Decoupled decay: with a zero gradient nothing but the decay moves theta (u = 0, so
    m = 0), hence theta_t = theta_0 (1 - eta lambda)^t exactly; lambda = 0 changes nothing;
    and the decay acts before the update: one step equals a plain step from the shrunk theta."""
    rng = _rng(41)
    shapes = [(4, 5), (6,)]
    th0 = [rng.normal(size=s) for s in shapes]
    h = O.Hyper(lr=1e-2)
    A = O.TensorList(shapes, [t.copy() for t in th0])
    for _ in range(5):
        A.step([np.zeros(s) for s in shapes], h, lib=lib, weight_decay=0.3)
    for t, t0 in zip(A.theta, th0):
        np.testing.assert_allclose(t, t0 * (1 - 1e-2 * 0.3) ** 5, rtol=1e-14)
    g = [rng.normal(size=s) for s in shapes]
    B = O.TensorList(shapes, [t.copy() for t in th0])
    C = O.TensorList(shapes, [t.copy() for t in th0])
    B.step(g, h, lib=lib, weight_decay=0.0)
    C.step(g, h, lib=lib)
    D = O.TensorList(shapes, [t.copy() for t in th0])
    E = O.TensorList(shapes, [t * (1 - 1e-2 * 0.3) for t in th0])
    D.step(g, h, lib=lib, weight_decay=0.3)
    E.step(g, h, lib=lib)
    for i in range(2):
        assert np.array_equal(B.theta[i], C.theta[i])
        np.testing.assert_allclose(D.theta[i], E.theta[i], rtol=1e-15)
        assert np.array_equal(D.state[i].M, E.state[i].M)
        assert not np.array_equal(D.theta[i], C.theta[i])


def pin_vectors_without_confidence(lib):
    """Option: 1-D parameters move by -eta m_t (Algorithm 1's last line) while matrices keep
    Algorithm 2.  The vector's m and v are the same as with confidence (those lines do not
    involve S), its s stays zero, theta_t - theta_{t-1} = -eta m_t; the matrices are untouched
    by the option."""
    rng = _rng(42)
    shapes = [(4, 5), (7,), (3, 3), (9,)]
    th0 = [rng.normal(size=s) for s in shapes]
    h = O.Hyper(lr=1e-2)
    A = O.TensorList(shapes, [t.copy() for t in th0])
    B = O.TensorList(shapes, [t.copy() for t in th0])
    for _ in range(4):
        g = [rng.normal(size=s) for s in shapes]
        before = [t.copy() for t in A.theta]
        A.step(g, h, lib=lib, vector_confidence=False)
        B.step(g, h, lib=lib)
        for i, s in enumerate(shapes):
            if len(s) == 2:
                assert np.array_equal(A.theta[i], B.theta[i]) and np.array_equal(A.state[i].R, B.state[i].R)
            else:
                np.testing.assert_allclose(A.state[i].M, B.state[i].M, rtol=1e-13)
                np.testing.assert_allclose(A.state[i].v, B.state[i].v, rtol=1e-13)
                assert not A.state[i].s.any() and B.state[i].s.all()
                np.testing.assert_allclose(A.theta[i] - before[i], -h.lr * A.state[i].M, rtol=1e-9, atol=1e-15)
                assert not np.allclose(A.theta[i], B.theta[i])


ALL_PINS = [
    pin_step1_rank1_reconstruction,
    pin_rms_clip,
    pin_dense_brute_force,
    pin_state_size,
    pin_step1_closed_form,
    pin_zero_gradient,
    pin_vector_is_nx1_matrix,
    pin_instability_identity,
    pin_sum_and_positivity,
    pin_scale_covariance,
    pin_transpose_covariance,
    pin_permutation_equivariance,
    pin_adafactor_subset,
    pin_worked_example,
    pin_list_driver,
    pin_bf16_rounding_by_hand,
    pin_bf16_rounding_matches_library,
    pin_bf16_momentum_mode,
    pin_weight_decay,
    pin_vectors_without_confidence,
]
