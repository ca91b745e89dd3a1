"""ctypes front end of the CPU oracle (oracle/came_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg.  Nothing under paper_2307_02047_amd/ may import it.

All arrays are C-contiguous numpy float64 and are updated in place, exactly as
the C functions document.  build() compiles the C file with gcc next to itself.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "came_oracle.c")
_LIB = os.path.join(_HERE, "libcame_oracle.so")

_c_double_p = ctypes.POINTER(ctypes.c_double)


class _Hyper(ctypes.Structure):
    _fields_ = [(k, ctypes.c_double) for k in
                ("beta1", "beta2", "beta3", "eps1", "eps2", "clip_d", "lr")]


@dataclass
class Hyper:
    """Hyper-parameters of Algorithm 2 (defaults: Section 3.3 toy example and
    Section 4.1 'Implementation Detail')."""
    beta1: float = 0.9
    beta2: float = 0.999
    beta3: float = 0.9999
    eps1: float = 1e-30
    eps2: float = 1e-16
    clip_d: float = 1.0
    lr: float = 2e-4

    def c(self) -> _Hyper:
        return _Hyper(self.beta1, self.beta2, self.beta3, self.eps1, self.eps2,
                      self.clip_d, self.lr)


def build(src: str = _SRC, out: str = _LIB, openmp: bool = True) -> str:
    """Compile the oracle with gcc (plain C99, -O2)."""
    cmd = ["gcc", "-std=c99", "-O2", "-Wall", "-Wextra", "-fPIC", "-shared"]
    if openmp:
        cmd.append("-fopenmp")
    cmd += [src, "-o", out, "-lm"]
    subprocess.run(cmd, check=True)
    return out


_lib = None


def load(path: str | None = None) -> ctypes.CDLL:
    """Load (building first if the library is absent or older than its source)."""
    global _lib
    if path is None:
        if _lib is not None:
            return _lib
        if (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
            build()
        path = _LIB
    lib = ctypes.CDLL(path)
    i64, i32, dp, hp = ctypes.c_int64, ctypes.c_int32, _c_double_p, ctypes.POINTER(_Hyper)
    lib.came_oracle_matrix_step.argtypes = [i64, i64, dp, dp, dp, dp, dp, dp, dp, hp, dp]
    lib.came_oracle_matrix_step.restype = ctypes.c_int
    lib.came_oracle_vector_step.argtypes = [i64, dp, dp, dp, dp, dp, hp, dp]
    lib.came_oracle_vector_step.restype = ctypes.c_int
    lib.came_oracle_dense_step.argtypes = [i64, i64, dp, dp, dp, dp, dp, dp, dp, dp, dp, hp]
    lib.came_oracle_dense_step.restype = ctypes.c_int
    lib.adafactor_oracle_matrix_step.argtypes = [i64, i64, dp, dp, dp, dp, dp, hp, dp]
    lib.adafactor_oracle_matrix_step.restype = ctypes.c_int
    pp = ctypes.POINTER(_c_double_p)
    lib.came_oracle_step_list.argtypes = [i32, ctypes.POINTER(i64), ctypes.POINTER(i64),
                                          ctypes.POINTER(i32), pp, pp, pp, pp, pp, pp, pp, hp, i32]
    lib.came_oracle_step_list.restype = ctypes.c_int
    lib.came_oracle_round_bf16.argtypes = [ctypes.c_double]
    lib.came_oracle_round_bf16.restype = ctypes.c_double
    lib.came_oracle_store_bf16.argtypes = [dp, i64]
    lib.came_oracle_store_bf16.restype = None
    lib.came_oracle_decay.argtypes = [dp, i64, ctypes.c_double, ctypes.c_double]
    lib.came_oracle_decay.restype = None
    lib.came_oracle_max_threads.argtypes = []
    lib.came_oracle_max_threads.restype = i32
    if path == _LIB:
        _lib = lib
    return lib


def _p(a: np.ndarray):
    assert a.dtype == np.float64 and a.flags.c_contiguous, "oracle arrays are contiguous float64"
    return a.ctypes.data_as(_c_double_p)


class MatrixState:
    """State of one n x m matrix: M (n*m) plus the factored r, R (n) and c, C (m),
    all zero at t = 0 (Algorithm 2 input list; R_0 = C_0 = 0 by our reading)."""

    def __init__(self, n: int, m: int):
        self.n, self.m = n, m
        self.M = np.zeros((n, m))
        self.r = np.zeros(n)
        self.c = np.zeros(m)
        self.R = np.zeros(n)
        self.C = np.zeros(m)

    def elems(self) -> int:
        return self.M.size + self.r.size + self.c.size + self.R.size + self.C.size

    def factored_elems(self) -> int:
        return self.r.size + self.c.size + self.R.size + self.C.size


class VectorState:
    """State of one length-n vector: M, v, s (n each)."""

    def __init__(self, n: int):
        self.n = n
        self.M = np.zeros(n)
        self.v = np.zeros(n)
        self.s = np.zeros(n)

    def elems(self) -> int:
        return 3 * self.n


def matrix_step(theta: np.ndarray, g: np.ndarray, st: MatrixState, h: Hyper, lib=None):
    """One Algorithm-2 step in place; returns (RMS(u), RMS(u_hat))."""
    lib = lib or load()
    n, m = st.n, st.m
    assert theta.shape == (n, m) and g.shape == (n, m)
    diag = np.zeros(2)
    hc = h.c()
    rc = lib.came_oracle_matrix_step(n, m, _p(theta), _p(g), _p(st.M), _p(st.r), _p(st.c),
                                     _p(st.R), _p(st.C), ctypes.byref(hc), _p(diag))
    if rc != 0:
        raise RuntimeError(f"came_oracle_matrix_step failed: {rc}")
    return float(diag[0]), float(diag[1])


def vector_step(theta: np.ndarray, g: np.ndarray, st: VectorState, h: Hyper, lib=None):
    lib = lib or load()
    assert theta.shape == (st.n,) and g.shape == (st.n,)
    diag = np.zeros(2)
    hc = h.c()
    rc = lib.came_oracle_vector_step(st.n, _p(theta), _p(g), _p(st.M), _p(st.v), _p(st.s),
                                     ctypes.byref(hc), _p(diag))
    if rc != 0:
        raise RuntimeError(f"came_oracle_vector_step failed: {rc}")
    return float(diag[0]), float(diag[1])


class DenseState:
    """O(nm) brute-force state: M, full V and full Ubar; r, c, R, C are outputs."""

    def __init__(self, n: int, m: int):
        self.n, self.m = n, m
        self.M = np.zeros((n, m))
        self.V = np.zeros((n, m))
        self.Ubar = np.zeros((n, m))
        self.r = np.zeros(n)
        self.c = np.zeros(m)
        self.R = np.zeros(n)
        self.C = np.zeros(m)


def dense_step(theta: np.ndarray, g: np.ndarray, st: DenseState, h: Hyper, lib=None):
    lib = lib or load()
    hc = h.c()
    rc = lib.came_oracle_dense_step(st.n, st.m, _p(theta), _p(g), _p(st.M), _p(st.V), _p(st.Ubar),
                                    _p(st.r), _p(st.c), _p(st.R), _p(st.C), ctypes.byref(hc))
    if rc != 0:
        raise RuntimeError(f"came_oracle_dense_step failed: {rc}")


def adafactor_matrix_step(theta, g, M, r, c, h: Hyper, lib=None):
    """One Algorithm-1 step in place; returns (RMS(u), RMS(u_hat))."""
    lib = lib or load()
    n, m = theta.shape
    diag = np.zeros(2)
    hc = h.c()
    rc = lib.adafactor_oracle_matrix_step(n, m, _p(theta), _p(g), _p(M), _p(r), _p(c),
                                          ctypes.byref(hc), _p(diag))
    if rc != 0:
        raise RuntimeError(f"adafactor_oracle_matrix_step failed: {rc}")
    return float(diag[0]), float(diag[1])


class TensorList:
    """A list of parameter tensors with oracle state, stepped together.

    shapes: list of (n, m) for matrices or (n,) for vectors.
    thetas: list of float64 arrays of those shapes (owned by the caller, updated in place).
    """

    def __init__(self, shapes, thetas):
        self.shapes = [tuple(int(x) for x in s) for s in shapes]
        self.theta = [np.ascontiguousarray(t, dtype=np.float64) for t in thetas]
        self.state = [MatrixState(*s) if len(s) == 2 else VectorState(s[0]) for s in self.shapes]
        for s, t in zip(self.shapes, self.theta):
            assert t.shape == s

    def state_elems(self) -> int:
        return sum(s.elems() for s in self.state)

    def step(self, grads, h: Hyper, nthreads: int = 1, lib=None, momentum_bf16: bool = False,
             weight_decay: float = 0.0, vector_confidence: bool = True) -> None:
        """One step of every tensor.  momentum_bf16: after the step (theta and all other
        state already updated from the unrounded m_t) every momentum is replaced by its
        nearest bfloat16, the value the next step reads as m_{t-1}.  weight_decay: decoupled
        decay theta <- theta - eta*lambda*theta applied before the step.  vector_confidence
        False: 1-D parameters take Algorithm 1's update theta <- theta - eta*m_t (no
        instability / confidence statistics; their s stays untouched); matrices are unaffected."""
        lib = lib or load()
        if weight_decay != 0.0:
            for th in self.theta:
                lib.came_oracle_decay(_p(th.reshape(-1)), th.size, h.lr, float(weight_decay))
        if not vector_confidence:
            self._step_vectors_without_confidence(grads, h, lib)
            mats = [i for i, s in enumerate(self.shapes) if len(s) == 2]
            if mats:
                sub = TensorList.__new__(TensorList)
                sub.shapes = [self.shapes[i] for i in mats]
                sub.theta = [self.theta[i] for i in mats]
                sub.state = [self.state[i] for i in mats]
                sub.step([grads[i] for i in mats], h, nthreads=nthreads, lib=lib)
            if momentum_bf16:
                for st in self.state:
                    store_bf16(st.M, lib)
            return
        T = len(self.shapes)
        grads = [np.ascontiguousarray(g, dtype=np.float64) for g in grads]
        rows = (ctypes.c_int64 * T)(*[s[0] for s in self.shapes])
        cols = (ctypes.c_int64 * T)(*[(s[1] if len(s) == 2 else 1) for s in self.shapes])
        ndim = (ctypes.c_int32 * T)(*[len(s) for s in self.shapes])
        arr = _c_double_p * T
        null = ctypes.cast(None, _c_double_p)

        def ptrs(fn):
            return arr(*[fn(i) for i in range(T)])

        th = ptrs(lambda i: _p(self.theta[i]))
        gg = ptrs(lambda i: _p(grads[i]))
        MM = ptrs(lambda i: _p(self.state[i].M))
        rr = ptrs(lambda i: _p(self.state[i].r) if len(self.shapes[i]) == 2 else _p(self.state[i].v))
        cc = ptrs(lambda i: _p(self.state[i].c) if len(self.shapes[i]) == 2 else null)
        RR = ptrs(lambda i: _p(self.state[i].R) if len(self.shapes[i]) == 2 else _p(self.state[i].s))
        CC = ptrs(lambda i: _p(self.state[i].C) if len(self.shapes[i]) == 2 else null)
        hc = h.c()
        rc = lib.came_oracle_step_list(T, rows, cols, ndim, th, gg, MM, rr, cc, RR, CC,
                                       ctypes.byref(hc), nthreads)
        if rc != 0:
            raise RuntimeError(f"came_oracle_step_list failed: {rc}")
        if momentum_bf16:
            for st in self.state:
                store_bf16(st.M, lib)


def _vector_adafactor(self, grads, h, lib):
    """Algorithm 1 on every 1-D parameter of the list, as its n x 1 matrix (then c is the
    scalar sum of v, kept beside the state)."""
    for i, s in enumerate(self.shapes):
        if len(s) != 1:
            continue
        st = self.state[i]
        if not hasattr(st, "c1"):
            st.c1 = np.zeros(1)
        g = np.ascontiguousarray(grads[i], dtype=np.float64)
        adafactor_matrix_step(self.theta[i].reshape(-1, 1), g.reshape(-1, 1), st.M.reshape(-1, 1), st.v, st.c1, h, lib)


TensorList._step_vectors_without_confidence = _vector_adafactor


def round_bf16(x: float, lib=None) -> float:
    """Nearest bfloat16 (ties to even) of the binary32 nearest to x."""
    return float((lib or load()).came_oracle_round_bf16(float(x)))


def store_bf16(a: np.ndarray, lib=None) -> None:
    """round_bf16 on every element of a float64 array, in place."""
    (lib or load()).came_oracle_store_bf16(_p(a.reshape(-1)), a.size)


def max_threads(lib=None) -> int:
    return int((lib or load()).came_oracle_max_threads())
