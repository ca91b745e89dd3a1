"""ctypes binding of include/came.h.  Same names, argument marshalling only.

There is no CPU fallback: if libcame_hip.so is missing the import of the
library fails loudly (build it with `python -m paper_2307_02047_amd.build`).
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Sequence

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libcame_hip.so")

GRAD_F32, GRAD_BF16 = 0, 1
ALGO_CAME, ALGO_ADAFACTOR = 0, 1
MOMENTUM_F32, MOMENTUM_BF16 = 0, 1
VECTOR_ALGORITHM2, VECTOR_MOMENTUM_ONLY = 0, 1
RESIDENT_AUTO, RESIDENT_OFF, RESIDENT_ON = 0, 1, 2
ETIMEOUT = -6

EXPORTS = ("came_state_size", "came_init_state", "came_step", "came_step_bf16_copy", "came_step_noalloc", "came_state_view_get",
           "came_plan_query", "came_plan_traffic", "came_device_status", "came_algorithmic_bytes", "came_probe_placement", "came_profile_enable",
           "came_profile_read", "came_last_hip_error",
           "came_destroy", "came_strerror")


class CameError(RuntimeError):
    def __init__(self, status: int, what: str, hip_error: int = 0):
        self.status, self.hip_error = status, hip_error
        extra = f" (hipError_t {hip_error})" if hip_error else ""
        super().__init__(f"{what}: status {status}{extra}")


class _Desc(ctypes.Structure):
    _fields_ = [("rows", ctypes.c_int64), ("cols", ctypes.c_int64), ("ndim", ctypes.c_int32),
                ("grad_dtype", ctypes.c_int32)]


class _Hyper(ctypes.Structure):
    _fields_ = [(k, ctypes.c_double) for k in ("beta1", "beta2", "beta3", "eps1", "eps2", "clip_d", "weight_decay")]


class _Options(ctypes.Structure):
    _fields_ = [("tile_rows", ctypes.c_int32), ("algo", ctypes.c_int32),
                ("group_elements", ctypes.c_int64), ("momentum_dtype", ctypes.c_int32),
                ("vector_rule", ctypes.c_int32), ("resident", ctypes.c_int32), ("resident_wait_us", ctypes.c_int32),
                ("tile_rows3", ctypes.c_int32), ("reserved", ctypes.c_int32)]


class _View(ctypes.Structure):
    _fields_ = [(k, ctypes.c_void_p) for k in ("m", "r", "c", "R", "C")]


@dataclass
class CameHyper:
    """Algorithm 2's hyper-parameters (defaults: Section 3.3 / Section 4.1)."""
    beta1: float = 0.9
    beta2: float = 0.999
    beta3: float = 0.9999
    eps1: float = 1e-30
    eps2: float = 1e-16
    clip_d: float = 1.0
    weight_decay: float = 0.0  # decoupled weight decay (not in the paper); 0 = Algorithm 2 as printed

    def _c(self) -> _Hyper:
        return _Hyper(self.beta1, self.beta2, self.beta3, self.eps1, self.eps2, self.clip_d, self.weight_decay)


_lib = None


def load_library(path: str | None = None) -> ctypes.CDLL:
    global _lib
    if _lib is not None and path is None:
        return _lib
    p = path or _LIB_PATH
    if not os.path.exists(p):
        raise ImportError(f"{p} not found: build it with `python -m paper_2307_02047_amd.build` "
                          "(there is no CPU fallback)")
    lib = ctypes.CDLL(p)
    vp, i32, i64, dbl = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_double
    szp = ctypes.POINTER(ctypes.c_size_t)
    lib.came_state_size.argtypes = [ctypes.POINTER(_Desc), i32, ctypes.POINTER(_Options), szp, szp]
    lib.came_state_size.restype = ctypes.c_int
    lib.came_init_state.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(_Desc), i32, ctypes.POINTER(_Options),
                                    vp, ctypes.c_size_t, vp, ctypes.c_size_t, vp]
    lib.came_init_state.restype = ctypes.c_int
    lib.came_step.argtypes = [vp, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(_Hyper), dbl, i64, vp]
    lib.came_step.restype = ctypes.c_int
    lib.came_step_bf16_copy.argtypes = [vp, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp),
                                        ctypes.POINTER(_Hyper), dbl, i64, vp]
    lib.came_step_bf16_copy.restype = ctypes.c_int
    lib.came_step_noalloc.argtypes = [ctypes.POINTER(_Desc), i32, ctypes.POINTER(_Options), vp, ctypes.c_size_t, i32,
                                      ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(_Hyper), dbl, i64, vp]
    lib.came_step_noalloc.restype = ctypes.c_int
    lib.came_state_view_get.argtypes = [vp, i32, ctypes.POINTER(_View)]
    lib.came_state_view_get.restype = ctypes.c_int
    lib.came_plan_query.argtypes = [ctypes.POINTER(_Desc), i32, ctypes.POINTER(_Options), ctypes.POINTER(i64)]
    lib.came_plan_query.restype = ctypes.c_int
    lib.came_plan_traffic.argtypes = [ctypes.POINTER(_Desc), i32, ctypes.POINTER(_Options), ctypes.POINTER(dbl)]
    lib.came_plan_traffic.restype = ctypes.c_int
    lib.came_device_status.argtypes = [vp, vp]
    lib.came_device_status.restype = ctypes.c_int
    lib.came_algorithmic_bytes.argtypes = [i32, i32, i32, i32]
    lib.came_algorithmic_bytes.restype = dbl
    lib.came_probe_placement.argtypes = [vp, ctypes.POINTER(vp), ctypes.POINTER(vp), vp, i32, ctypes.POINTER(dbl)]
    lib.came_probe_placement.restype = ctypes.c_int
    lib.came_profile_enable.argtypes = [vp, i32]
    lib.came_profile_enable.restype = ctypes.c_int
    lib.came_profile_read.argtypes = [vp, ctypes.POINTER(dbl), ctypes.POINTER(i64)]
    lib.came_profile_read.restype = ctypes.c_int
    lib.came_last_hip_error.argtypes = [vp]
    lib.came_last_hip_error.restype = ctypes.c_int
    lib.came_destroy.argtypes = [vp]
    lib.came_destroy.restype = None
    lib.came_strerror.argtypes = [ctypes.c_int]
    lib.came_strerror.restype = ctypes.c_char_p
    if path is None:
        _lib = lib
    return lib


def matrix_view_of(shape: Sequence[int]) -> tuple:
    """The (rows, cols) a parameter of this shape is factored as: itself for 2-D; for more
    dimensions the leading ones are merged (the paper defines the method for matrices only;
    a contiguous tensor of shape (a, b, ..., z) is the row-major matrix (a*b*..., z))."""
    s = tuple(int(x) for x in shape)
    if len(s) <= 2:
        return s
    rows = 1
    for x in s[:-1]:
        rows *= x
    return (rows, s[-1])


def _descs(shapes: Sequence[Sequence[int]], grad_dtypes: Sequence[int]):
    arr = (_Desc * len(shapes))()
    for i, (s, d) in enumerate(zip(shapes, grad_dtypes)):
        s = matrix_view_of(s)
        if len(s) == 2:
            arr[i] = _Desc(s[0], s[1], 2, int(d))
        elif len(s) == 1:
            arr[i] = _Desc(s[0], 1, 1, int(d))
        else:
            raise ValueError(f"tensor {i}: a parameter needs at least one dimension, got shape {s}")
    return arr


def _options(tile_rows: int = 0, algo: int = ALGO_CAME, group_elements: int = 0,
             momentum_dtype: int = MOMENTUM_F32, vector_rule: int = VECTOR_ALGORITHM2,
             resident: int = RESIDENT_AUTO, resident_wait_us: int = 0, tile_rows3: int = 0):
    o = _Options()
    o.tile_rows, o.algo, o.group_elements = int(tile_rows), int(algo), int(group_elements)
    o.momentum_dtype, o.vector_rule = int(momentum_dtype), int(vector_rule)
    o.resident, o.resident_wait_us = int(resident), int(resident_wait_us)
    o.tile_rows3 = int(tile_rows3)
    return o


def _check(lib, status: int, what: str, ctx=None):
    if status != 0:
        msg = lib.came_strerror(status).decode()
        hip = lib.came_last_hip_error(ctx) if ctx else 0
        raise CameError(status, f"{what}: {msg}", hip)


def state_size(shapes, grad_dtypes, **opts) -> tuple[int, int]:
    """came_state_size: (state_bytes, scratch_bytes).  Host only."""
    lib = load_library()
    d, o = _descs(shapes, grad_dtypes), _options(**opts)
    sb, wb = ctypes.c_size_t(), ctypes.c_size_t()
    _check(lib, lib.came_state_size(d, len(shapes), ctypes.byref(o), ctypes.byref(sb), ctypes.byref(wb)),
           "came_state_size")
    return sb.value, wb.value


def plan_query(shapes, grad_dtypes, **opts) -> dict:
    """came_plan_query as a dict.  Host only."""
    lib = load_library()
    d, o = _descs(shapes, grad_dtypes), _options(**opts)
    out = (ctypes.c_int64 * 8)()
    _check(lib, lib.came_plan_query(d, len(shapes), ctypes.byref(o), out), "came_plan_query")
    keys = ("tile_rows", "tile_cols", "sweep_items", "finalize_items", "groups", "matrices", "vectors",
            "elements")
    return dict(zip(keys, [int(x) for x in out]))


def plan_traffic(shapes, grad_dtypes, **opts) -> dict:
    """came_plan_traffic as a dict.  Host only."""
    lib = load_library()
    d, o = _descs(shapes, grad_dtypes), _options(**opts)
    out = (ctypes.c_double * 4)()
    _check(lib, lib.came_plan_traffic(d, len(shapes), ctypes.byref(o), out), "came_plan_traffic")
    return {"resident_matrices": int(out[0]), "resident_elements": int(out[1]), "bytes_per_step": float(out[2]),
            "bytes_per_step_streaming": float(out[3])}


def algorithmic_bytes(grad_bytes: int, momentum_bytes: int = 4, algo: int = ALGO_CAME, which: int = 0) -> float:
    return float(load_library().came_algorithmic_bytes(int(grad_bytes), int(momentum_bytes), int(algo), int(which)))


def step_noalloc(shapes, grad_dtypes, state, zero_state: bool, thetas, grads, hyper: CameHyper, lr: float, step: int,
                 stream=None, **opts) -> None:
    """came_step_noalloc: one step on the library's own scratch.  `state` is the caller's uint8
    state blob (state_size()'s bytes, 256-byte aligned)."""
    import torch
    lib = load_library()
    n = len(shapes)
    d, o = _descs(shapes, grad_dtypes), _options(**opts)
    th = (ctypes.c_void_p * n)(*[t.data_ptr() for t in thetas])
    gr = (ctypes.c_void_p * n)(*[g.data_ptr() for g in grads])
    h = hyper._c()
    with torch.cuda.device(state.device):
        s = stream if stream is not None else torch.cuda.current_stream(state.device).cuda_stream
        st = lib.came_step_noalloc(d, n, ctypes.byref(o), state.data_ptr(), state.numel(), 1 if zero_state else 0,
                                   th, gr, ctypes.byref(h), float(lr), int(step), s)
    if st != 0:
        raise CameError(st, f"came_step_noalloc: {lib.came_strerror(st).decode()}", lib.came_last_hip_error(None))


class CameStep:
    """came_init_state / came_step / came_state_view_get / came_destroy for one tensor list.

    The state and scratch blobs are torch uint8 tensors on `device` (PyTorch is the
    device-memory allocator); everything else happens inside the library.
    """

    def __init__(self, shapes, grad_dtypes, device="cuda:0", tile_rows: int = 0, algo: int = ALGO_CAME,
                 group_elements: int = 0, momentum_dtype: int = MOMENTUM_F32,
                 vector_rule: int = VECTOR_ALGORITHM2, resident: int = RESIDENT_AUTO, resident_wait_us: int = 0,
                 tile_rows3: int = 0, place_against=None, place_against_grads=None,
                 placement_candidates: int = 8, placement_spacer_bytes: int = 16 << 30,
                 placement_accept_ratio: float = 1.04, placement_reserve_bytes: int = 2 << 30, blobs=None):
        """blobs: (state, scratch), two uint8 tensors on `device` of at least state_size()'s bytes
        at 256-byte aligned addresses, when the caller wants to place them itself; by default
        both are allocated here.
        place_against: the parameter tensors the context will be stepped with (and, in
        place_against_grads, the gradient buffers if they are long-lived).  When given, the
        state blob is allocated at up to `placement_candidates` different addresses, each
        followed by `placement_spacer_bytes` of temporary spacers; each is measured with
        came_probe_placement against the parameters and the fastest is kept.  The search is
        bounded by what torch.cuda.mem_get_info reports as free (a candidate is only tried if it,
        its spacers and placement_reserve_bytes fit) and stops early at the first candidate
        that is placement_accept_ratio times faster than the first one, i.e. than the place the
        allocator chose by itself: on MI355X the read+write sweep is ~10 % faster when theta
        and the state sit in different 96 GB regions of the HBM address space.  Memory is
        only allocated and measured here; nothing about the arithmetic changes."""
        import torch
        self._torch = torch
        self.lib = load_library()
        self.shapes = [tuple(int(x) for x in s) for s in shapes]
        self.grad_dtypes = [int(d) for d in grad_dtypes]
        self.device = torch.device(device)
        self._d = _descs(self.shapes, self.grad_dtypes)
        self._o = _options(tile_rows, algo, group_elements, momentum_dtype, vector_rule, resident, resident_wait_us,
                           tile_rows3)
        self.momentum_dtype = int(momentum_dtype)
        n = len(self.shapes)
        sb, wb = ctypes.c_size_t(), ctypes.c_size_t()
        _check(self.lib, self.lib.came_state_size(self._d, n, ctypes.byref(self._o), ctypes.byref(sb),
                                                  ctypes.byref(wb)), "came_state_size")
        self.state_bytes, self.scratch_bytes = sb.value, wb.value
        self._theta_arr = (ctypes.c_void_p * n)()
        self._grad_arr = (ctypes.c_void_p * n)()
        self.placement_log = []  # (candidate index, probe GB/s)
        self._blobs = blobs
        if blobs is not None and place_against is not None:
            raise ValueError("blobs and place_against exclude each other")
        if place_against is None:
            self.state, self.scratch, self._ctx = self._create()
            return
        if len(place_against) != n or (place_against_grads is not None and len(place_against_grads) != n):
            raise ValueError(f"place_against(_grads) must hold the {n} parameter (gradient) tensors")
        # Every candidate and spacer stays allocated until the search ends, so that each new
        # candidate really lies at a new place (a freed block would be handed out again).
        tried, spacers, best = [], [], None
        need = self.state_bytes + self.scratch_bytes + int(placement_reserve_bytes)
        for k in range(max(1, placement_candidates)):
            if k > 0:
                free_bytes, _ = torch.cuda.mem_get_info(self.device)
                if free_bytes < need + int(placement_spacer_bytes):
                    break  # no room for another candidate behind a spacer: keep the best so far
                # in pieces of at most 1 GiB: the allocator lays small allocations out one after the
                # other, whereas a single huge spacer may be put somewhere else entirely
                left = int(placement_spacer_bytes)
                while left > 0:
                    piece = min(left, 1 << 30)
                    spacers.append(torch.empty(piece, dtype=torch.uint8, device=self.device))
                    left -= piece
            cand = self._create()
            tried.append(cand)
            self.state, self.scratch, self._ctx = cand
            gbs = self.probe_placement(place_against, place_against_grads)
            self.placement_log.append((k, gbs))
            if best is None or gbs > best[0]:
                best = (gbs, cand)
            if k > 0 and gbs >= placement_accept_ratio * self.placement_log[0][1]:
                break
        for cand in tried:
            if cand is not best[1]:
                self._destroy(cand)
        self.state, self.scratch, self._ctx = best[1]
        del spacers, tried, cand
        torch.cuda.empty_cache()  # hand the losing candidates and the spacers back to the driver

    def _create(self):
        torch = self._torch
        n = len(self.shapes)
        with torch.cuda.device(self.device):
            if self._blobs is not None:
                state, scratch = self._blobs
                if state.dtype != torch.uint8 or scratch.dtype != torch.uint8 or not (state.is_contiguous() and scratch.is_contiguous()):
                    raise ValueError("blobs must be contiguous uint8 tensors")
            else:
                state = torch.empty(self.state_bytes, dtype=torch.uint8, device=self.device)
                scratch = torch.empty(self.scratch_bytes, dtype=torch.uint8, device=self.device)
            ctx = ctypes.c_void_p()
            stream = torch.cuda.current_stream(self.device).cuda_stream
            st = self.lib.came_init_state(ctypes.byref(ctx), self._d, n, ctypes.byref(self._o),
                                          state.data_ptr(), state.numel(),
                                          scratch.data_ptr(), scratch.numel(), stream)
        _check(self.lib, st, "came_init_state")
        return state, scratch, ctx

    def _destroy(self, cand) -> None:
        self._torch.cuda.synchronize(self.device)
        self.lib.came_destroy(cand[2])

    def probe_placement(self, thetas, grads=None, repeats: int = 2) -> float:
        """came_probe_placement: GB/s of sweep 3's memory traffic (theta and M rewritten in place,
        contents unchanged) and, when the gradient buffers are given, of sweep 2's as well."""
        torch = self._torch
        n = len(self.shapes)
        arr = (ctypes.c_void_p * n)(*[t.data_ptr() for t in thetas])
        garr = None if grads is None else (ctypes.c_void_p * n)(*[g.data_ptr() for g in grads])
        out = ctypes.c_double()
        with torch.cuda.device(self.device):
            s = torch.cuda.current_stream(self.device).cuda_stream
            st = self.lib.came_probe_placement(self._ctx, arr, garr, s, int(repeats), ctypes.byref(out))
        _check(self.lib, st, "came_probe_placement", self._ctx)
        return float(out.value)

    def step(self, thetas, grads, hyper: CameHyper, lr: float, step: int, stream=None, bf16_copies=None) -> None:
        """came_step, or came_step_bf16_copy when bf16_copies is given (a list with, per tensor,
        a bfloat16 tensor of the parameter's shape or None)."""
        torch = self._torch
        n = len(self.shapes)
        if len(thetas) != n or len(grads) != n:
            raise ValueError(f"expected {n} parameters and {n} gradients, got {len(thetas)} and {len(grads)}")
        for i in range(n):
            self._theta_arr[i] = thetas[i].data_ptr()
            self._grad_arr[i] = grads[i].data_ptr()
        h = hyper._c()
        with torch.cuda.device(self.device):
            s = stream if stream is not None else torch.cuda.current_stream(self.device).cuda_stream
            if bf16_copies is None:
                st = self.lib.came_step(self._ctx, self._theta_arr, self._grad_arr, ctypes.byref(h), float(lr),
                                        int(step), s)
                what = "came_step"
            else:
                if len(bf16_copies) != n:
                    raise ValueError(f"expected {n} bf16 copy entries (tensor or None), got {len(bf16_copies)}")
                arr = (ctypes.c_void_p * n)()
                for i, c in enumerate(bf16_copies):
                    if c is not None:
                        if c.dtype != torch.bfloat16 or tuple(c.shape) != self.shapes[i] or not c.is_contiguous():
                            raise ValueError(f"tensor {i}: bf16 copy must be a contiguous bfloat16 tensor of shape {self.shapes[i]}")
                        arr[i] = c.data_ptr()
                st = self.lib.came_step_bf16_copy(self._ctx, self._theta_arr, self._grad_arr, arr, ctypes.byref(h),
                                                  float(lr), int(step), s)
                what = "came_step_bf16_copy"
        _check(self.lib, st, what, self._ctx)

    def check_tensors(self, thetas, grads) -> None:
        """Host-side shape/dtype check of what step() will hand to the kernels."""
        torch = self._torch
        for i, (s, d) in enumerate(zip(self.shapes, self.grad_dtypes)):
            want = torch.bfloat16 if d == GRAD_BF16 else torch.float32
            t, g = thetas[i], grads[i]
            if tuple(t.shape) != s or tuple(g.shape) != s:
                raise ValueError(f"tensor {i}: shapes {tuple(t.shape)}/{tuple(g.shape)} do not match plan {s}")
            if t.dtype != torch.float32 or g.dtype != want:
                raise ValueError(f"tensor {i}: dtypes {t.dtype}/{g.dtype}, expected float32/{want}")
            if not (t.is_contiguous() and g.is_contiguous()):
                raise ValueError(f"tensor {i}: tensors must be contiguous")
            if t.device != self.device or g.device != self.device:
                raise ValueError(f"tensor {i}: tensors must live on {self.device}")

    def state_view(self, i: int) -> dict:
        """came_state_view_get as torch views into the state blob (float32; M is bfloat16
        when the context keeps a bfloat16 momentum)."""
        v = _View()
        _check(self.lib, self.lib.came_state_view_get(self._ctx, int(i), ctypes.byref(v)), "came_state_view_get")
        base = self.state.data_ptr()
        f = self.state.view(self._torch.float32)
        s = self.shapes[i]
        mv = matrix_view_of(s)
        n, m = (mv[0], mv[1]) if len(mv) == 2 else (mv[0], 1)

        def sl(ptr, count, shape):
            if not ptr:
                return None
            off = (ptr - base) // 4
            return f[off:off + count].view(shape)

        if self.momentum_dtype == MOMENTUM_BF16:
            h = self.state.view(self._torch.bfloat16)
            off = (v.m - base) // 2
            M = h[off:off + n * m].view(s)
        else:
            M = sl(v.m, n * m, s)
        return {"M": M, "r": sl(v.r, n, (n,)), "c": sl(v.c, m, (m,)),
                "R": sl(v.R, n, (n,)), "C": sl(v.C, m, (m,))}

    PHASES = ("sweep1", "finalize1", "sweep2", "finalize2", "sweep3", "vectors", "resident")

    def device_status(self, stream=None) -> int:
        """came_device_status: waits for the stream; 0, or ETIMEOUT when the on-chip kernel gave up a wait."""
        torch = self._torch
        with torch.cuda.device(self.device):
            s = stream if stream is not None else torch.cuda.current_stream(self.device).cuda_stream
            return int(self.lib.came_device_status(self._ctx, s))

    def profile_enable(self, on: bool = True) -> None:
        _check(self.lib, self.lib.came_profile_enable(self._ctx, 1 if on else 0), "came_profile_enable")

    def profile_read(self) -> dict:
        """came_profile_read: {phase: (total_ms, launches)} since the previous read."""
        ms = (ctypes.c_double * 7)()
        cnt = (ctypes.c_int64 * 7)()
        _check(self.lib, self.lib.came_profile_read(self._ctx, ms, cnt), "came_profile_read", self._ctx)
        return {k: (float(ms[i]), int(cnt[i])) for i, k in enumerate(self.PHASES)}

    def close(self) -> None:
        if getattr(self, "_ctx", None) and self._ctx.value:
            self._torch.cuda.synchronize(self.device)
            self.lib.came_destroy(self._ctx)
            self._ctx = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
