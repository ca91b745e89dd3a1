"""torch.optim front end of the library: the step of Algorithm 2 inside a PyTorch training loop.

Argument marshalling only.  Each parameter group becomes one context of the C library
(one grouped launch sequence per phase for all tensors of the group); the optimizer state
lives in the library's state blob, and `self.state[p]` holds torch views into it under the
paper's names (M, r, c, R, C; for 1-D parameters M, v, s), so that `state_dict()` /
`load_state_dict()` checkpoint it like any other optimizer's.

Requirements: parameters are float32, contiguous and on one GPU; gradients are float32 or
bfloat16 (decided at the first step, per parameter) and dense.  Every parameter of a group
must have a gradient at every step (the library updates the whole list in one go).
"""
from __future__ import annotations

import torch

from .binding import (ALGO_ADAFACTOR, ALGO_CAME, GRAD_BF16, GRAD_F32, MOMENTUM_BF16, MOMENTUM_F32,
                      VECTOR_ALGORITHM2, VECTOR_MOMENTUM_ONLY, CameHyper, CameStep)


class CAME(torch.optim.Optimizer):
    """CAME (Algorithm 2 of the paper) on MI355X.

    lr: eta.  betas: (beta1, beta2, beta3).  eps: (eps1, eps2).  clip_threshold: d of Eq. 1.
    weight_decay: decoupled, theta <- theta - eta*lambda*theta before the update (0: none, as in
    the paper).  algorithm: "came" (Algorithm 2) or "adafactor" (Algorithm 1, momentum only).
    momentum_dtype: "f32" or "bf16" (M stored as bfloat16 between steps).
    vector_confidence: False updates 1-D parameters by -eta*M (no confidence statistics).
    All of these are per parameter group.
    place_state: search for a fast address of the state blob relative to the parameters at the
    first step (see CameStep's place_against; temporarily allocates a lot of device memory).
    """

    def __init__(self, params, lr: float = 2e-4, betas=(0.9, 0.999, 0.9999), eps=(1e-30, 1e-16),
                 clip_threshold: float = 1.0, weight_decay: float = 0.0, algorithm: str = "came",
                 momentum_dtype: str = "f32", vector_confidence: bool = True, place_state: bool = False):
        if algorithm not in ("came", "adafactor"):
            raise ValueError(f"algorithm must be 'came' or 'adafactor', got {algorithm!r}")
        if momentum_dtype not in ("f32", "bf16"):
            raise ValueError(f"momentum_dtype must be 'f32' or 'bf16', got {momentum_dtype!r}")
        defaults = dict(lr=lr, betas=tuple(betas), eps=tuple(eps), clip_threshold=clip_threshold,
                        weight_decay=weight_decay, algorithm=algorithm, momentum_dtype=momentum_dtype,
                        vector_confidence=vector_confidence)
        super().__init__(params, defaults)
        self._place_state = bool(place_state)
        self._engines = {}  # index of the parameter group -> (CameStep, [params], step count)

    # ------------------------------------------------------------------ engine per group
    def _engine(self, gi: int, group, grads):
        if gi in self._engines:
            return self._engines[gi]
        ps = group["params"]
        for p in ps:
            if p.dtype != torch.float32 or not p.is_contiguous() or not p.is_cuda:
                raise ValueError("CAME: parameters must be contiguous float32 CUDA tensors")
            if p.device != ps[0].device:
                raise ValueError("CAME: all parameters of a group must be on one device")
        dts = []
        for g in grads:
            if g.dtype == torch.float32:
                dts.append(GRAD_F32)
            elif g.dtype == torch.bfloat16:
                dts.append(GRAD_BF16)
            else:
                raise ValueError(f"CAME: gradients must be float32 or bfloat16, got {g.dtype}")
        eng = CameStep([tuple(p.shape) if p.dim() > 0 else (1,) for p in ps], dts, device=ps[0].device,
                       algo=ALGO_CAME if group["algorithm"] == "came" else ALGO_ADAFACTOR,
                       momentum_dtype=MOMENTUM_BF16 if group["momentum_dtype"] == "bf16" else MOMENTUM_F32,
                       vector_rule=VECTOR_ALGORITHM2 if group["vector_confidence"] else VECTOR_MOMENTUM_ONLY,
                       place_against=[p.data for p in ps] if self._place_state else None)
        self._engines[gi] = [eng, list(ps), 0]
        for k, p in enumerate(ps):
            self.state[p] = self._views(eng, k, p, 0)
        return self._engines[gi]

    @staticmethod
    def _views(eng: CameStep, k: int, p, step: int) -> dict:
        v = eng.state_view(k)
        if p.dim() >= 2:
            return {"step": step, "M": v["M"], "r": v["r"], "c": v["c"], "R": v["R"], "C": v["C"]}
        return {"step": step, "M": v["M"], "v": v["r"], "s": v["R"]}

    # ------------------------------------------------------------------ step
    @torch.no_grad()
    def step(self, closure=None, grads=None):
        """One optimizer step.  grads: optional list (one list per parameter group, or a flat list
        for a single group) of gradient tensors to use instead of `p.grad` -- e.g. bfloat16
        gradients of a bf16 compute copy while the float32 master parameters are updated."""
        loss = None
        if closure is not None:
            with torch.enable_grad():
                loss = closure()
        if grads is not None and len(self.param_groups) == 1 and (len(grads) == 0 or torch.is_tensor(grads[0])):
            grads = [grads]
        for gi, group in enumerate(self.param_groups):
            ps = group["params"]
            gs = list(grads[gi]) if grads is not None else [p.grad for p in ps]
            if any(g is None for g in gs):
                raise RuntimeError("CAME: every parameter of a group needs a gradient at every step")
            gs = [g if g.is_contiguous() else g.contiguous() for g in gs]
            if any(g.is_sparse for g in gs):
                raise RuntimeError("CAME: sparse gradients are not supported")
            entry = self._engine(gi, group, gs)
            eng, plist, t = entry
            if len(plist) != len(ps) or any(a is not b for a, b in zip(plist, ps)):
                raise RuntimeError("CAME: the parameters of a group must not change after the first step")
            b1, b2, b3 = group["betas"]
            e1, e2 = group["eps"]
            h = CameHyper(b1, b2, b3, e1, e2, group["clip_threshold"], group["weight_decay"])
            eng.check_tensors([p.data.view(s) for p, s in zip(ps, eng.shapes)],
                              [g.view(s) for g, s in zip(gs, eng.shapes)])
            eng.step([p.data for p in ps], gs, h, float(group["lr"]), t + 1)
            entry[2] = t + 1
            for p in ps:
                self.state[p]["step"] = t + 1
        return loss

    # ------------------------------------------------------------------ checkpointing
    def load_state_dict(self, state_dict) -> None:
        """Loads a checkpoint made by state_dict(): the tensors are copied INTO the library's state
        blob (the entries of self.state stay views of it).  The contexts are created here if no
        step has run yet, with the gradient dtype recorded in the checkpoint."""
        super().load_state_dict(state_dict)
        for gi, group in enumerate(self.param_groups):
            ps = group["params"]
            loaded = [self.state.get(p) for p in ps]
            if all(not st for st in loaded):
                continue
            if any(not st for st in loaded):
                raise RuntimeError("CAME: checkpoint holds state for only some parameters of a group")
            if gi not in self._engines:
                dts = group.get("grad_dtypes")
                if dts is None:
                    raise RuntimeError("CAME: checkpoint lacks the gradient dtypes of its groups")
                fake = [torch.empty(0, dtype=torch.bfloat16 if d == GRAD_BF16 else torch.float32) for d in dts]
                self._engine(gi, group, fake)
            entry = self._engines[gi]
            eng = entry[0]
            step = 0
            for k, (p, st) in enumerate(zip(ps, loaded)):
                views = self._views(eng, k, p, int(st["step"]))
                for name, dst in views.items():
                    if name != "step":
                        dst.copy_(st[name].to(dst.dtype))
                self.state[p] = views
                step = int(st["step"])
            entry[2] = step

    def state_dict(self):
        """The usual optimizer state_dict; its tensors are COPIES of the state blob's arrays (the
        blob holds arrays of different dtypes side by side, which a serialiser cannot store as
        views of one storage)."""
        for gi, group in enumerate(self.param_groups):
            if gi in self._engines:
                group["grad_dtypes"] = list(self._engines[gi][0].grad_dtypes)
        sd = super().state_dict()
        sd["state"] = {k: {name: (v.clone() if torch.is_tensor(v) else v) for name, v in st.items()}
                       for k, st in sd["state"].items()}
        return sd

    def close(self) -> None:
        for eng, _, _ in self._engines.values():
            eng.close()
        self._engines.clear()
