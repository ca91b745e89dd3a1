"""Seeded synthetic workloads: tensor-shape lists and gradient generators.

This module holds NO optimizer arithmetic.  It only says which tensors a
workload has and draws parameters / gradients from a seed, so that the GPU
library and the CPU oracle (which never import each other) can be fed the very
same bits.  The shape lists stand in for the models the CAME paper trains
(BERT-Base/Large: Sections 4.2-4.3; GPT-2 medium: Section 4.4) plus a
Llama-7B-shaped list for the headline measurement; the paper's datasets and
checkpoints are not needed because the cost and the arithmetic of the
optimizer step depend on shapes, dtypes and the gradient distribution only.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import torch

GRAD_F32, GRAD_BF16 = 0, 1


@dataclass
class Workload:
    name: str
    shapes: list            # (n, m) matrices and (n,) vectors, in model order
    grad_dtype: int         # GRAD_F32 or GRAD_BF16 (all tensors of a workload share it)
    seed: int
    steps: int              # steps of the parity run
    grad_kind: str          # "normal" | "student_t3"
    scale_range: tuple | None  # per-tensor scale s_T log-uniform in this range; None = fixed_scale
    fixed_scale: float = 1.0
    zero_row_fraction: float = 0.0
    lr: float = 2e-4
    extra: dict = field(default_factory=dict)

    @property
    def n_params(self) -> int:
        return sum(math.prod(s) for s in self.shapes)

    @property
    def grad_bytes(self) -> int:
        return 2 if self.grad_dtype == GRAD_BF16 else 4

    def torch_grad_dtype(self):
        return torch.bfloat16 if self.grad_dtype == GRAD_BF16 else torch.float32


def _encoder_shapes(vocab, positions, types, layers, hidden, ffn):
    """BERT-shaped list: embeddings, then per layer Q,K,V,O, two FFN matrices,
    their biases and two LayerNorm gamma/beta pairs."""
    s = [(vocab, hidden), (positions, hidden), (types, hidden)]
    for _ in range(layers):
        s += [(hidden, hidden)] * 4 + [(hidden, ffn), (ffn, hidden)]
        s += [(hidden,)] * 4 + [(ffn,), (hidden,)]
        s += [(hidden,)] * 4
    return s


def _gpt2_shapes(vocab, positions, layers, hidden):
    s = [(vocab, hidden), (positions, hidden)]
    for _ in range(layers):
        s += [(hidden, 3 * hidden), (hidden, hidden), (hidden, 4 * hidden), (4 * hidden, hidden)]
        s += [(3 * hidden,), (hidden,), (4 * hidden,), (hidden,)]
        s += [(hidden,)] * 4
    return s


def _llama_shapes(vocab, layers, hidden, ffn):
    s = [(vocab, hidden)]
    for _ in range(layers):
        s += [(hidden, hidden)] * 4 + [(hidden, ffn), (hidden, ffn), (ffn, hidden)]
        s += [(hidden,)] * 2
    s += [(hidden,), (vocab, hidden)]
    return s


def single_matrix() -> Workload:
    return Workload("single-256x512+bias", [(256, 512), (512,)], GRAD_F32, seed=1, steps=10,
                    grad_kind="normal", scale_range=None, fixed_scale=0.01)


def bert_base() -> Workload:
    return Workload("bert-base-shaped", _encoder_shapes(30522, 512, 2, 12, 768, 3072), GRAD_F32, seed=2,
                    steps=100, grad_kind="normal", scale_range=(1e-4, 1e-1))


def gpt2_medium() -> Workload:
    return Workload("gpt2-medium-shaped", _gpt2_shapes(50257, 1024, 24, 1024), GRAD_F32, seed=3, steps=100,
                    grad_kind="student_t3", scale_range=(1e-4, 1e-1))


def bert_large() -> Workload:
    return Workload("bert-large-shaped-bf16", _encoder_shapes(30522, 512, 2, 24, 1024, 4096), GRAD_BF16,
                    seed=4, steps=100, grad_kind="normal", scale_range=(1e-5, 1e-1), zero_row_fraction=0.01)


def llama_7b() -> Workload:
    return Workload("llama-6.7b-shaped-bf16", _llama_shapes(32000, 32, 4096, 11008), GRAD_BF16, seed=5,
                    steps=20, grad_kind="normal", scale_range=(1e-5, 1e-2))


CONFIGS = [single_matrix, bert_base, gpt2_medium, bert_large, llama_7b]


def square_matrices(k: int, side: int = 4096) -> Workload:
    """k square bf16-gradient matrices: a list whose size is a chosen multiple of one matrix
    (used to see what staying inside the on-package cache is worth)."""
    return Workload(f"square{side}x{k}", [(side, side)] * k, GRAD_BF16, seed=6, steps=2, grad_kind="normal",
                    scale_range=(1e-4, 1e-2))


def by_name(name: str) -> Workload:
    if name.startswith("square"):  # "square4096x32": 32 matrices of 4096 x 4096
        side, k = name[len("square"):].split("x")
        return square_matrices(int(k), int(side))
    for f in CONFIGS:
        w = f()
        if w.name == name or f.__name__ == name:
            return w
    raise KeyError(name)


class Generator:
    """Draws theta_0 and the per-step gradients of a workload from its seed.

    Tensor i at step t is drawn from a torch generator seeded with a hash of
    (seed, i, t), so any single tensor/step can be re-drawn alone (that is how
    the parity tests sample tensors of the large workloads).  Per-tensor scales
    and zeroed-row masks are fixed across steps.
    """

    def __init__(self, w: Workload, device="cpu"):
        self.w = w
        self.device = torch.device(device)
        g = torch.Generator(device="cpu")
        g.manual_seed(1_000_003 * w.seed + 17)
        n = len(w.shapes)
        if w.scale_range is None:
            self.scales = [w.fixed_scale] * n
        else:
            lo, hi = (math.log(x) for x in w.scale_range)
            u = torch.rand(n, generator=g, dtype=torch.float64)
            self.scales = [math.exp(lo + (hi - lo) * float(x)) for x in u]
        self._row_masks = {}

    def _gen(self, i: int, t: int) -> torch.Generator:
        g = torch.Generator(device=self.device)
        g.manual_seed((self.w.seed * 1_000_003 + i) * 1_000_033 + t)
        return g

    def theta0(self, i: int) -> torch.Tensor:
        """theta_0 ~ N(0, 0.02^2), float32."""
        s = self.w.shapes[i]
        return torch.randn(s, generator=self._gen(i, 0), device=self.device, dtype=torch.float32) * 0.02

    def row_mask(self, i: int):
        """Rows of matrix i whose gradient is identically zero (fixed per tensor)."""
        s = self.w.shapes[i]
        if self.w.zero_row_fraction <= 0 or len(s) != 2:
            return None
        if i not in self._row_masks:
            g = torch.Generator(device="cpu")
            g.manual_seed(self.w.seed * 7_919 + i)
            k = max(1, int(round(self.w.zero_row_fraction * s[0])))
            self._row_masks[i] = torch.randperm(s[0], generator=g)[:k].to(self.device)
        return self._row_masks[i]

    def grad(self, i: int, t: int) -> torch.Tensor:
        """Gradient of tensor i at step t (1-based), in the workload's gradient dtype."""
        s = self.w.shapes[i]
        gen = self._gen(i, t)
        x = torch.randn(s, generator=gen, device=self.device, dtype=torch.float32)
        if self.w.grad_kind == "student_t3":
            # Student-t with 3 degrees of freedom: Z / sqrt(chi2_3 / 3)
            chi = torch.zeros(s, device=self.device, dtype=torch.float32)
            for _ in range(3):
                z = torch.randn(s, generator=gen, device=self.device, dtype=torch.float32)
                chi += z * z
            x = x / torch.sqrt(chi / 3.0)
        elif self.w.grad_kind != "normal":
            raise ValueError(self.w.grad_kind)
        x *= self.scales[i]
        mask = self.row_mask(i)
        if mask is not None:
            x[mask] = 0.0
        return x.to(self.w.torch_grad_dtype())
