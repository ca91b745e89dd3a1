"""Nothing outside the caller's buffers is written.

Every buffer the library is handed -- parameters, gradients, bfloat16 parameter copies, the
state blob and the scratch blob -- is carved out of one pattern-filled arena with at least
4 KiB of untouched bytes on either side.  After a few steps on ragged, unaligned, single-row,
single-column and long-vector shapes, with both gradient types, both momentum types and the
bfloat16-copy entry point, every margin byte must still hold the pattern, the gradients must
be bit-identical to what was handed over, and the bytes of the state blob that belong to no
array (the padding between them) must still be the zeros came_init_state wrote."""
import numpy as np
import pytest
import torch

import paper_2307_02047_amd as P
from paper_2307_02047_amd import workloads as W
from test_gpu_parity import ODD_SHAPES

pytestmark = pytest.mark.gpu

PATTERN = 0xA5
MARGIN = 4096


class Arena:
    """One uint8 allocation filled with PATTERN; carve() hands out 256-byte aligned slices
    separated by at least MARGIN pattern bytes."""

    def __init__(self, nbytes, device="cuda:0"):
        self.buf = torch.full((nbytes,), PATTERN, dtype=torch.uint8, device=device)
        base = self.buf.data_ptr()
        self.pos = (-base) % 256 + MARGIN
        self.used = []  # (offset, bytes)

    def carve(self, nbytes):
        off = self.pos
        assert (self.buf.data_ptr() + off) % 256 == 0
        self.used.append((off, nbytes))
        self.pos = (off + nbytes + MARGIN + 255) // 256 * 256
        assert self.pos <= self.buf.numel(), "arena too small"
        return self.buf[off:off + nbytes]

    def margins_intact(self):
        mask = torch.ones(self.buf.numel(), dtype=torch.bool, device=self.buf.device)
        for off, nbytes in self.used:
            mask[off:off + nbytes] = False
        return bool((self.buf[mask] == PATTERN).all())


def _typed(arena, shape, dtype):
    n = int(np.prod(shape))
    return arena.carve(n * torch.empty((), dtype=dtype).element_size()).view(dtype).view(shape)


@pytest.mark.parametrize("momentum", [P.MOMENTUM_F32, P.MOMENTUM_BF16], ids=["m-f32", "m-bf16"])
@pytest.mark.parametrize("dtype", [W.GRAD_F32, W.GRAD_BF16], ids=["g-f32", "g-bf16"])
@pytest.mark.parametrize("tile_rows", [8, 0, -1], ids=["tr8", "tr-auto", "on-chip"])
def test_margins_stay_untouched(dtype, momentum, tile_rows):
    # "on-chip": the matrices that qualify (rows 16-byte aligned) take the on-chip path
    resident = P.RESIDENT_ON if tile_rows < 0 else P.RESIDENT_OFF
    tile_rows = max(tile_rows, 0)
    shapes = ODD_SHAPES + [(300, 1032), (64, 2048), (1,), (7,), (255,), (257,), (5000,), (16385,), (50257,)]
    n = len(shapes)
    w = W.Workload("canary", shapes, dtype, seed=123, steps=3, grad_kind="normal", scale_range=(1e-3, 1e-1),
                   zero_row_fraction=0.1)
    gen = W.Generator(w, device="cuda:0")
    tile_rows3 = 12 if tile_rows == 8 else 0  # the update sweep's own tiling: a ragged height once, the default otherwise
    state_bytes, scratch_bytes = P.state_size(shapes, [dtype] * n, tile_rows=tile_rows, tile_rows3=tile_rows3,
                                              momentum_dtype=momentum, resident=resident)
    total = sum(int(np.prod(s)) for s in shapes)
    arena = Arena(total * (4 + 4 + 2) + state_bytes + scratch_bytes + (3 * n + 4) * (MARGIN + 512) + (1 << 16))
    gdt = torch.bfloat16 if dtype == W.GRAD_BF16 else torch.float32
    theta = [_typed(arena, s, torch.float32) for s in shapes]
    grads = [_typed(arena, s, gdt) for s in shapes]
    copies = [_typed(arena, s, torch.bfloat16) for s in shapes]
    state, scratch = arena.carve(state_bytes), arena.carve(scratch_bytes)
    for i in range(n):
        theta[i].copy_(gen.theta0(i))
    opt = P.CameStep(shapes, [dtype] * n, tile_rows=tile_rows, tile_rows3=tile_rows3, momentum_dtype=momentum,
                     resident=resident, blobs=(state, scratch))
    try:
        assert opt.state.data_ptr() == state.data_ptr()
        for t in range(1, 4):
            fresh = [gen.grad(i, t) for i in range(n)]
            for i in range(n):
                grads[i].copy_(fresh[i])
            # plain step, then the entry point that also writes bfloat16 copies (every other tensor)
            opt.step(theta, grads, P.CameHyper(weight_decay=0.01), 1e-3, t,
                     bf16_copies=None if t == 1 else [copies[i] if i % 2 == 0 else None for i in range(n)])
            torch.cuda.synchronize()
            for i in range(n):
                assert torch.equal(grads[i].view(torch.int16 if gdt == torch.bfloat16 else torch.int32),
                                   fresh[i].view(torch.int16 if gdt == torch.bfloat16 else torch.int32)), f"gradient {i} was written"
            assert arena.margins_intact(), f"step {t}: bytes outside the buffers were written"
        for i in range(n):
            assert torch.isfinite(theta[i]).all()
            if i % 2 == 1:   # copies that were never asked for still hold the pattern
                assert bool((copies[i].view(torch.uint8) == PATTERN).all())
            else:
                assert torch.equal(copies[i].view(torch.int16), theta[i].to(torch.bfloat16).view(torch.int16))
        # inside the state blob: whatever belongs to no array is still zero
        live = torch.zeros(state_bytes, dtype=torch.bool, device="cuda:0")
        base = state.data_ptr()
        for i in range(n):
            for k, a in opt.state_view(i).items():
                if a is not None:
                    off = a.data_ptr() - base
                    live[off:off + a.numel() * a.element_size()] = True
        assert not bool(state[~live].any()), "padding inside the state blob was written"
    finally:
        opt.close()


def test_placement_probe_keeps_to_its_buffers():
    """The placement probe reads and rewrites theta and M only."""
    shapes = [(300, 1032), (64, 2048), (33, 512), (700,)]
    w = W.Workload("canary-probe", shapes, W.GRAD_BF16, seed=5, steps=1, grad_kind="normal", scale_range=(1e-3, 1e-1))
    gen = W.Generator(w, device="cuda:0")
    state_bytes, scratch_bytes = P.state_size(shapes, [1] * 4, tile_rows=16)
    arena = Arena(sum(int(np.prod(s)) for s in shapes) * 6 + state_bytes + scratch_bytes + 16 * (MARGIN + 512))
    theta = [_typed(arena, s, torch.float32) for s in shapes]
    grads = [_typed(arena, s, torch.bfloat16) for s in shapes]
    for i in range(4):
        theta[i].copy_(gen.theta0(i))
        grads[i].copy_(gen.grad(i, 1))
    opt = P.CameStep(shapes, [1] * 4, tile_rows=16, blobs=(arena.carve(state_bytes), arena.carve(scratch_bytes)))
    try:
        opt.step(theta, grads, P.CameHyper(), 1e-3, 1)
        torch.cuda.synchronize()
        before = [t.clone() for t in theta]
        assert opt.probe_placement(theta, repeats=2) > 0 and opt.probe_placement(theta, grads, repeats=2) > 0
        assert arena.margins_intact()
        assert all(torch.equal(a, b) for a, b in zip(before, theta))
    finally:
        opt.close()
