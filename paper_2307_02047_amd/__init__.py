"""MI355X-native CAME optimizer step: a C-ABI HIP library plus this thin binding.

The arithmetic of the step runs entirely in the gfx950 kernels of
libcame_hip.so; Python only marshals arguments.  PyTorch is used for device
memory and streams.
"""
from .binding import (CameHyper, CameStep, GRAD_BF16, GRAD_F32, ALGO_CAME, ALGO_ADAFACTOR,  # noqa: F401
                      MOMENTUM_F32, MOMENTUM_BF16, VECTOR_ALGORITHM2, VECTOR_MOMENTUM_ONLY, CameError, algorithmic_bytes,
                      RESIDENT_AUTO, RESIDENT_OFF, RESIDENT_ON, ETIMEOUT,
                      load_library, plan_query, plan_traffic, state_size, step_noalloc)


def __getattr__(name):
    # torch is only needed for the optimizer front end; the C-ABI binding imports without it
    if name == "CAME":
        from .optim import CAME
        return CAME
    raise AttributeError(name)
