"""fp64 CPU oracle of the multi-adapter LoRA linear layer (test infrastructure).

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It imports nothing from the GPU package.
"""
from .oracle import (  # noqa: F401
    Oracle,
    FusedProjections,
    build_oracle,
    token_task,
    forward,
    backward_dx,
    backward_grads,
    adam_step,
)
