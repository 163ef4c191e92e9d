"""Float64 CPU oracle for the local Newton-CG x-update of Newton-ADMM.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path (the HIP library and
its Python binding) imports, links or executes anything in this package; only
the test-suite, the smoke check and the benchmark's CPU-baseline leg do.  The
oracle shares no code, tables or constants with the GPU path.
"""
from .nadmm_oracle import (  # noqa: F401
    Problem,
    logits,
    lse_parts,
    probabilities,
    row_losses,
    penalty,
    loss,
    grad,
    loss_grad,
    hessvec,
    cg,
    line_search,
    local_newton,
)
