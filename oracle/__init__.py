"""Float64 CPU oracle for the tensor comprehensions (test infrastructure only).

Nothing in the product package imports this; only tests/, the smoke check and
the benchmark's cpu_baseline leg do.
"""
from .tc_oracle import (  # noqa: F401
    build,
    tbmm,
    mlp_fcrelu,
    group_conv,
    group_conv_infer,
    kron,
    sconv2d,
    sconv2d_infer,
    lut,
    set_threads,
    get_threads,
    max_threads,
)
