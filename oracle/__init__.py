"""CPU oracle for the forward convolution layer -- TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and ``bench.py``'s cpu_baseline leg
may import this package.  It shares no code with the HIP library and never
imports it.  The arithmetic lives in ``conv_oracle.c`` (plain C, double
accumulation); this module only builds that file with gcc and marshals numpy
arrays into it.
"""
from .conv_oracle import (  # noqa: F401
    build,
    conv_fwd,
    conv_fwd_f16,
    conv_out_dims,
    maxpool_fwd,
    num_threads,
    sgemm,
)
