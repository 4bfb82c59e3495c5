"""CPU oracle (test infrastructure only).

Holds the plain fp64 direct convolution and max-pool written out from the
paper's definition (``conv_oracle.c``) and a ctypes wrapper around it.  Only
``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package; the product package never does, and this
package never imports the product package.
"""
from .conv_oracle import (  # noqa: F401
    build,
    conv_fwd,
    conv_fwd_points,
    conv_out_shape,
    maxpool_fwd,
    max_normalised_error,
    set_threads,
    threads,
)
