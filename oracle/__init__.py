"""CPU oracle (test infrastructure only).

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may
import this package.  It never imports the HIP package and shares no code with it.
"""
from .ref import (  # noqa: F401
    build_oracle,
    double_to_half,
    half_to_double,
    ref_compress,
    ref_compress_bound,
    ref_compress_bound_v2,
    ref_compress_v2,
    ref_decompress_v2,
    ref_inspect_v2,
    ref_decompress,
    ref_inspect,
    ref_spmm_f64,
    ref_threads,
)
from .roofline import ci_dense, ci_sparse_load, roof_fraction  # noqa: F401
