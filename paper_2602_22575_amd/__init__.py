"""S2O causal prefill attention for AMD MI355X (gfx950): hand-written HIP kernels behind a
C ABI (include/s2o.h, libs2o.so) plus this thin ctypes binding.  Importing the package does
not load the library; the first call does, and fails loudly if it has not been built."""
from .binding import (Plan, S2OError, S2OParams, load_library, make_params, s2o_attention,  # noqa: F401
                      s2o_attention_local, s2o_attention_prefix, s2o_attention_sizes, s2o_plan,
                      s2o_plan_sizes)
