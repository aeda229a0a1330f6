"""CPU oracle for the SpecKV verify-and-select stage.

TEST INFRASTRUCTURE, not product code.  Only ``tests/``, ``__graft_entry__.smoke()``
and the ``cpu_baseline`` leg of ``bench.py`` may import this package.  It never
imports the HIP package and shares no code with it.

``oracle.ref`` wraps ``libspeckv_oracle.so`` (plain C, float64; see
``speckv_oracle.c`` for what is computed and which passage of the paper
defines each piece).
"""
from .ref import (  # noqa: F401
    DTYPE_CODES,
    philox4x32_10,
    load_logits,
    row_softmax,
    signals,
    verify,
    verify_greedy,
    sample_draft,
    select_gamma,
    residual,
    inverse_cdf,
    set_threads,
    FLAG_NONFINITE,
    FLAG_BAD_TOKEN,
    FLAG_FALLBACK,
    RESID_FLOOR,
)
