"""CPU oracle (test infrastructure only) for RainFusion's ARM + sparse attention.

Thin ctypes/numpy front for ``rf_oracle.c``: fp64 arithmetic, plain loops,
written from the paper's definitions (Sec. 3.1-3.3, Eq. 1-6, Alg. 1).  Only
``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package; the GPU library never does.
"""
from .api import (  # noqa: F401
    SPATIAL, TEMPORAL, TEXTURAL, DENSE, SAMPLE_FIRST_FRAME, SAMPLE_EQUAL_INTERVAL,
    Layout, Params, build, keep, keep_matrix, radius, num_tokens, attention_rows,
    attention, attention_blockskip, arm_recall, arm_classify, arm_classify_plus, decide, kept_fraction,
    sample_tokens, num_threads,
)
