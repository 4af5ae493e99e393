"""MI355X-native scoring of claimed sampled tokens against verifier logits.

The product is ``libdifr.so`` (hand-written HIP kernels for gfx950 behind the C ABI of
``include/difr.h``).  This package is only its Python binding: one function per entry
point, with the entry point's name less the ``difr_`` prefix (``score_both``,
``gumbel_score``, ``ipt_score``, ``seq_reduce``, ``classify``, ``lmhead_score``, ...).
Each marshals torch device tensors into the C call and returns torch tensors; every step
of the computation runs in the library's kernels.  There is no CPU fallback: if the
library is missing, ``load_library()`` - and with it every call - fails loudly.
"""
from .binding import (  # noqa: F401
    admissible_count,
    DifrError,
    FLAG_INVALID_CLAIM,
    FLAG_MATCH,
    FLAG_NONFINITE,
    FLAG_SLOW_PATH,
    classify,
    debug_gumbel_map,
    debug_noise,
    gumbel_likelihood,
    gumbel_score,
    ipt_score,
    ipt_score_filtered,
    lib_path,
    lmhead_outputs,
    lmhead_score,
    lmhead_score_static,
    lmhead_workspace_bytes,
    load_library,
    philox4x32_10,
    score_both,
    score_both_admissible,
    score_both_filtered,
    score_both_peaked,
    seq_reduce,
    version,
)
