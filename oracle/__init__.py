"""CPU oracle for the active-vocabulary LM head: test infrastructure, not product.

Only `tests/`, `__graft_entry__.smoke()` and the `cpu_baseline` leg of `bench.py`
may import this package.  It never imports the GPU package and shares no code
with it.  See `evospec_oracle.c` for what is computed and which passages of the
paper it follows (Eq. 1; Eq. 3; Algorithm 1, draft phase restricted to V_t), and
`arc_oracle.py` for the dynamic-buffer manager (appendix, ARC maintenance and safeguards).
"""
from .oracle import (  # noqa: F401
    build,
    active_gather,
    logits,
    logz,
    topk,
    active_lmhead_topk,
    active_lmhead_topk_segmented,
    num_threads,
    set_num_threads,
)
from .arc_oracle import ArcOracle  # noqa: F401,E402
from .candidates_oracle import exact_mips, form_candidates  # noqa: F401,E402
from .kl_gate_oracle import kl_gate  # noqa: F401,E402
