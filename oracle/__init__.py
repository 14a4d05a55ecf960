"""fp64 CPU oracle for the TOVA bounded-cache decode step.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path (the HIP library and
its Python binding) imports, calls or links anything in this package; only the
tests, the smoke check and the CPU-baseline leg of the benchmark do.  The
oracle shares no code with the HIP path and never reads its results.

What is pinned and what is not:
  * attend / select / update (the per-step arithmetic and the victim rule) are
    pinned by the CPU tests against textbook full attention when the cache
    never fills, brute-force recomputation from the raw stream on tiny inputs,
    the ordered-list formulation of the paper's appendix algorithm, the mask
    formulation over a whole prompt (which also defines what a multi-token call
    must produce), closed
    forms (capacity 1, identical keys, a dominating key) and invariants.
  * the step with re-assigned positions (tova_positions: compressed gaps between retained
    tokens, rotary embedding at those positions) is pinned by closed forms of the gap rule,
    complex multiplication for the rotary embedding, ordinary rotary attention when nothing
    is dropped, a two-dimensional case with closed-form logits, independence of the stream's
    origin, and brute force from the raw stream on tiny inputs.
  * the absolute victim sequences on the large synthetic configurations are
    "parity unpinned" by the paper itself (it prints no worked numeric
    example); they are trusted only because the routine that produces them
    passes the pins above.
"""
from .tova_oracle import TovaOracle, TovaHeadOracle, run_stream  # noqa: F401
from .tova_literal import OrderedTova  # noqa: F401
from .tova_masked import tova_masked_prompt  # noqa: F401
from .tova_positions import TovaPositionsOracle, compress_gap, compressed_positions, rope  # noqa: F401
