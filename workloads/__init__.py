"""Seeded synthetic decode streams (q_t, k_t, v_t per layer and sequence).

This package only produces inputs.  It holds none of the method's arithmetic
(no attention, no softmax, no eviction) and imports neither the CPU oracle nor
the HIP library; both consume what it generates.
"""
from .streams import CONFIGS, StreamSpec, Stream, spec_for  # noqa: F401
