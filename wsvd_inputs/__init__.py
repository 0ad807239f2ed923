"""Seeded synthetic inputs for the WSVD decode path.

This module only draws numbers.  It holds none of the method's arithmetic: no latent
projection of a token through the append path, no quantiser, no attention.  Both the CPU
oracle's tests and the HIP library's tests / benchmark read their inputs from here, so the
two sides see identical bytes.  All draws come from numpy's counter-based Philox generator
keyed by (seed, stream id), so any tensor can be regenerated on its own.

Shapes and value laws follow the five workloads of this build (VLM-shaped: an image-token
prefix of 576 rows, 7B-class head geometry, 1 % of hidden channels scaled x20 as activation
outliers, cf. the channel-wise outliers discussed in Section 3.3 of the paper).
"""
from .synth import *  # noqa: F401,F403
from .synth import __all__  # noqa: F401
