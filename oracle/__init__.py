"""CPU oracle for the WSVD decode hot path (test infrastructure, not product code).

Everything under ``oracle/`` is a plain, slow, fp64 restatement of what the paper
defines: per-head latent caches C_Kh = X A_Kh, C_Vh = X A_Vh, keys and values
recovered as K_h = C_Kh B_Kh, V_h = C_Vh B_Vh (Section 3.1, "Fine-grained Per-Head
SVD Operation"), followed by textbook softmax attention, which is what the fused
kernel of Section 3.4 computes "without any loss of accuracy".

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It shares no code with the HIP library and
never imports it.
"""
from .wsvd_oracle import *  # noqa: F401,F403
from .wsvd_oracle import __all__  # noqa: F401
