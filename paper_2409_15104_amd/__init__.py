"""MI355X-native blockwise causal prefill attention (one GPU's share of a ring prefill).

`binding` wraps the C-ABI library built from `csrc/` (see include/pec_attn.h);
`synth` holds the seeded input generators.  Importing this package does not load
the HIP library; the first call into `binding` does, and raises if it is missing.
"""
from . import synth  # noqa: F401

__all__ = ["synth", "binding", "build"]
