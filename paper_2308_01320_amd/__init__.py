"""MI355X-native actor generation engine (prefill + KV-cached decode of an
OPT-style decoder), the experience-generation phase of RLHF step 3.

`synth` (seeded inputs) imports nothing heavy; `binding` loads the HIP
library on first use and fails loudly when it has not been built.
"""
from . import synth  # noqa: F401

__all__ = ["synth"]
