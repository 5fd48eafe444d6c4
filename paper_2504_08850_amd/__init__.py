"""MI355X-native SpecEE speculative early-exit predictor (hot path only).

`paper_2504_08850_amd.specee` is the Python binding of the C-ABI library
(`include/specee.h`); `paper_2504_08850_amd.synth` draws seeded inputs.
Nothing is loaded at import time: the HIP library is opened on the first call
of a binding function and a missing library is a hard error.
"""
__all__ = ["synth", "specee"]
