"""MI355X-native rollout generation path behind the `areal_*` C-ABI.

`synth` (input generators) is importable anywhere; `binding` loads the HIP
shared library and fails loudly if it has not been built.
"""
__all__ = ["synth", "binding"]
