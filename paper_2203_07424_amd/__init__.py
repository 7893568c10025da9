"""MI355X-native forward pass of DLRM-class recommendation models.

`synth` draws seeded inputs and can be imported anywhere; `binding` loads the
HIP library and raises if it has not been built.  Nothing is imported eagerly
so that input generation never depends on the device code.
"""
__all__ = ["synth", "binding", "build"]
