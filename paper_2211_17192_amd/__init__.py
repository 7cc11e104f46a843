"""MI355X-native hot path of speculative decoding (Algorithm 1 of arXiv 2211.17192).

The compute lives in the HIP library built from csrc/ and reached through the
C ABI declared in include/sd.h; `binding` is its thin ctypes wrapper and
`synth` the seeded synthetic-input generators.  Submodules are imported on
demand so that `synth` can be used without the GPU library.
"""
__all__ = ["binding", "synth", "build"]
