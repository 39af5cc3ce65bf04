"""MI355X-native whole-model decode kernel behind a C ABI (libflashformer.so).

`synth` (seeded input generators) imports without the native library; `binding` loads it and
fails loudly if it has not been built.
"""
__all__ = ["synth", "binding"]
