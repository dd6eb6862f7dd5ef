"""MI355X-native verify pass for speculative decoding of visual autoregressive models.

`synth` (seeded input generators) imports on any machine; `binding` needs the built HIP library and
fails loudly when it is missing."""
__all__ = ["synth", "binding"]
