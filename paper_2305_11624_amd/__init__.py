"""MI355X-native ConvBN block in Tune mode (and the Eval-mode comparison path).

`synth` (input generators) imports without the GPU library; everything in
`binding` needs the compiled HIP library and fails loudly without it.
"""
__all__ = ["synth", "binding"]
