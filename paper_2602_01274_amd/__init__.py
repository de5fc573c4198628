"""MI355X-native hot path of Pacer adaptive speculative decoding.

`synth` (seeded synthetic inputs) imports without a GPU; `binding` loads the HIP
library and fails loudly when it has not been built.
"""
