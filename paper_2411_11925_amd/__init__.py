"""MI355X-native hot path of continuous speculative decoding (arxiv 2411.11925).

`synth` (input generators) imports without a GPU; `binding` loads the HIP
library and raises if it has not been built.
"""
__all__ = ["synth", "binding"]
