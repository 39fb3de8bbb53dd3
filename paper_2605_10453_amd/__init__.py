"""MI355X-native low-rank drafter LM-head with fused top-k / log-probabilities.

`binding` wraps the C ABI of libslimspec.so (hand-written HIP for gfx950);
`synth` draws the seeded synthetic inputs; `build` compiles the library.
Importing the package does not import torch; `binding` does.
"""
__all__ = ["binding", "synth", "build"]
