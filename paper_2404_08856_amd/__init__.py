"""MI355X-native hot path of speculative decoding for a LLaVA-style MLLM.

`spd` is the Python binding of the C-ABI library (HIP kernels for gfx950);
`synth` generates the seeded synthetic inputs.  Importing the package does not
load the library; `spd` does, and fails loudly if it has not been built.
"""
