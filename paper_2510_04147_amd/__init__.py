"""MI355X-native hot path of Self Speculative Decoding for masked-diffusion LLMs.

`synth` (seeded synthetic inputs) imports nothing else from here; the binding
to the HIP library is loaded on first use of `paper_2510_04147_amd.binding`.
"""
