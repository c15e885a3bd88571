"""MI355X-native decode path of LineAR (arxiv 2512.04857): line-structured,
progressively evicted visual KV cache with fused inter-line scoring.

`paper_2512_04857_amd.binding` loads the HIP library (and fails loudly if it has
not been built); `paper_2512_04857_amd.synth` only makes seeded inputs and can
be imported without it.
"""
