"""MI355X-native FP8 3D sliding-tile attention (forward hot path of arXiv 2506.04648).

`paper_2506_04648_amd.fps` is the thin ctypes binding over the C-ABI library built from `csrc/`;
`paper_2506_04648_amd.synth` is the seeded synthetic-input generator.  Importing the package does
not load the HIP library; the first call through `fps` does, and fails loudly if it is missing.
"""
