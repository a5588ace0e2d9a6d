"""MI355X (gfx950) implementation of the per-decode-step KV-cache management pass.

``paper_2604_26968_amd.kvm`` is the ctypes binding over the C-ABI library
built from ``csrc/``; ``paper_2604_26968_amd.synth`` makes seeded synthetic
inputs.  Importing the package itself loads nothing.
"""
