"""MI355X-native training of fully connected networks: a thin Python binding
over the C-ABI library libdn (hand-written HIP kernels for gfx950).

``paper_2001_04206_amd.dn`` holds the binding; ``paper_2001_04206_amd.synth``
the seeded input generators; ``paper_2001_04206_amd.build`` compiles the library.
Nothing here computes: every step of a training pass runs in the library's kernels.
"""
