"""libmodet: the ModeT motion-decomposition operator (ModeTv2, Section 3.3.1) on MI355X.

`paper_2403_16526_amd.modet`  -- ctypes binding of the C ABI in include/modet.h (needs the built
                                 libmodet.so; imported lazily so the input generator works without it)
`paper_2403_16526_amd.synth`  -- seeded synthetic inputs (no operator arithmetic)
`paper_2403_16526_amd.build`  -- in-tree hipcc build
"""
