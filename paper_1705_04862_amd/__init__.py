"""PAAC hot path (batched action selection + actor-critic train step) for MI355X.

`paper_1705_04862_amd.paac` is the ctypes binding over the C-ABI library built from
`csrc/`; `paper_1705_04862_amd.inputs` holds the seeded synthetic input generators.
Nothing is imported eagerly so that `inputs` can be used without the HIP library.
"""
