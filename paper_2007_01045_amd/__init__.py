"""One pipeline stage of synchronous pipelined training (early-backward / 1F1B
micro-batch order, K resident activation slots, fp32 gradient accumulation) as
hand-written gfx950 HIP kernels behind a C-ABI library.

Importing the package loads nothing native: `paper_2007_01045_amd.binding`
loads the shared library on first use and raises if it has not been built.
`paper_2007_01045_amd.inputs` is the seeded synthetic-input generator and holds
none of the method's arithmetic.
"""
