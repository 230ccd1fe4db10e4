"""libwhalesplit: the column-split fully-connected + softmax head on MI355X (gfx950).

`paper_2011_09208_amd.binding` is the ctypes binding over the C-ABI library;
`paper_2011_09208_amd.inputs` the seeded synthetic inputs.  Nothing is imported
eagerly so that the input generators can be used without the built library.
"""
__all__ = ["binding", "inputs", "buildlib"]
