"""w2mm: 2-bit-weight mixed-precision matmul for MI355X (gfx950).

`binding` wraps the C ABI of libw2mm.so (HIP kernels); `synth` draws the seeded
synthetic inputs; `build` compiles the library in-tree.  Importing the package
does not load the library; importing `binding` does, and fails if it is absent.
"""
__all__ = ["binding", "synth", "build"]
