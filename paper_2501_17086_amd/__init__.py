"""Highway-BP backward pass for one MI355X (gfx950).

`binding` holds the ctypes marshalling over the C-ABI library (include/hbp.h);
`synth` the seeded synthetic inputs; `build` compiles the HIP sources in-tree.
Importing the package loads nothing: the library is opened on first use of
`binding`, and that fails loudly when it has not been built.
"""
