"""MI355X (gfx950) library for the low-precision SGD update with Kahan
summation over dynamic fixed-point parameters, and its Python binding.

    from paper_1810_05486_amd import binding as lpk

The package does no arithmetic of the method in Python: `binding` marshals
arguments into the C ABI of liblpk.so (include/lpk.h), `workloads` only draws
seeded synthetic inputs.  Importing the package does not load the library; the
first call does, and raises if it has not been built
(`python -m paper_1810_05486_amd.build`).
"""
__all__ = ["binding", "workloads", "build"]
