"""Transit-parallel graph sampling for one AMD MI355X (gfx950).

`binding` mirrors the C ABI of include/nd.h (it needs torch and the built
libnd.so); `inputs` holds the seeded synthetic workloads; `build` compiles
the HIP library in-tree.  Importing the package loads none of them.
"""
__all__ = ["binding", "inputs", "build"]
