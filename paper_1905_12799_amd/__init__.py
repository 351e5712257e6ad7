"""MI355X-native adaptive-sampling hot path: tree scoring, k-means sweep, knee pick, snap to valid.

`binding` wraps the C ABI of include/rls.h (HIP kernels in csrc/); `synth` makes seeded inputs;
`build` compiles the library.  Importing the package loads nothing: the library is opened on first use.
"""
__all__ = ["binding", "synth", "build"]
