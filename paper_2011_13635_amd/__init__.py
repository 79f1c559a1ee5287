"""MSLT stage step for AMD MI355X: hand-written HIP kernels behind a C ABI (libmslt.so).

`binding` holds the thin ctypes layer (argument marshalling only); `synth` the seeded
synthetic inputs; `build` compiles the library in-tree.  Nothing here falls back to a CPU
or PyTorch implementation: without the built library and a GPU the binding raises.
"""
__all__ = ["binding", "synth", "build"]
