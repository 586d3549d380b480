"""CMPQ (arXiv 2410.13056) quantization path for AMD MI355X: HIP kernels behind a C ABI
(include/cmpq.h), a ctypes binding (`binding`), the host driver (`pipeline`) and the
seeded input generators (`synth`).  Submodules are imported on demand so that the
generators can be used where the library has not been built."""
__all__ = ["binding", "pipeline", "synth", "build"]
