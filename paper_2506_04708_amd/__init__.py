"""STAND speculation step for AMD MI355X: HIP kernels behind a C ABI (libstand.so).

`synth` (input generators) imports without the library; `binding` needs it built.
"""
