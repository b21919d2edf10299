"""MI355X-native DiffuSpec speculative round: HIP kernels behind a C-ABI library.

Importing the package is cheap and loads nothing native; `paper_2510_02358_amd.binding`
loads `libdiffuspec.so` on first use and raises if it has not been built.
"""
__all__ = ["synth", "binding"]
