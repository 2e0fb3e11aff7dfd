"""CompilerKV prefill-end retention step for AMD MI355X (gfx950): HIP kernels behind a C ABI.

``paper_2602_08686_amd.binding`` wraps the shared library (``csrc/`` -> ``libckv.so``) with the same
four calls the C header declares; ``paper_2602_08686_amd.workloads`` draws the seeded synthetic
inputs. Importing the package loads nothing native; the binding raises if the library is missing.
"""
__all__ = ["binding", "workloads"]
