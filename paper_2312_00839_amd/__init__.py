"""PipeOptim fused optimizer step + weight prediction for MI355X (gfx950).

``binding`` wraps the C-ABI library built from ``csrc/``; ``workloads`` holds
the seeded synthetic stage inputs.  Importing the package loads nothing; the
binding raises if the HIP library has not been built.
"""
