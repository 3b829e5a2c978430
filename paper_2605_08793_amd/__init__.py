"""MI355X-native streaming kernels for the entropic-OT dual (objective, gradient,
threshold-sparsified plan, log-domain Sinkhorn half-steps).

Importing the package loads nothing native; `paper_2605_08793_amd.binding`
opens the HIP library on first use and raises if it is not built.
"""
__all__ = ["binding", "workloads", "build"]
