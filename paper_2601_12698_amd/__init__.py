"""MI355X-native fused residual-add + RMSNorm with a two-stage (template +
search) tuner.  The compute runs in the HIP library ``libaddrms.so``; this
package is its argument-marshalling binding plus the seeded workload
generators.  Importing the package does not load the library; the first call
into :mod:`paper_2601_12698_amd.binding` does, and fails loudly if it is missing.
"""
__all__ = ["binding", "workloads"]
