"""MI355X-native GRAWA distributed update (gradient-norm weighted averaging of
data-parallel workers): a C-ABI HIP library plus this thin ctypes binding.

Importing the package does not load the GPU library; the first call into
``paper_2403_04206_amd.grawa`` does, and raises if it has not been built.
"""
__all__ = ["grawa", "workloads", "buildlib"]
