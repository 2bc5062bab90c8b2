"""libmmvseg: segmented scan, segmented sum and COO SpMV on MI355X (gfx950).

The compute path is the C-ABI library ``libmmvseg.so`` built from
``csrc/`` (hand-written HIP kernels); ``binding`` marshals torch device
tensors into its calls.  ``workloads`` draws the seeded synthetic inputs.
Importing the package does not load the library; the first call does, and it
raises if the library has not been built.
"""

__all__ = ["binding", "workloads", "build"]
