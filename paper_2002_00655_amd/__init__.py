"""Parameter server with dynamic parameter allocation driving blocked
latent-factor SGD, for one AMD MI355X (gfx950).

``paper_2002_00655_amd.ps``        thin binding of the C-ABI library (HIP kernels)
``paper_2002_00655_amd.workloads`` seeded synthetic inputs (no method arithmetic)
"""
__all__ = ["workloads"]
