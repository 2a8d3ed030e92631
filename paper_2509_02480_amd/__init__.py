"""MI355X-native update-phase hot path of MLP-Offload (arXiv 2509.02480).

``paper_2509_02480_amd.binding`` wraps the C-ABI library ``libmlpo.so`` (hand-written HIP kernels for gfx950);
``paper_2509_02480_amd.workloads`` generates the seeded synthetic inputs.  Importing the package loads no native
code; the first call into ``binding`` does, and raises if the library has not been built.
"""
__all__ = ["binding", "workloads"]
