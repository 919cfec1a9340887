"""SharpV two-stage visual-token / KV-cache pruning on MI355X (gfx950).

`paper_2511_08003_amd.sharpv` is the Python binding of the C-ABI library (HIP kernels);
`paper_2511_08003_amd.workloads` draws the seeded synthetic inputs.  Importing the package
loads nothing: the shared library is opened on first use of the binding.
"""
__all__ = ["sharpv", "workloads"]
