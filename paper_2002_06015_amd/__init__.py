"""MI355X-native K-FAC hot path (SP-NGD, arXiv 2002.06015).

``paper_2002_06015_amd.kfac`` is the Python binding of the C-ABI HIP library
(argument marshalling only); ``paper_2002_06015_amd.workloads`` holds layer
shapes and seeded synthetic inputs.  Importing the package loads nothing.
"""
__all__ = ["kfac", "workloads"]
