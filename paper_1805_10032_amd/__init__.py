"""MI355X-native Zeno aggregation step (arXiv 1805.10032): a C-ABI HIP library
for gfx950 plus a thin ctypes binding.  `workloads` makes seeded synthetic
inputs; `binding` marshals torch device pointers into the C calls."""

__all__ = ["binding", "workloads", "build"]
