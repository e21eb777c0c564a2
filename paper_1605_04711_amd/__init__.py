"""MI355X-native hot path of Ternary Weight Networks (arXiv 1605.04711).

The product is the C-ABI library built from `csrc/` (HIP, gfx950); `api` is a
thin ctypes binding with the same entry-point names.  `workloads` holds the
seeded synthetic inputs and layer tables and needs no GPU library.
"""

__all__ = ["api", "workloads", "build"]
