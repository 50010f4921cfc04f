"""librollattn: paged-KV decode and observation-append attention for gfx950.

The compute lives in the C-ABI shared library built from `csrc/`; `binding` wraps
its entry points for torch tensors (argument marshalling only) and `workloads`
draws the synthetic batches.  Importing this package does not load the library;
`binding.lib()` does, and raises if it has not been built.
"""
__all__ = ["binding", "workloads"]
