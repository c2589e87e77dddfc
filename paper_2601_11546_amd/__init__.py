"""MI355X-native layer step for relQuery serving batches (mixed prefill + decode).

`paper_2601_11546_amd.workloads` draws the seeded synthetic inputs;
`paper_2601_11546_amd.binding` is the thin ctypes layer over the C-ABI library
built from `csrc/`.  Importing the package loads neither.
"""
__all__ = ["workloads", "binding"]
