"""MI355X-native decode / compress / masked-prefill path of Breadcrumbs Reasoning.

`paper_2510_13797_amd.bc` is the thin ctypes binding over the C-ABI library
(libbc.so, built from csrc/ by __graft_entry__.build()); it is imported lazily
so that `paper_2510_13797_amd.workloads` (pure NumPy input generators) can be
used without the library.
"""
