"""MI355X-native cache-reusing prefill and query-level match (PerCache, arXiv 2601.11553).

``paper_2601_11553_amd.binding`` is the thin ctypes layer over the C-ABI library built from
``csrc/``; ``paper_2601_11553_amd.workloads`` holds the seeded synthetic input recipes.
Nothing is loaded at package import time.
"""
