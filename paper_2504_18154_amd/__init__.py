"""MI355X-native paged-attention hot path of an EcoServe instance (arXiv 2504.18154).

Sub-modules:
  binding    -- thin ctypes layer over the C ABI in include/ecoserve.h (loads the HIP library)
  workloads  -- seeded synthetic input generators (no method arithmetic)
  accounting -- algorithmic byte / FLOP counts used for roofline reporting
  build      -- compiles csrc/*.hip for gfx950 into libecoserve.so

Nothing is imported eagerly: `import paper_2504_18154_amd.workloads` must work without a
built library, while `paper_2504_18154_amd.binding` fails loudly if the library is missing.
"""
__all__ = ["binding", "workloads", "accounting", "build"]
