"""canz: per-rank Muon optimizer step for MI355X (gfx950) behind a C ABI.

``paper_2602_06079_amd.binding`` wraps the shared library built from ``csrc/``;
``paper_2602_06079_amd.workloads`` holds the seeded synthetic inputs.  Importing
the package loads nothing native; the binding raises if the library is missing.
"""
__version__ = "0.4.0"
