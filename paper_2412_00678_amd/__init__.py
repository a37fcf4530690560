"""MI355X-native 2D selective scan (the operator of 2DMamba, Sec. 3.3-3.4).

Sub-modules:
  workloads -- seeded synthetic inputs (no scan arithmetic; importable without a GPU)
  scan2d    -- thin ctypes binding of the C-ABI library built from csrc/ (HIP, gfx950)
  build     -- compiles csrc/ with hipcc

Importing the package itself loads nothing; `scan2d` loads the shared library on import and
raises if it has not been built.
"""
__all__ = ["workloads", "scan2d", "build"]
